/*
 * keyformer.h -- C ABI of the MI355X (gfx950) Keyformer decode hot path.
 *
 * Keyformer (arXiv 2403.09054) keeps, per layer and per head, a KV cache of k
 * tokens: the w most recent ones plus the k-w "key tokens" with the largest
 * accumulated score f.  The score of a step is a softmax of the attention
 * logits perturbed by a logit adjustment zeta and divided by a temperature tau
 * that grows over the generation (Eq. 4, Eq. 11, Eq. 12, Algorithm 1).
 *
 * Conventions
 *  - A "unit" is one (layer, batch, head) triple: an independent cache with its
 *    own scores.  Unit index u = (l*B + b)*H + h.  Every call handles all units.
 *  - Every pointer marked DEVICE is GPU memory owned by the caller; the library
 *    never allocates, frees or keeps it.  Pointers marked HOST are read during
 *    the call only.
 *  - The calls that take a stream only enqueue kernels on `stream` (a hipStream_t passed
 *    as void*, NULL = the default stream) and return; they do not synchronise.
 *  - Arguments are validated on the host before anything is launched; a call
 *    that returns an error has launched nothing.  kf_last_error() describes the
 *    last failure of the calling thread.
 *  - The workspace is DEVICE memory of at least kf_workspace_bytes() bytes,
 *    16-byte aligned, zero-filled once by the caller before its first use; the
 *    library leaves it reusable after every call.  Calls that share a workspace
 *    must be ordered on one stream.
 *  - Supported element type / head dimension pairs: bf16 and IEEE half with d in
 *    {64,128,256}, fp32 with d in {64,128}; query heads per cached head: 1, 2, 4
 *    or 8.  Q, K, V, k_new and v_new share the cache's element type.
 */
#ifndef KEYFORMER_H
#define KEYFORMER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KF_OK = 0,
    KF_EINVAL = -1,       /* null pointer, size out of range, non-finite tau ... */
    KF_EUNSUPPORTED = -2, /* dtype / head-dimension pair not built */
    KF_EWORKSPACE = -3,   /* workspace missing, misaligned or too small */
    KF_EDEVICE = -4       /* the HIP runtime refused a launch */
} kf_status;

typedef enum { KF_F32 = 0, KF_BF16 = 1, KF_F16 = 2 /* IEEE half */ } kf_dtype;

/* Logit adjustment zeta of Eq. 4.  GUMBEL is the method (Eq. 7); NONE is the
 * accumulated-attention score of prior work; GAUSSIAN (Eq. 5, mean 0.5772,
 * std 1.2825) and CONSTANT (0.5772) are the paper's ablation variants. */
typedef enum {
    KF_NOISE_NONE = 0,
    KF_NOISE_GUMBEL = 1,
    KF_NOISE_GAUSSIAN = 2,
    KF_NOISE_CONSTANT = 3
} kf_noise;

/* How kf_select_evict keeps the survivors.
 *  ORDERED  slots stay sorted by original position: rows behind an evicted slot
 *           move down (Algorithm 1 slices f[:-w], i.e. presumes positional order).
 *  SLOT     the cache is an unordered set of (pos, K, V, score) entries: on a
 *           decode step the newest entry takes the evicted entry's slot, one row
 *           moves.  Window membership and tie-breaks are decided through pos, so
 *           the retained SET is the same as in ORDERED.  Needs len <= k+1. */
typedef enum { KF_LAYOUT_ORDERED = 0, KF_LAYOUT_SLOT = 1 } kf_layout;

/* The per-layer, per-head caches (Fig. 5: scores accumulate "for each layer
 * and head").  Row j of a unit is one cached token. */
typedef struct {
    void *K;        /* DEVICE [L][B][H][cap][d] keys,   element type `dtype`, 16-byte aligned */
    void *V;        /* DEVICE [L][B][H][cap][d] values                                   */
    float *score;   /* DEVICE [L][B][H][cap]    accumulated score f_theta (Sec. 3.3.2)    */
    int32_t *pos;   /* DEVICE [L][B][H][cap]    original position of each token ("Org Pos",
                       Sec. 4.4.2); ascending over slots [0,len)                          */
    int32_t *len;   /* DEVICE [L][B][H]         live tokens per unit                      */
    int32_t L, B, H, d, cap;
    int32_t dtype;  /* kf_dtype */
    int32_t layer0; /* model-wide index of the cache's first layer; enters the noise key only, so
                       a cache that holds a subset of the layers draws the same noise */
    int32_t q_per_kv; /* query heads served by each cached head: 1 (or 0) = multi-head attention;
                       2, 4 or 8 = grouped-query / multi-query attention (Sec. 6: the method applies
                       unchanged).  Cached head h then serves query heads h*G .. h*G+G-1: Q, q and
                       out hold H*G heads ([L][B][H*G]...), alibi_slopes holds H*G slopes, each query
                       head has its own logits, attention output and noise stream (keyed by the
                       QUERY head index), and score[.][.][h] accumulates the SUM of its G query
                       heads' increments -- the heads share the cached tokens, hence the decision */
} kf_cache;

/* Which positions the position bias sees (Sec. 4.4.2): the tokens' original
 * positions ("Org Pos", the default and the better ablation), or their positions
 * within the reduced cache ("New Pos": key j at slot j, the query at slot m-1).
 * The noise key always uses original positions.  KF_POS_NEW reads a token's position off its slot, so it
 * presumes the ordered layout (in KF_LAYOUT_SLOT the slots carry no order). */
typedef enum { KF_POS_ORIGINAL = 0, KF_POS_NEW = 1 } kf_pos_mode;

/* Whether every layer accumulates its own score (the method, and the better
 * ablation) or one score serves all layers (Sec. 4.4.1, "Shared"): then each
 * scoring call adds the contributions of ALL layers of the cache, in layer
 * order, to the score of every (batch, head), every layer's `score` rows hold
 * the same copy of it, and so all layers retain the same tokens.  A shared score
 * needs all layers in one cache, holding the same tokens (equal len and pos per
 * (batch, head) over the layers); a call on layers that disagree in len leaves
 * the scores of that (batch, head) alone and increments the workspace error word. */
typedef enum { KF_SCORE_PER_LAYER = 0, KF_SCORE_SHARED = 1 } kf_score_mode;

/* Parameters of the score function (Eq. 11) for one call. */
typedef struct {
    float tau;                 /* temperature of this iteration, from kf_tau()            */
    float scale;               /* logit scale, 1/sqrt(d) in Eq. 1                         */
    int32_t noise;             /* kf_noise                                                */
    const uint64_t *seeds;     /* DEVICE [B] one noise seed per sequence; may be NULL
                                  when noise is NONE or CONSTANT                          */
    const float *alibi_slopes; /* DEVICE [H] or NULL.  Adds -slope[h]*(q_pos - pos_j) to
                                  the logits (MPT's position bias)                        */
    int32_t pos_mode;          /* kf_pos_mode; only matters with alibi_slopes, decode only */
    int32_t score_mode;        /* kf_score_mode                                           */
    const int32_t *seq_q_pos;  /* DEVICE [B] or NULL.  Decode only: sequence b's new token sits at
                                  seq_q_pos[b] instead of the call's q_pos -- for batches whose
                                  sequences are at different points of their generation         */
    const float *seq_tau;      /* DEVICE [B] or NULL.  Decode only: sequence b's temperature of this
                                  step (Eq. 12 with its own t and T) instead of tau; every entry
                                  must be finite and positive (not checked: device memory)      */
    const int32_t *seq_n;      /* DEVICE [B] or NULL.  Prompt scoring only: sequence b's prompt has
                                  seq_n[b] tokens, rows seq_n[b]..n-1 of its Q and K are padding
                                  (a batch of prompts of different lengths, padded at the end)   */
} kf_score_cfg;

/* Library version, for the binding to check it loaded what it expects. */
int32_t kf_version(void);

/* Text of the calling thread's last error ("" if none). */
const char *kf_last_error(void);

/* Temperature schedule, Eq. 12: tau_init + t*(tau_end - tau_init)/T, evaluated
 * in fp32.  t = 0 is the prompt iteration, t = 1..T the decode steps. */
float kf_tau(int32_t t, int32_t T, float tau_init, float tau_end);

/* Host mirror of the device noise hash: the 32 random bits behind zeta for
 * (seed, layer, head, query position, key's original position).  The uniform is
 * u = (2*(bits>>9)+1)/2^24 and the Gumbel variate of Eq. 7 is -ln(-ln u). */
uint32_t kf_noise_bits(uint64_t seed, uint32_t layer, uint32_t head, uint32_t q_pos, uint32_t k_pos);

/* Bytes of workspace that suffice for any call of this library on this
 * cache, with prompt length up to n_max (pass 0 if kf_prefill_score is not
 * used).  Only the cache's dimensions are read. */
size_t kf_workspace_bytes(const kf_cache *c, int32_t n_max);

/* How kf_decode_step would shape its launch for this cache and m_hint (0 = cap):
 * *splits = workgroups per unit, *chunk = cache rows per workgroup.  Host only;
 * for callers that want to reason about occupancy.  Returns KF_EINVAL /
 * KF_EUNSUPPORTED like the hot calls. */
kf_status kf_decode_launch_shape(const kf_cache *c, int32_t m_hint, int32_t *splits, int32_t *chunk);

/* Device-side error counter: the first int32 of the workspace counts units a
 * kernel had to skip (kf_decode_step on a unit with len >= cap, kf_select_evict in
 * the SLOT layout on a unit more than one token over budget).  Exposed as a
 * constant so callers can read it back themselves. */
#define KF_WS_ERROR_WORD 0
/* The second int32 of the workspace is a counter the library uses within a launch and leaves at zero. */
#define KF_WS_TICKET_WORD 1

/*
 * Prompt-phase scoring (Sec. 3.4, Algorithm 1 prompt branch).  For every unit,
 * with the n prompt keys already stored in rows 0..n-1 of K:
 *     x_ij = scale*<Q_i, K_j> - slope_h*(i-j)          j <= i   (causal)
 *     z_i  = softmax_j((x_ij + zeta_ij)/tau)                    (Eq. 4, Eq. 11)
 *     score[j] = sum_{i>=j} z_ij ;  pos[j] = j ;  len = n
 * Q is DEVICE [L][B][H][n][d] in the cache's dtype.  V is not touched.
 * With cfg->seq_n every unit of sequence b is scored over its own first
 * n_b = seq_n[b] rows exactly as if it had been passed alone with n = n_b (the
 * padding rows are neither queries nor keys; score and pos beyond n_b are left
 * as they were; len = n_b); Q keeps the row stride n.  A sequence whose seq_n[b]
 * lies outside [1, n] is skipped and each of its units counted in the error word.
 * Errors: KF_EINVAL if n < 1 or n > cap, tau not finite or <= 0, null pointers,
 * seeds missing for a random adjustment.
 */
kf_status kf_prefill_score(const kf_cache *c, const void *Q, int32_t n, const kf_score_cfg *cfg,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * One generation step (Algorithm 1 else-branch) for every unit:
 *   append   K[len] = k_new, V[len] = v_new, pos[len] = q_pos, score[len] = 0; m = len+1
 *   logits   x_j = scale*<q, K_j> - slope_h*(q_pos - pos_j)              (Eq. 1)
 *   attend   out = sum_j softmax(x)_j V_j                   (no noise, no tau)
 *   score    score[j] += softmax((x + zeta)/tau)_j   for all j < m  (Eq. 11, Sec. 3.3.2)
 *   len      = m
 * q, k_new, v_new are DEVICE [L][B][H][d] in the cache's dtype; out is DEVICE
 * [L][B][H][d] fp32.  q_pos is the absolute position of the new token (n+t-1
 * at decode step t).  m_hint is an upper bound of len+1 over all units, used
 * only to shape the launch; pass 0 (= cap) if unknown.
 * A unit whose len is already cap is skipped: its `out` is zero-filled and the
 * workspace error word is incremented.
 * Errors: KF_EINVAL for null pointers, q_pos < 0, bad tau, m_hint > cap;
 * KF_EWORKSPACE if the workspace is too small.
 */
kf_status kf_decode_step(kf_cache *c, const void *q, const void *k_new, const void *v_new,
                         int32_t q_pos, int32_t m_hint, const kf_score_cfg *cfg, float *out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * Key-token selection and KV compaction (Algorithm 1: S_w, S_key, S_k; Sec. 3.4).
 * Units with len <= k are left untouched.  Otherwise the survivors are the last
 * w slots plus the k-w slots of [0, len-w) with the largest score, equal scores
 * resolved in favour of the lower slot; K, V, score and pos rows of the
 * survivors move to slots [0,k) in their original order, in place; len = k.
 * kept_idx, if not NULL, is DEVICE [L][B][H][k] and receives the pre-compaction
 * slot of every survivor (identity, then -1 padding, for untouched units).
 * layout is a kf_layout.  With KF_LAYOUT_SLOT a unit more than one token over
 * budget is left untouched and the workspace error word is incremented; the
 * recent window is then the entries with pos > newest pos - w (the w largest
 * positions, given that a generation appends consecutive positions), and equal
 * scores keep the lower pos.
 * Errors: KF_EINVAL if k < 1, w < 0, w > k, k > cap or layout unknown.
 */
kf_status kf_select_evict(kf_cache *c, int32_t k, int32_t w, int32_t layout, int32_t *kept_idx,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same selection (ordered layout), but the survivors are gathered into
 * ANOTHER cache: layer l of `src` goes to layer dst_layer0 + l of `dst`, slots
 * [0,k), in original order; dst len = min(src len, k).  `src` is not modified.
 * This is the prompt-phase eviction (Sec. 3.4: n - k tokens are dropped right
 * after the prompt) for callers that stage a layer's n-token prompt cache and
 * keep only a (k+1)-token cache per layer for the generation.  B, H, d and
 * dtype must agree, dst->cap >= k, and the two caches must not share buffers.
 * The workspace is sized by the SOURCE cache (kf_workspace_bytes(src, ...)).
 */
kf_status kf_select_evict_into(const kf_cache *src, kf_cache *dst, int32_t dst_layer0, int32_t k, int32_t w,
                               int32_t *kept_idx, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Beam search with one cache per beam (Sec. 4: every evaluation runs 4 beams;
 * Sec. 6: tokens are discarded across heads, layers and beams).  Rows of the
 * batch dimension are beams; after a search step row b continues the hypothesis
 * that row parent[b] held.  For every b with parent[b] != b the live entries of
 * all of row parent[b]'s units (K, V, score, pos rows [0, len), and len) are
 * copied to row b's; rows with parent[b] == b are not touched.  A parent must
 * continue itself (parent[parent[b]] == parent[b]: its row is read while others
 * are written), which the caller arranges by numbering the new beams so that
 * every surviving hypothesis keeps its row for one of its continuations and the
 * others take the rows of hypotheses that died.  Only forked beams cost traffic.
 * parent is DEVICE [B].  A row whose parent is out of range or does not continue
 * itself is left as it is and each of its units counted in the error word.
 * Errors: KF_EINVAL for null pointers.
 */
kf_status kf_beam_fork(kf_cache *c, const int32_t *parent, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One whole generation step: kf_decode_step followed by kf_select_evict, with
 * the same arguments, results and error behaviour as the two calls in a row,
 * in as few kernel launches as the shape allows: one in the slot layout when
 * every unit is handled by a single workgroup (that workgroup also evicts and
 * stores the new token straight into the freed slot), else the merge of the
 * decode kernel's split-wise results rides in the selection kernel where that
 * pays.  Algorithm 1, one iteration of the else-branch including the S_w /
 * S_key / S_k lines.
 */
kf_status kf_decode_select_step(kf_cache *c, const void *q, const void *k_new, const void *v_new,
                                int32_t q_pos, int32_t m_hint, const kf_score_cfg *cfg, float *out,
                                int32_t k, int32_t w, int32_t layout, int32_t *kept_idx, void *workspace,
                                size_t workspace_bytes, void *stream);

/* The generation schedule of Algorithm 1, for the call below that takes the
 * step number from device memory. */
typedef struct {
    int32_t n;       /* prompt length: decode step t appends the token at position n + t - 1 */
    int32_t T;       /* planned generation length of Eq. 12; steps beyond T keep tau_end      */
    float tau_init;  /* temperature of the prompt iteration (t = 0)                           */
    float tau_end;   /* temperature of step T                                                 */
} kf_schedule;

/*
 * kf_decode_select_step with the step number t read from DEVICE memory when the
 * kernels run: q_pos = n + t - 1 and tau = kf_tau(min(t, T), T, tau_init,
 * tau_end) (the same fp32 operations, so the same bits; cfg->tau is ignored),
 * and the last kernel of the step stores t + 1 back.  One such call captured in
 * a HIP graph therefore replays as successive generation steps (Algorithm 1's
 * loop over t) with no host work in between; the caller refreshes q, k_new and
 * v_new in place between replays, or captures several calls with their own
 * input buffers.  `step` is DEVICE [1] int32, set to 1 by the caller before the
 * first decode step; values below 1 are read as 1.  `sched` is HOST memory read
 * during the call.  Everything else as kf_decode_select_step.
 * Errors: additionally KF_EINVAL if step or sched is NULL, n < 0, T < 1, or the
 * temperatures are not finite and positive.
 */
kf_status kf_decode_select_step_at(kf_cache *c, const void *q, const void *k_new, const void *v_new,
                                   const kf_schedule *sched, int32_t *step, int32_t m_hint,
                                   const kf_score_cfg *cfg, float *out, int32_t k, int32_t w, int32_t layout,
                                   int32_t *kept_idx, void *workspace, size_t workspace_bytes, void *stream);

/*
 * kf_decode_select_step for callers that cannot allocate device memory and have
 * no workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same step, same kernels, same results as
 * kf_decode_select_step; the scratch the kernels need (split-wise partial
 * results, score increments, survivor lists, counters) lives in a buffer of
 * KF_NOALLOC_SCRATCH_BYTES built into the library's device code, one per GPU,
 * held from the library's load until the process ends.  The call allocates and
 * frees nothing, and clears the buffer's counters itself by a kernel (no memset
 * node), so it can be captured.
 *  - `skipped`, DEVICE [1] or NULL, plays the workspace error word: it is
 *    incremented by one for every unit the kernels had to skip.  The caller
 *    zeroes it; with NULL the count is dropped.
 *  - Every call on a GPU uses that GPU's one buffer: calls on the same GPU
 *    must not overlap (order them on one stream, or by events); overlapping
 *    calls race.
 *  - The first call on a device looks up the buffer's device address
 *    (hipGetSymbolAddress); make that call outside a stream capture.
 * Errors: as kf_decode_select_step; KF_EWORKSPACE if the cache's shape needs
 * more than KF_NOALLOC_SCRATCH_BYTES of scratch (kf_workspace_bytes(c, 0) tells);
 * KF_EDEVICE if the buffer's address cannot be resolved.
 */
#define KF_NOALLOC_SCRATCH_BYTES (32u << 20)
kf_status kf_decode_select_step_noalloc(kf_cache *c, const void *q, const void *k_new, const void *v_new,
                                        int32_t q_pos, int32_t m_hint, const kf_score_cfg *cfg, float *out,
                                        int32_t k, int32_t w, int32_t layout, int32_t *kept_idx,
                                        int32_t *skipped, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KEYFORMER_H */
