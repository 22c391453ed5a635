// C ABI of the Keyformer library: argument validation on the host, workspace
// carving, kernel launches.  Nothing here allocates device memory.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "kf_device.h"
#include "kf_internal.h"

// Built-in scratch of the allocation-free entry point (kf_decode_select_step_noalloc): one array per GPU
// the library runs on, held until the process ends.  In host code the name is only a handle: it is never
// passed to a kernel or a copy; the runtime is asked once per device for the array's device address
// (scratch_of_current_device below) and that address is used from then on.
static __device__ __align__(256) unsigned char scratch[KF_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char g_err[256] = "";

kf_status fail(kf_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int64_t kMaxGrid = 0x7fffffff;  // workgroups of a one-dimensional launch
// A fused step folds the merge of a split unit into the selection kernel (one workgroup per unit) only
// while that workgroup walks the unit's tokens in a few strides; longer units take the merge launch,
// which spreads a unit over several workgroups (32 heads x 9.8k tokens: 55.5 us folded, 52.6 us apart).
constexpr int64_t kTailMergeMaxTokens = 4096;
constexpr int64_t kWideMaxUnits = 256;
constexpr int32_t kPreselMinTokens = 4096;

bool supported(int32_t dtype, int32_t d) {
    if (dtype == KF_BF16 || dtype == KF_F16) return d == 64 || d == 128 || d == 256;
    if (dtype == KF_F32) return d == 64 || d == 128;
    return false;
}

bool group_supported(int32_t g) { return g == 0 || g == 1 || g == 2 || g == 4 || g == 8; }
int32_t group_of(const kf_cache* c) { return c->q_per_kv > 1 ? c->q_per_kv : 1; }

kf_status check_cache(const kf_cache* c) {
    if (!c) return fail(KF_EINVAL, "cache is NULL");
    if (!c->K || !c->V || !c->score || !c->pos || !c->len) return fail(KF_EINVAL, "cache has a NULL buffer");
    if (c->L < 1 || c->B < 1 || c->H < 1 || c->cap < 1 || c->d < 1)
        return fail(KF_EINVAL, "cache dimensions must be positive (L=%d B=%d H=%d d=%d cap=%d)", c->L, c->B, c->H,
                    c->d, c->cap);
    if ((int64_t)c->L * c->B * c->H > (int64_t)1 << 24) return fail(KF_EINVAL, "too many units");
    if (c->layer0 < 0) return fail(KF_EINVAL, "layer0 must be non-negative");
    if (c->dtype != KF_F32 && c->dtype != KF_BF16 && c->dtype != KF_F16) return fail(KF_EINVAL, "unknown dtype %d", c->dtype);
    if (!supported(c->dtype, c->d))
        return fail(KF_EUNSUPPORTED, "dtype %d with head dimension %d is not built", c->dtype, c->d);
    if (((uintptr_t)c->K | (uintptr_t)c->V) & 15) return fail(KF_EINVAL, "K and V must be 16-byte aligned");
    if (c->q_per_kv < 0) return fail(KF_EINVAL, "q_per_kv must not be negative");
    if (!group_supported(c->q_per_kv))
        return fail(KF_EUNSUPPORTED, "%d query heads per cached head is not built (1, 2, 4 or 8)", c->q_per_kv);
    return KF_OK;
}

kf_status check_cfg(const kf_score_cfg* cfg) {
    if (!cfg) return fail(KF_EINVAL, "score configuration is NULL");
    if (!(cfg->tau > 0.0f) || !isfinite(cfg->tau)) return fail(KF_EINVAL, "tau must be finite and positive");
    if (!isfinite(cfg->scale)) return fail(KF_EINVAL, "scale must be finite");
    if (cfg->noise < KF_NOISE_NONE || cfg->noise > KF_NOISE_CONSTANT)
        return fail(KF_EINVAL, "unknown noise mode %d", cfg->noise);
    if (cfg->pos_mode != KF_POS_ORIGINAL && cfg->pos_mode != KF_POS_NEW)
        return fail(KF_EINVAL, "unknown pos_mode %d", cfg->pos_mode);
    if (cfg->score_mode != KF_SCORE_PER_LAYER && cfg->score_mode != KF_SCORE_SHARED)
        return fail(KF_EINVAL, "unknown score_mode %d", cfg->score_mode);
    if ((cfg->noise == KF_NOISE_GUMBEL || cfg->noise == KF_NOISE_GAUSSIAN) && !cfg->seeds)
        return fail(KF_EINVAL, "a random logit adjustment needs seeds");
    return KF_OK;
}

// Workspace layout (all regions 256-byte aligned):
//   [0]        error word + padding (the only part that must start as zero)
//   region X   the largest of
//                decode : partial records U*S*G*(d+4) floats, then increments U*G*cap floats, then
//                         per-unit token counts U int32 (shared score), then (fused step) the
//                         survivor index list U*cap int32
//                select : survivor index list U*cap int32
//                prefill: row normalisers U*G*n_pad floats, then row keys U*G*n_pad uint32, then
//                         (G > 1) per-query-head column sums U*G*n_pad floats
//              (G = query heads per cached head)
struct WsLayout {
    size_t region, fused_idx, wide, total;  // wide: boundary entries of the two-launch ordered eviction
    int32_t nb;                             // boundary slots per unit
};

// Bytes of the wide eviction's scratch: evicted slot per unit, then per unit and boundary the K and V rows,
// then the scores, then the positions (each part 256-byte aligned).
size_t wide_part(size_t bytes) { return align_up(bytes, 256); }

size_t decode_region(int64_t U, const kf_cache* c) {
    const int32_t G = group_of(c);
    const kf::DecodePlan p = kf::plan_decode(U, c->cap, c->d, c->dtype, G);
    return align_up((size_t)U * p.S * G * (c->d + 4) * sizeof(float), 256) +
           align_up((size_t)U * G * c->cap * sizeof(float), 256) + align_up((size_t)U * sizeof(int32_t), 256);
}

WsLayout ws_layout(const kf_cache* c, int32_t n_max) {
    const int64_t U = (int64_t)c->L * c->B * c->H;
    WsLayout w;
    w.region = 256;
    const size_t dec = decode_region(U, c);
    const size_t sel = align_up((size_t)U * c->cap * sizeof(int32_t), 256);
    w.fused_idx = w.region + dec;  // a fused step keeps the decode records while it selects
    size_t x = dec + sel;
    if (n_max > 0) {
        const size_t n_pad = align_up((size_t)n_max, kf::kPrefillRowPad);
        const int32_t G = group_of(c);
        const size_t pre = (G > 1 ? 3 : 2) * align_up((size_t)U * G * n_pad * sizeof(float), 256);
        if (pre > x) x = pre;
    }
    w.wide = w.region + x;
    const int32_t row_bytes = c->d * (c->dtype == KF_F32 ? 4 : 2);
    w.nb = U <= kWideMaxUnits ? c->cap / kf::wide_chunk_rows(row_bytes) : 0;  // only small launches go wide
    w.total = w.wide + wide_part((size_t)U * 4) + wide_part((size_t)U * w.nb * 2 * row_bytes) +
              2 * wide_part((size_t)U * w.nb * 4) + wide_part((size_t)U * kf::kPreselMaxSlices * 8) +
              wide_part((size_t)U * kf::kPreselMaxSlices * 4);
    return w;
}

// Whether the two-launch ordered eviction is the faster one for U units of budget k.
// Measured (MI355X): 32 units x 32k tokens 770 -> 240 us per step, 32 x 9.8k 237 -> 88, 16 x 1k 53 -> 29,
// 256 x 2k 129 -> 125; from a few hundred units on one workgroup per unit moves the rows at the chip's copy
// rate by itself (448 x 1k: 49 vs 53 us, 8192 x 2k: 1229 vs 1324 us).
bool wide_pays(int64_t U, int32_t k) { return U <= kWideMaxUnits && k >= 64; }

kf_status check_ws(const void* ws, size_t have, size_t need) {
    if (!ws) return fail(KF_EWORKSPACE, "workspace is NULL");
    if ((uintptr_t)ws & 15) return fail(KF_EWORKSPACE, "workspace must be 16-byte aligned");
    if (have < need) return fail(KF_EWORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
    return KF_OK;
}

// ---- built-in scratch of the allocation-free entry point (kf_decode_select_step_noalloc) ----
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once resolved
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch`.
kf_status scratch_of_current_device(void** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(KF_EDEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(KF_EDEVICE, "device index %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(KF_EDEVICE, "address of the built-in scratch on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return KF_OK;
}

// The words of a workspace that must start a call as zero (error word, ticket word): a fill kernel, not a
// memset node, so that the call can be captured in a HIP graph.
__global__ void clear_header_kernel(int32_t* head) { head[threadIdx.x] = 0; }

}  // namespace

extern "C" {

int32_t kf_version(void) { return 1; }

const char* kf_last_error(void) { return g_err; }

float kf_tau(int32_t t, int32_t T, float tau_init, float tau_end) {
    const float dtau = (tau_end - tau_init) / (float)T;
    return kf::schedule_tau(tau_init, dtau, t);
}

uint32_t kf_noise_bits(uint64_t seed, uint32_t layer, uint32_t head, uint32_t q_pos, uint32_t k_pos) {
    return kf::logit_bits(kf::row_key(kf::unit_key(seed, layer, head), q_pos), k_pos);
}

size_t kf_workspace_bytes(const kf_cache* c, int32_t n_max) {
    if (!c || c->L < 1 || c->B < 1 || c->H < 1 || c->cap < 1 || !supported(c->dtype, c->d)) return 0;
    if (!group_supported(c->q_per_kv)) return 0;
    if (n_max < 0) n_max = 0;
    return ws_layout(c, n_max).total;
}

kf_status kf_decode_launch_shape(const kf_cache* c, int32_t m_hint, int32_t* splits, int32_t* chunk) {
    if (!c || !splits || !chunk) return fail(KF_EINVAL, "NULL argument");
    if (c->L < 1 || c->B < 1 || c->H < 1 || c->cap < 1) return fail(KF_EINVAL, "cache dimensions must be positive");
    if (!supported(c->dtype, c->d))
        return fail(KF_EUNSUPPORTED, "dtype %d with head dimension %d is not built", c->dtype, c->d);
    if (m_hint < 0 || m_hint > c->cap) return fail(KF_EINVAL, "m_hint %d outside [0, cap=%d]", m_hint, c->cap);
    if (!group_supported(c->q_per_kv))
        return fail(KF_EUNSUPPORTED, "%d query heads per cached head is not built", c->q_per_kv);
    const kf::DecodePlan p =
        kf::plan_decode((int64_t)c->L * c->B * c->H, m_hint ? m_hint : c->cap, c->d, c->dtype, group_of(c));
    *splits = p.S;
    *chunk = p.chunk;
    return KF_OK;
}

kf_status kf_prefill_score(const kf_cache* c, const void* Q, int32_t n, const kf_score_cfg* cfg, void* workspace,
                           size_t workspace_bytes, void* stream) {
    kf_status st = check_cache(c);
    if (st != KF_OK) return st;
    st = check_cfg(cfg);
    if (st != KF_OK) return st;
    if (!Q) return fail(KF_EINVAL, "Q is NULL");
    if ((uintptr_t)Q & 15) return fail(KF_EINVAL, "Q must be 16-byte aligned");
    if (n < 1 || n > c->cap) return fail(KF_EINVAL, "prompt length %d outside [1, cap=%d]", n, c->cap);
    const WsLayout w = ws_layout(c, n);
    st = check_ws(workspace, workspace_bytes, w.total);
    if (st != KF_OK) return st;

    const int32_t G = group_of(c);
    const int64_t U = (int64_t)c->L * c->B * c->H * G;  // query units
    if ((U + 7) / 8 * 8 * ((n + 127) / 128) > kMaxGrid)  // one workgroup per 128 prompt rows of a unit
        return fail(KF_EUNSUPPORTED, "%lld query units of %d prompt rows exceed the largest launch", (long long)U, n);
    const size_t n_pad = align_up((size_t)n, kf::kPrefillRowPad);
    kf::PrefillArgs a;
    a.Q = Q;
    a.K = c->K;
    a.score = c->score;
    a.pos = c->pos;
    a.len = c->len;
    a.seeds = cfg->seeds;
    a.slopes = cfg->alibi_slopes;
    a.seq_n = cfg->seq_n;
    a.ws_err = (int32_t*)workspace + KF_WS_ERROR_WORD;
    a.ws_c = (float*)((char*)workspace + w.region);
    a.ws_r = (uint32_t*)((char*)workspace + w.region + align_up((size_t)U * n_pad * sizeof(float), 256));
    a.ws_f = (float*)((char*)workspace + w.region + 2 * align_up((size_t)U * n_pad * sizeof(float), 256));
    a.G = G;
    a.B = c->B;
    a.H = c->H * G;
    a.cap = c->cap;
    a.layer0 = c->layer0;
    a.n = n;
    a.n_pad = (int32_t)n_pad;
    a.noise = cfg->noise;
    a.inv_tau = 1.0f / cfg->tau;
    a.scale = cfg->scale;
    hipError_t e = kf::launch_prefill(a, U, c->d, c->dtype, (hipStream_t)stream);
    if (e == hipSuccess && cfg->score_mode == KF_SCORE_SHARED) {
        kf::ShareArgs sh;
        sh.score = c->score;
        sh.inc = nullptr;
        sh.m = c->len;
        sh.ws_err = (int32_t*)workspace + KF_WS_ERROR_WORD;
        sh.L = c->L;
        sh.BH = c->B * c->H;
        sh.cap = c->cap;
        sh.inc_unit = 0;
        e = kf::launch_share(sh, (hipStream_t)stream);
    }
    if (e != hipSuccess) return fail(KF_EDEVICE, "prefill launch: %s", hipGetErrorString(e));
    g_err[0] = 0;
    return KF_OK;
}

// Validates the arguments of a decode step and fills the kernel arguments.
static kf_status prepare_decode(kf_cache* c, const void* q, const void* k_new, const void* v_new, int32_t q_pos,
                                int32_t m_hint, const kf_score_cfg* cfg, float* out, void* workspace,
                                size_t workspace_bytes, kf::DecodeArgs* a, kf::DecodePlan* plan) {
    kf_status st = check_cache(c);
    if (st != KF_OK) return st;
    st = check_cfg(cfg);
    if (st != KF_OK) return st;
    if (!q || !k_new || !v_new || !out) return fail(KF_EINVAL, "q, k_new, v_new and out must not be NULL");
    if (((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new) & 15)
        return fail(KF_EINVAL, "q, k_new and v_new must be 16-byte aligned");
    if (q_pos < 0) return fail(KF_EINVAL, "q_pos must be non-negative");
    if (m_hint < 0 || m_hint > c->cap) return fail(KF_EINVAL, "m_hint %d outside [0, cap=%d]", m_hint, c->cap);
    if (m_hint == 0) m_hint = c->cap;
    const WsLayout w = ws_layout(c, 0);
    st = check_ws(workspace, workspace_bytes, w.total);
    if (st != KF_OK) return st;

    const int64_t U = (int64_t)c->L * c->B * c->H;
    const int32_t G = group_of(c);
    const kf::DecodePlan p = kf::plan_decode(U, m_hint, c->d, c->dtype, G);
    // the partial-record region is sized for the plan at m = cap, the largest
    const kf::DecodePlan pmax = kf::plan_decode(U, c->cap, c->d, c->dtype, G);
    if (p.S > pmax.S) return fail(KF_EWORKSPACE, "internal: split count %d exceeds the sized %d", p.S, pmax.S);
    if (U * p.S > kMaxGrid)
        return fail(KF_EUNSUPPORTED, "%lld units in %d splits each exceed the largest launch", (long long)U, p.S);
    a->K = c->K;
    a->V = c->V;
    a->score = c->score;
    a->pos = c->pos;
    a->len = c->len;
    a->q = q;
    a->k_new = k_new;
    a->v_new = v_new;
    a->out = out;
    a->seeds = cfg->seeds;
    a->slopes = cfg->alibi_slopes;
    a->ws_err = (int32_t*)workspace + KF_WS_ERROR_WORD;
    a->ws_part = (float*)((char*)workspace + w.region);
    a->ws_e =
        (float*)((char*)workspace + w.region + align_up((size_t)U * pmax.S * G * (c->d + 4) * sizeof(float), 256));
    a->ws_m = (int32_t*)((char*)a->ws_e + align_up((size_t)U * G * c->cap * sizeof(float), 256));
    a->G = G;
    a->B = c->B;
    a->H = c->H;
    a->cap = c->cap;
    a->layer0 = c->layer0;
    a->S = p.S;
    a->chunk = p.chunk;
    a->q_pos = q_pos;
    a->noise = cfg->noise;
    a->new_pos = cfg->pos_mode == KF_POS_NEW ? 1 : 0;
    a->shared = cfg->score_mode == KF_SCORE_SHARED ? 1 : 0;
    if (a->shared && c->L > 65535) return fail(KF_EUNSUPPORTED, "a shared score over %d layers is not built", c->L);
    a->seq_q_pos = cfg->seq_q_pos;
    a->seq_tau = cfg->seq_tau;
    a->fuse_k = 0;
    a->pre_slices = 0;
    a->pre_k = a->pre_w = a->pre_layout = 0;
    a->pre_min = nullptr;
    a->pre_slot = nullptr;
    a->fuse_w = 0;
    a->fuse_idx = nullptr;
    a->step_inc = nullptr;
    a->ws_ticket = (int32_t*)workspace + KF_WS_TICKET_WORD;
    a->step = nullptr;
    a->n0 = 0;
    a->T = 1;
    a->tau_init = 0.0f;
    a->dtau = 0.0f;
    a->inv_tau = 1.0f / cfg->tau;
    a->scale = cfg->scale;
    *plan = p;
    return KF_OK;
}

// Second half of a scoring call with a shared score: the layers' contributions are added up.
static hipError_t share_after_decode(const kf_cache* c, const kf::DecodeArgs& a, hipStream_t stream) {
    kf::ShareArgs sh;
    sh.score = c->score;
    sh.inc = a.ws_e;
    sh.m = a.ws_m;
    sh.ws_err = a.ws_err;
    sh.L = c->L;
    sh.BH = c->B * c->H;
    sh.cap = c->cap;
    sh.inc_unit = a.G * c->cap;
    return kf::launch_share(sh, stream);
}

// Same for a selection.  In a fused step the decode records occupy region X of
// the workspace, so the survivor index list (needed only when the caller wants
// no kept_idx) lives behind them.
static kf_status prepare_select(kf_cache* c, int32_t k, int32_t w, int32_t layout, int32_t* kept_idx,
                                void* workspace, size_t workspace_bytes, bool fused, kf::SelectArgs* a) {
    kf_status st = check_cache(c);
    if (st != KF_OK) return st;
    if (k < 1 || k > c->cap) return fail(KF_EINVAL, "budget k=%d outside [1, cap=%d]", k, c->cap);
    if (w < 0 || w > k) return fail(KF_EINVAL, "window w=%d outside [0, k=%d]", w, k);
    if (layout != KF_LAYOUT_ORDERED && layout != KF_LAYOUT_SLOT) return fail(KF_EINVAL, "unknown layout %d", layout);
    const WsLayout wl = ws_layout(c, 0);
    st = check_ws(workspace, workspace_bytes, wl.total);
    if (st != KF_OK) return st;
    const int64_t U = (int64_t)c->L * c->B * c->H;
    a->K = c->K;
    a->V = c->V;
    a->score = c->score;
    a->pos = c->pos;
    a->len = c->len;
    a->idx = kept_idx ? kept_idx : (int32_t*)((char*)workspace + (fused ? wl.fused_idx : wl.region));
    a->cap = c->cap;
    a->k = k;
    a->w = w;
    a->row_bytes = c->d * (c->dtype == KF_F32 ? 4 : 2);
    a->idx_is_output = kept_idx ? 1 : 0;
    a->layout = layout;
    a->move = 1;
    a->ws_err = (int32_t*)workspace + KF_WS_ERROR_WORD;
    a->step_inc = nullptr;
    // Few units, or long ones: one workgroup per unit cannot move the rows of an ordered eviction at the
    // chip's rate, so a second launch spreads every unit's rows over many workgroups.
    a->chunk_rows = kf::wide_chunk_rows(a->row_bytes);
    a->nb = wl.nb;
    a->wide = (layout == KF_LAYOUT_ORDERED && a->nb > 0 && wide_pays(U, k)) ? 1 : 0;
    char* wp = (char*)workspace + wl.wide;
    a->ws_evict = (int32_t*)wp;
    wp += wide_part((size_t)U * 4);
    a->ws_brow = wp;
    wp += wide_part((size_t)U * wl.nb * 2 * a->row_bytes);
    a->ws_bscore = (float*)wp;
    wp += wide_part((size_t)U * wl.nb * 4);
    a->ws_bpos = (int32_t*)wp;
    wp += wide_part((size_t)U * wl.nb * 4);
    // long units of a small launch: the candidate scan is cut into slices by a launch of its own
    a->presel = 0;
    a->presel_done = 0;
    if (U <= kWideMaxUnits && c->cap >= kPreselMinTokens) {
        a->presel = (c->cap + 2047) / 2048;
        if (a->presel > kf::kPreselMaxSlices) a->presel = kf::kPreselMaxSlices;
    }
    a->ws_pmin = (unsigned long long*)wp;
    wp += wide_part((size_t)U * kf::kPreselMaxSlices * 8);
    a->ws_pslot = (int32_t*)wp;
    return KF_OK;
}

kf_status kf_decode_step(kf_cache* c, const void* q, const void* k_new, const void* v_new, int32_t q_pos,
                         int32_t m_hint, const kf_score_cfg* cfg, float* out, void* workspace,
                         size_t workspace_bytes, void* stream) {
    kf::DecodeArgs a;
    kf::DecodePlan p;
    const kf_status st = prepare_decode(c, q, k_new, v_new, q_pos, m_hint, cfg, out, workspace, workspace_bytes, &a, &p);
    if (st != KF_OK) return st;
    const int64_t U = (int64_t)c->L * c->B * c->H;
    hipError_t e = kf::launch_decode(a, U, c->d, c->dtype, p.lds_bytes, (hipStream_t)stream);
    if (e == hipSuccess && a.shared) e = share_after_decode(c, a, (hipStream_t)stream);
    if (e != hipSuccess) return fail(KF_EDEVICE, "decode launch: %s", hipGetErrorString(e));
    g_err[0] = 0;
    return KF_OK;
}

kf_status kf_select_evict(kf_cache* c, int32_t k, int32_t w, int32_t layout, int32_t* kept_idx, void* workspace,
                          size_t workspace_bytes, void* stream) {
    kf::SelectArgs a;
    const kf_status st = prepare_select(c, k, w, layout, kept_idx, workspace, workspace_bytes, false, &a);
    if (st != KF_OK) return st;
    const int64_t U = (int64_t)c->L * c->B * c->H;
    const hipError_t e = kf::launch_select(a, U, (hipStream_t)stream);
    if (e != hipSuccess) return fail(KF_EDEVICE, "select launch: %s", hipGetErrorString(e));
    g_err[0] = 0;
    return KF_OK;
}

kf_status kf_beam_fork(kf_cache* c, const int32_t* parent, void* workspace, size_t workspace_bytes, void* stream) {
    kf_status st = check_cache(c);
    if (st != KF_OK) return st;
    if (!parent) return fail(KF_EINVAL, "parent is NULL");
    const WsLayout w = ws_layout(c, 0);
    st = check_ws(workspace, workspace_bytes, w.total);
    if (st != KF_OK) return st;
    kf::ForkArgs f;
    f.K = c->K;
    f.V = c->V;
    f.score = c->score;
    f.pos = c->pos;
    f.len = c->len;
    f.parent = parent;
    f.ws_err = (int32_t*)workspace + KF_WS_ERROR_WORD;
    f.L = c->L;
    f.B = c->B;
    f.H = c->H;
    f.cap = c->cap;
    f.row_bytes = c->d * (c->dtype == KF_F32 ? 4 : 2);
    const int64_t U = (int64_t)c->L * c->B * c->H;
    if ((U + 32767) / 32768 > 65535) return fail(KF_EUNSUPPORTED, "%lld units exceed the largest launch", (long long)U);
    const hipError_t e = kf::launch_fork(f, (hipStream_t)stream);
    if (e != hipSuccess) return fail(KF_EDEVICE, "fork launch: %s", hipGetErrorString(e));
    g_err[0] = 0;
    return KF_OK;
}

kf_status kf_select_evict_into(const kf_cache* src, kf_cache* dst, int32_t dst_layer0, int32_t k, int32_t w,
                               int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* stream) {
    kf_status st = check_cache(dst);
    if (st != KF_OK) return st;
    if (!src) return fail(KF_EINVAL, "source cache is NULL");
    if (src->B != dst->B || src->H != dst->H || src->d != dst->d || src->dtype != dst->dtype)
        return fail(KF_EINVAL, "source and destination must agree in B, H, d and dtype");
    if (dst_layer0 < 0 || dst_layer0 + src->L > dst->L)
        return fail(KF_EINVAL, "layers [%d, %d) do not fit the destination's %d layers", dst_layer0,
                    dst_layer0 + src->L, dst->L);
    if (k > dst->cap) return fail(KF_EINVAL, "budget k=%d exceeds the destination capacity %d", k, dst->cap);
    const char *s0 = (const char*)src->K, *d0 = (const char*)dst->K;
    if (s0 == d0 || src->V == dst->V || src->score == dst->score)
        return fail(KF_EINVAL, "source and destination must be different caches (use kf_select_evict in place)");
    kf::SelectArgs a;
    kf_cache src_mut = *src;  // the selection kernel only reads it in this mode
    st = prepare_select(&src_mut, k, w, KF_LAYOUT_ORDERED, kept_idx, workspace, workspace_bytes, false, &a);
    if (st != KF_OK) return st;
    a.move = 0;
    a.wide = 0;  // rows are gathered out of place by the launch below
    a.presel = 0;
    a.presel_done = 0;
    const int64_t U = (int64_t)src->L * src->B * src->H;
    hipError_t e = kf::launch_select(a, U, (hipStream_t)stream);
    if (e != hipSuccess) return fail(KF_EDEVICE, "select launch: %s", hipGetErrorString(e));
    kf::GatherArgs g;
    g.src_K = src->K;
    g.src_V = src->V;
    g.src_score = src->score;
    g.src_pos = src->pos;
    g.src_len = src->len;
    g.dst_K = dst->K;
    g.dst_V = dst->V;
    g.dst_score = dst->score;
    g.dst_pos = dst->pos;
    g.dst_len = dst->len;
    g.idx = a.idx;
    g.units = U;
    g.dst_unit0 = (int64_t)dst_layer0 * dst->B * dst->H;
    g.src_cap = src->cap;
    g.dst_cap = dst->cap;
    g.k = k;
    g.row_bytes = a.row_bytes;
    e = kf::launch_gather(g, (hipStream_t)stream);
    if (e != hipSuccess) return fail(KF_EDEVICE, "gather launch: %s", hipGetErrorString(e));
    g_err[0] = 0;
    return KF_OK;
}

// One generation step in one call.  With a schedule, the step number comes from device memory.
// `skipped`, if not NULL, takes the place of the workspace's error word; `clear_header` zeroes the
// workspace's first words by a kernel ahead of the step (a workspace whose contents are unknown).
static kf_status fused_step(kf_cache* c, const void* q, const void* k_new, const void* v_new, int32_t q_pos,
                            const kf_schedule* sched, int32_t* step, int32_t m_hint, const kf_score_cfg* cfg,
                            float* out, int32_t k, int32_t w, int32_t layout, int32_t* kept_idx, void* workspace,
                            size_t workspace_bytes, void* stream, int32_t* skipped = nullptr,
                            bool clear_header = false) {
    kf::DecodeArgs da;
    kf::DecodePlan p;
    kf_status st = prepare_decode(c, q, k_new, v_new, q_pos, m_hint, cfg, out, workspace, workspace_bytes, &da, &p);
    if (st != KF_OK) return st;
    kf::SelectArgs sa;
    st = prepare_select(c, k, w, layout, kept_idx, workspace, workspace_bytes, true, &sa);
    if (st != KF_OK) return st;
    if (skipped) da.ws_err = sa.ws_err = skipped;
    if (clear_header) {
        hipLaunchKernelGGL(clear_header_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (int32_t*)workspace);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return fail(KF_EDEVICE, "step launch: %s", hipGetErrorString(e0));
    }
    if (sched) {
        da.step = step;
        da.n0 = sched->n;
        da.T = sched->T;
        da.tau_init = sched->tau_init;
        da.dtau = (sched->tau_end - sched->tau_init) / (float)sched->T;  // as in kf_tau
        sa.step_inc = step;
    }
    const int64_t U = (int64_t)c->L * c->B * c->H;
    hipError_t e;
    if (da.S == 1 && layout == KF_LAYOUT_SLOT && !da.shared) {
        // one workgroup owns each unit and nothing orders the slots: the whole step is one launch
        da.fuse_k = k;
        da.fuse_w = w;
        da.fuse_idx = kept_idx;
        if (sched) da.step_inc = step;  // the launch's last workgroup moves the step number on
        e = kf::launch_decode(da, U, c->d, c->dtype, p.lds_bytes, (hipStream_t)stream);
    } else if (da.shared) {  // shared score: the layers' increments are added up between the merge and the selection
        e = kf::launch_decode(da, U, c->d, c->dtype, p.lds_bytes, (hipStream_t)stream);
        if (e == hipSuccess) e = share_after_decode(c, da, (hipStream_t)stream);
        if (e == hipSuccess) e = kf::launch_select(sa, U, (hipStream_t)stream);
    } else if (da.S > 1 && (int64_t)da.S * da.chunk <= kTailMergeMaxTokens && !sa.presel) {
        // few units in splits: the merge rides in the selection launch, whatever the number of query heads
        if (layout == KF_LAYOUT_SLOT || sa.wide) {
            // the merge has every final score in a register once: it also finds the smallest candidate, and the
            // selection part of the launch takes the evicted slot from there instead of reading the scores again
            da.pre_slices = sa.presel = 1;
            da.pre_k = k;
            da.pre_w = w;
            da.pre_layout = layout;
            da.pre_min = sa.ws_pmin;
            da.pre_slot = sa.ws_pslot;
            sa.presel_done = 1;
        }
        e = kf::launch_decode_split(da, U, c->d, c->dtype, p.lds_bytes, (hipStream_t)stream);
        if (e == hipSuccess) e = kf::launch_step_tail(da, sa, U, c->d, (hipStream_t)stream);
        if (e == hipSuccess && sa.wide) e = kf::launch_shift(sa, U, (hipStream_t)stream);  // few units: rows move in a launch of their own
    } else {  // one workgroup per unit (nothing to merge), or units too long to merge inside the selection
        if (da.S > 1 && sa.presel) {
            // few long units: the merge launch, which forms the final scores, also leaves what the selection's
            // candidate scan launch would look for -- one launch less (32 heads x 9.8k tokens: 47.8 -> 41 us per step)
            da.pre_slices = sa.presel = kf::decode_merge_slices(da.S, da.chunk);
            da.pre_k = k;
            da.pre_w = w;
            da.pre_layout = layout;
            da.pre_min = sa.ws_pmin;
            da.pre_slot = sa.ws_pslot;
            sa.presel_done = 1;
        }
        e = kf::launch_decode(da, U, c->d, c->dtype, p.lds_bytes, (hipStream_t)stream);
        if (e == hipSuccess) e = kf::launch_select(sa, U, (hipStream_t)stream);
    }
    if (e != hipSuccess) return fail(KF_EDEVICE, "step launch: %s", hipGetErrorString(e));
    g_err[0] = 0;
    return KF_OK;
}

kf_status kf_decode_select_step(kf_cache* c, const void* q, const void* k_new, const void* v_new, int32_t q_pos,
                                int32_t m_hint, const kf_score_cfg* cfg, float* out, int32_t k, int32_t w,
                                int32_t layout, int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                                void* stream) {
    return fused_step(c, q, k_new, v_new, q_pos, nullptr, nullptr, m_hint, cfg, out, k, w, layout, kept_idx,
                      workspace, workspace_bytes, stream);
}

kf_status kf_decode_select_step_noalloc(kf_cache* c, const void* q, const void* k_new, const void* v_new,
                                        int32_t q_pos, int32_t m_hint, const kf_score_cfg* cfg, float* out, int32_t k,
                                        int32_t w, int32_t layout, int32_t* kept_idx, int32_t* skipped, void* stream) {
    kf_status st = check_cache(c);
    if (st != KF_OK) return st;
    const size_t need = ws_layout(c, 0).total;
    if (need > (size_t)KF_NOALLOC_SCRATCH_BYTES)
        return fail(KF_EWORKSPACE,
                    "a step on this cache needs %zu bytes of scratch, the built-in buffer holds %zu: use "
                    "kf_decode_select_step with a workspace of the caller's",
                    need, (size_t)KF_NOALLOC_SCRATCH_BYTES);
    void* ptr = nullptr;
    st = scratch_of_current_device(&ptr);
    if (st != KF_OK) return st;
    return fused_step(c, q, k_new, v_new, q_pos, nullptr, nullptr, m_hint, cfg, out, k, w, layout, kept_idx, ptr,
                      (size_t)KF_NOALLOC_SCRATCH_BYTES, stream, skipped, true);
}

kf_status kf_decode_select_step_at(kf_cache* c, const void* q, const void* k_new, const void* v_new,
                                   const kf_schedule* sched, int32_t* step, int32_t m_hint, const kf_score_cfg* cfg,
                                   float* out, int32_t k, int32_t w, int32_t layout, int32_t* kept_idx,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    if (!sched || !step) return fail(KF_EINVAL, "sched and step must not be NULL");
    if (sched->n < 0 || sched->T < 1) return fail(KF_EINVAL, "schedule needs n >= 0 and T >= 1");
    if (!(sched->tau_init > 0.0f) || !(sched->tau_end > 0.0f) || !isfinite(sched->tau_init) ||
        !isfinite(sched->tau_end))
        return fail(KF_EINVAL, "schedule temperatures must be finite and positive");
    if (!cfg) return fail(KF_EINVAL, "score configuration is NULL");
    kf_score_cfg cfg2 = *cfg;
    cfg2.tau = sched->tau_init;  // ignored by the kernels; keeps the common validation meaningful
    return fused_step(c, q, k_new, v_new, 0, sched, step, m_hint, &cfg2, out, k, w, layout, kept_idx, workspace,
                      workspace_bytes, stream);
}

}  // extern "C"
