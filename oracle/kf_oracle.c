/*
 * Keyformer CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, double-precision implementation of the Keyformer decode hot
 * path, written from the paper (arXiv 2403.09054) alone.  It exists so that
 * the GPU library can be checked against something that can be read against
 * the paper by eye.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the GPU library never does, and the two share
 * no code.
 *
 * What is computed (paper passages in brackets):
 *   kfo_tau            temperature schedule                       [Eq. 12, Alg. 1]
 *   kfo_noise_bits     counter-based hash -> 32 random bits       [ours; the paper
 *                      only says the noise follows a Gumbel distribution]
 *   kfo_gumbel         standard Gumbel variate from those bits    [Eq. 7]
 *   kfo_prefill_score  prompt-phase score: column sums of the
 *                      row-wise softmax of the perturbed causal
 *                      logits                                     [Sec. 3.4, Alg. 1 prompt branch, Eq. 4, Eq. 11]
 *   kfo_decode_step    append the new token, attention over the
 *                      reduced cache, score accumulation          [Eq. 1, Eq. 11, Sec. 3.3.2, Alg. 1 else-branch]
 *   kfo_select_evict   recent window + top-(k-w) key tokens,
 *                      order-preserving compaction                [Alg. 1 last three lines, Sec. 3.4]
 *   (shared != 0 in the two scoring calls: the "Shared" score function of the
 *    ablation -- one f for all layers, each layer's increments added to it)  [Sec. 4.4.1]
 *   (G > 1 in the two scoring calls: grouped-query / multi-query attention, which
 *    the paper says the method applies to unchanged -- G query heads read one
 *    cached head and its f takes the sum of their increments)               [Sec. 6]
 *
 * All arithmetic is done in double on the exact input bits (fp32, or bf16 /
 * IEEE half given as 16-bit words).  State that persists between steps (the
 * accumulated score f) is stored as fp32, the new value being
 * (float)((double)f + delta).
 *
 * Pins: every function here is pinned by tests/test_oracle_*.py against
 * closed forms, limits, invariants and brute force.  The specific noise VALUES
 * (the hash) are fixed by our written spec, not by the paper: "parity unpinned"
 * by the paper for those; they are pinned in distribution only (mean, std,
 * Kolmogorov-Smirnov against Eq. 7's CDF, Gumbel-max frequencies).
 *
 * Layout of a cache (host memory, same logical layout the GPU library uses):
 *   K, V   [U][cap][d]   fp32 or bf16 bits      U = L*B*H, unit u = (l*B + b)*H + h
 *   score  [U][cap]      fp32, accumulated f
 *   pos    [U][cap]      int32, original token position, ascending in [0,len)
 *   len    [U]           int32
 * layer0 is the model-wide index of the cache's first layer (it only enters
 * the noise key), so that a cache holding a subset of the layers draws the
 * same noise as the full one.  head0 is the same for heads: cached head hk of
 * the cache is the model's cached head head0 + hk (noise key and slope index),
 * so that one (layer, sequence, head) unit of a large model can be computed
 * by itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KFO_F32 0
#define KFO_BF16 1
#define KFO_F16 2

#define KFO_NOISE_NONE 0
#define KFO_NOISE_GUMBEL 1
#define KFO_NOISE_GAUSSIAN 2
#define KFO_NOISE_CONSTANT 3

/* mean and standard deviation the paper prints for the standard Gumbel pdf,
 * reused by its Gaussian and constant ablations [Sec. 4.4.3] */
#define KFO_GUMBEL_MEAN 0.5772
#define KFO_GUMBEL_STD 1.2825

/* ------------------------------------------------------------------ */
/* element access                                                      */
/* ------------------------------------------------------------------ */
static double load_elem(const void *base, int dtype, size_t idx)
{
    if (dtype == KFO_F32)
        return (double)((const float *)base)[idx];
    if (dtype == KFO_F16) {
        /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        uint16_t hbits = ((const uint16_t *)base)[idx];
        int sign = hbits >> 15, e = (hbits >> 10) & 31, frac = hbits & 1023;
        double v;
        if (e == 0) v = ldexp((double)frac, -24);                   /* zero and subnormals */
        else if (e == 31) v = frac ? NAN : INFINITY;
        else v = ldexp(1.0 + (double)frac / 1024.0, e - 15);
        return sign ? -v : v;
    }
    /* bf16: the upper 16 bits of an fp32 */
    uint32_t w = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &w, 4);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == KFO_F32 ? 4 : 2; }

/* ------------------------------------------------------------------ */
/* tau schedule  [Eq. 12]: tau_t = tau_init + t * (tau_end - tau_init)/T */
/* t = 0 is the prompt iteration, t = 1..T are the decode steps.        */
/* Evaluated in fp32 so that a caller can hand identical bits to any    */
/* implementation.                                                      */
/* ------------------------------------------------------------------ */
float kfo_tau(int t, int T, float tau_init, float tau_end)
{
    float dtau = (tau_end - tau_init) / (float)T;
    return tau_init + (float)t * dtau;
}

/* ------------------------------------------------------------------ */
/* noise: counter-based hash of (seed, layer, head, q_pos, k_pos)       */
/* ------------------------------------------------------------------ */
static uint64_t mix64(uint64_t z)
{
    z ^= z >> 32;
    z *= 0x6A09E667F3BCC909ULL;
    z ^= z >> 29;
    z *= 0xBB67AE8584CAA73BULL;
    z ^= z >> 32;
    return z;
}

static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

uint32_t kfo_noise_bits(uint64_t seed, uint32_t layer, uint32_t head,
                        uint32_t q_pos, uint32_t k_pos)
{
    uint64_t ukey = mix64(mix64(seed + 0x9E3779B97F4A7C15ULL) + (((uint64_t)layer << 32) | (uint64_t)head));
    uint32_t ka = (uint32_t)ukey;
    uint32_t kb = (uint32_t)(ukey >> 32);
    uint32_t r = mix32(mix32(ka ^ (q_pos * 0x9E3779B9u)) + kb);
    return mix32(r ^ (k_pos * 0x243F6A89u));
}

/* uniform in (0,1) on a 2^-23 grid, never 0 or 1 */
static double bits_to_uniform(uint32_t bits)
{
    return (2.0 * (double)(bits >> 9) + 1.0) / 16777216.0;
}

/* standard Gumbel variate: pdf exp(-z - exp(-z))  [Eq. 7], i.e. the inverse
 * of the CDF exp(-exp(-z)) applied to a uniform */
double kfo_gumbel(uint32_t bits)
{
    double u = bits_to_uniform(bits);
    return -log(-log(u));
}

/* The logit adjustment zeta of Eq. 4 for one (query, key) pair. */
static double zeta(int noise, uint64_t seed, uint32_t layer, uint32_t head,
                   uint32_t q_pos, uint32_t k_pos)
{
    switch (noise) {
    case KFO_NOISE_GUMBEL:
        return kfo_gumbel(kfo_noise_bits(seed, layer, head, q_pos, k_pos));
    case KFO_NOISE_CONSTANT: /* y = x + c, c = 0.5772  [Sec. 4.4.3] */
        return KFO_GUMBEL_MEAN;
    case KFO_NOISE_GAUSSIAN: { /* Eq. 5 with the Gumbel's mean and std */
        /* two independent uniforms: the pair's hash, and the hash of that
         * hash's complement position (k_pos with the top bit set) */
        double u1 = bits_to_uniform(kfo_noise_bits(seed, layer, head, q_pos, k_pos));
        double u2 = bits_to_uniform(kfo_noise_bits(seed, layer, head, q_pos, k_pos ^ 0x80000000u));
        double g = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
        return KFO_GUMBEL_MEAN + KFO_GUMBEL_STD * g;
    }
    default:
        return 0.0;
    }
}

double kfo_zeta(int noise, uint64_t seed, uint32_t layer, uint32_t head,
                uint32_t q_pos, uint32_t k_pos)
{
    return zeta(noise, seed, layer, head, q_pos, k_pos);
}

/* ------------------------------------------------------------------ */
/* softmax of a vector, the textbook way: subtract the max, exponentiate, */
/* divide by the sum.                                                   */
/* ------------------------------------------------------------------ */
static void softmax_inplace(double *v, int m)
{
    double mx = v[0];
    for (int j = 1; j < m; ++j)
        if (v[j] > mx) mx = v[j];
    double s = 0.0;
    for (int j = 0; j < m; ++j) {
        v[j] = exp(v[j] - mx);
        s += v[j];
    }
    for (int j = 0; j < m; ++j)
        v[j] /= s;
}

/* ------------------------------------------------------------------ */
/* Prompt-phase scoring  [Sec. 3.4; Alg. 1 prompt branch]               */
/*   x_ij = scale*<q_i,k_j> - slope_h*(i-j)      for j <= i (causal)     */
/*   y_ij = (x_ij + zeta_ij)/tau                                         */
/*   z_i  = softmax_j(y_i.)                                              */
/*   f[j] = sum_{i>=j} z_ij ;  pos[j] = j ; len = n                       */
/* Q is [U*G][n][d]; K is the cache's K, [U][cap][d], rows 0..n-1 filled. */
/* G > 1: grouped-query attention [Sec. 6]: the cache's head h serves the   */
/* query heads h*G .. h*G+G-1 (each with its own slope and noise stream);   */
/* its f is the sum of their column sums.                                  */
/* ------------------------------------------------------------------ */
int kfo_prefill_score(const void *Q, const void *K, float *score, int32_t *pos,
                      int32_t *len, int L, int B, int H, int d, int cap,
                      int dtype, int layer0, int head0, int n, float tau, float scale, int noise,
                      const uint64_t *seeds, const float *slopes, int shared, int G)
{
    if (n < 1 || n > cap || !(tau > 0.0f) || G < 1) return -1;
    int U = L * B * H;
    /* "Shared" score function [Sec. 4.4.1]: every layer's column sums, kept in
     * double until the layers have been added up */
    double *fall = NULL;
    if (shared) {
        fall = (double *)calloc((size_t)U * n, sizeof(double));
        if (!fall) return -2;
    }
    for (int u = 0; u < U; ++u) {
        int hk = u % H, b = (u / H) % B, l = layer0 + u / (H * B);
        uint64_t seed = seeds ? seeds[b] : 0;
        double *q = (double *)malloc((size_t)n * d * sizeof(double));
        double *kk = (double *)malloc((size_t)n * d * sizeof(double));
        double *f = (double *)calloc((size_t)n, sizeof(double));
        if (!q || !kk || !f) { free(q); free(kk); free(f); free(fall); return -2; }
        for (size_t e = 0; e < (size_t)n * d; ++e)
            kk[e] = load_elem(K, dtype, (size_t)u * cap * d + e);
        int failed = 0;
        for (int g = 0; g < G; ++g) {
            int h = (head0 + hk) * G + g;              /* the query head */
            double slope = slopes ? (double)slopes[h] : 0.0;
            for (size_t e = 0; e < (size_t)n * d; ++e)
                q[e] = load_elem(Q, dtype, ((size_t)u * G + g) * n * d + e);
#pragma omp parallel
            {
                double *fl = (double *)calloc((size_t)n, sizeof(double));
                double *row = (double *)malloc((size_t)n * sizeof(double));
                int ok = fl && row;
                if (!ok) {
#pragma omp atomic write
                    failed = 1;
                }
#pragma omp for schedule(dynamic, 8)
                for (int i = 0; i < n; ++i) {
                    if (!ok) continue;
                    for (int j = 0; j <= i; ++j) {
                        double dot = 0.0;
                        for (int c = 0; c < d; ++c)
                            dot += q[(size_t)i * d + c] * kk[(size_t)j * d + c];
                        double x = (double)scale * dot - slope * (double)(i - j);
                        double z = zeta(noise, seed, (uint32_t)l, (uint32_t)h,
                                        (uint32_t)i, (uint32_t)j);
                        row[j] = (x + z) / (double)tau;
                    }
                    softmax_inplace(row, i + 1);
                    for (int j = 0; j <= i; ++j)
                        fl[j] += row[j];
                }
                /* add the threads' column sums one thread at a time */
                if (ok) {
#pragma omp critical
                    for (int j = 0; j < n; ++j)
                        f[j] += fl[j];
                }
                free(fl);
                free(row);
            }
        }
        if (failed) { free(q); free(kk); free(f); free(fall); return -2; }
        for (int j = 0; j < n; ++j) {
            if (shared) fall[(size_t)u * n + j] = f[j];
            else score[(size_t)u * cap + j] = (float)f[j];
            pos[(size_t)u * cap + j] = j;
        }
        len[u] = n;
        free(q);
        free(kk);
        free(f);
    }
    if (shared) {
        /* one score function for all layers: f[j] = sum over layers of that layer's
         * column sum; every layer's cache carries the same copy */
        int BH = B * H;
        for (int bh = 0; bh < BH; ++bh)
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int l = 0; l < L; ++l)
                    s += fall[((size_t)l * BH + bh) * n + j];
                for (int l = 0; l < L; ++l)
                    score[((size_t)l * BH + bh) * cap + j] = (float)s;
            }
        free(fall);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* One decode step  [Alg. 1 else-branch; Eq. 1; Eq. 11; Sec. 3.3.2]      */
/*   append (k_new, v_new) with pos = q_pos and f = 0;  m = len          */
/*   x_j = scale*<q,K_j> - slope_h*(q_pos - pos_j)                       */
/*   attention: p = softmax(x),          out = sum_j p_j V_j             */
/*   score:     df = softmax((x+zeta)/tau),  f_j += df_j  for all j < m  */
/* k_new, v_new are [U][d]; q is [U*G][d]; out is [U*G][d] fp32.         */
/* G > 1: grouped-query attention [Sec. 6]: the cache's head h serves the */
/* query heads h*G .. h*G+G-1, each with its own logits, attention output, */
/* slope and noise stream; f takes the sum of their increments (the heads  */
/* share the cached tokens, so they share the decision what to keep).     */
/* q_pos_seq, tau_seq (may be NULL): [B] per-sequence query position and    */
/* temperature, replacing the scalars q_pos and tau.                       */
/* Optional debug outputs (may be NULL): dbg_p, dbg_df [U*G][cap] doubles. */
/* ------------------------------------------------------------------ */
int kfo_decode_step(void *K, void *V, float *score, int32_t *pos, int32_t *len,
                    int L, int B, int H, int d, int cap, int dtype, int layer0, int head0,
                    const void *q, const void *k_new, const void *v_new,
                    int32_t q_pos, float tau, float scale, int noise,
                    const uint64_t *seeds, const float *slopes, int new_pos, int shared,
                    int G, const int32_t *q_pos_seq, const float *tau_seq,
                    float *out, double *dbg_p, double *dbg_df)
{
    if (!(tau > 0.0f) || G < 1) return -1;
    if (tau_seq)
        for (int b = 0; b < B; ++b)
            if (!(tau_seq[b] > 0.0f)) return -1;
    int U = L * B * H;
    size_t es = elem_size(dtype);
    for (int u = 0; u < U; ++u)
        if (len[u] < 0 || len[u] >= cap) return -1;
    /* "Shared" score function [Sec. 4.4.1]: all layers hold the same tokens (same
     * scores, hence the same evictions), and every layer's increment of this step
     * is added to the one score */
    double *dfall = NULL;
    if (shared) {
        for (int u = 0; u < U; ++u) {
            int u0 = u % (B * H);
            if (len[u] != len[u0]) return -1;
            for (int j = 0; j < len[u]; ++j)
                if (pos[(size_t)u * cap + j] != pos[(size_t)u0 * cap + j]) return -1;
        }
        dfall = (double *)calloc((size_t)U * cap, sizeof(double));
        if (!dfall) return -2;
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u) {
        int hk = u % H, b = (u / H) % B, l = layer0 + u / (H * B);
        uint64_t seed = seeds ? seeds[b] : 0;
        /* a batch whose sequences are at different points of their generation: each
         * has its own query position and its own temperature tau_t  [Eq. 12 per sequence] */
        int32_t q_pos_u = q_pos_seq ? q_pos_seq[b] : q_pos;
        double tau_u = tau_seq ? (double)tau_seq[b] : (double)tau;
        char *Ku = (char *)K + (size_t)u * cap * d * es;
        char *Vu = (char *)V + (size_t)u * cap * d * es;
        float *fu = score + (size_t)u * cap;
        int32_t *pu = pos + (size_t)u * cap;

        /* append */
        int slot = len[u];
        memcpy(Ku + (size_t)slot * d * es, (const char *)k_new + (size_t)u * d * es, d * es);
        memcpy(Vu + (size_t)slot * d * es, (const char *)v_new + (size_t)u * d * es, d * es);
        pu[slot] = q_pos_u;
        fu[slot] = 0.0f;
        int m = slot + 1;
        len[u] = m;

        double *p = (double *)malloc((size_t)m * sizeof(double));
        double *y = (double *)malloc((size_t)m * sizeof(double));
        double *df = (double *)calloc((size_t)m, sizeof(double));
        if (!p || !y || !df) {
            free(p); free(y); free(df);
#pragma omp atomic write
            failed = 1;
            continue;
        }
        for (int g = 0; g < G; ++g) {
            int h = (head0 + hk) * G + g;              /* the query head */
            size_t uq = (size_t)u * G + g;
            double slope = slopes ? (double)slopes[h] : 0.0;
            for (int j = 0; j < m; ++j) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += load_elem(q, dtype, uq * d + c) *
                           load_elem(Ku, dtype, (size_t)j * d + c);
                /* distance behind the position bias: original positions ("Org Pos"), or -- the
                 * paper's "New Pos" ablation, Sec. 4.4.2 -- positions within the reduced cache,
                 * where the query sits at slot m-1 and key j at slot j */
                double dist = new_pos ? (double)(m - 1 - j) : (double)(q_pos_u - pu[j]);
                double x = (double)scale * dot - slope * dist;
                p[j] = x;
                y[j] = (x + zeta(noise, seed, (uint32_t)l, (uint32_t)h,
                                 (uint32_t)q_pos_u, (uint32_t)pu[j])) / tau_u;
            }
            softmax_inplace(p, m); /* attention probabilities: clean logits */
            softmax_inplace(y, m); /* score increment: perturbed, tempered logits */
            for (int c = 0; c < d; ++c) {
                double o = 0.0;
                for (int j = 0; j < m; ++j)
                    o += p[j] * load_elem(Vu, dtype, (size_t)j * d + c);
                out[uq * d + c] = (float)o;
            }
            for (int j = 0; j < m; ++j) {
                df[j] += y[j];
                if (dbg_p) dbg_p[uq * cap + j] = p[j];
                if (dbg_df) dbg_df[uq * cap + j] = y[j];
            }
        }
        for (int j = 0; j < m; ++j) {
            if (shared) dfall[(size_t)u * cap + j] = df[j];
            else fu[j] = (float)((double)fu[j] + df[j]);
        }
        free(p);
        free(y);
        free(df);
    }
    if (shared && !failed) {
        int BH = B * H;
        for (int bh = 0; bh < BH; ++bh) {
            int m = len[bh];
            for (int j = 0; j < m; ++j) {
                double s = 0.0;
                for (int l = 0; l < L; ++l)
                    s += dfall[((size_t)l * BH + bh) * cap + j];
                for (int l = 0; l < L; ++l) {
                    float *f = score + ((size_t)l * BH + bh) * cap + j;
                    *f = (float)((double)*f + s);
                }
            }
        }
    }
    free(dfall);
    return failed ? -2 : 0;
}

/* ------------------------------------------------------------------ */
/* Selection and compaction  [Alg. 1: S_w, S_key, S_k; Sec. 3.4]        */
/*   units with len <= k are left alone; otherwise                       */
/*   S_w   = slots [len-w, len)                                          */
/*   S_key = the (k-w) slots of [0, len-w) with the largest f, equal f   */
/*           resolved in favour of the lower slot (the older token)      */
/*   the survivors keep their relative order; len = k                    */
/* kept_idx (may be NULL) is [U][k]: pre-compaction slot of each survivor */
/* (identity for untouched units, entries >= len set to -1).             */
/* ------------------------------------------------------------------ */
typedef struct {
    float f;
    int32_t idx;
} cand_t;

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->f > y->f) return -1; /* larger score first */
    if (x->f < y->f) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx); /* then lower slot first */
}

static int int_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int kfo_select_evict(void *K, void *V, float *score, int32_t *pos, int32_t *len,
                     int L, int B, int H, int d, int cap, int dtype, int k, int w,
                     int32_t *kept_idx)
{
    if (k < 1 || w < 0 || w > k || k > cap) return -1;
    int U = L * B * H;
    size_t es = elem_size(dtype);
    size_t rb = (size_t)d * es;
    for (int u = 0; u < U; ++u)
        if (len[u] < 0 || len[u] > cap) return -1;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < U; ++u) {
        char *Ku = (char *)K + (size_t)u * cap * rb;
        char *Vu = (char *)V + (size_t)u * cap * rb;
        float *fu = score + (size_t)u * cap;
        int32_t *pu = pos + (size_t)u * cap;
        int n = len[u];
        if (n <= k) {
            if (kept_idx)
                for (int i = 0; i < k; ++i)
                    kept_idx[(size_t)u * k + i] = i < n ? i : -1;
            continue;
        }
        int ncand = n - w, nkey = k - w;
        cand_t *c = (cand_t *)malloc((size_t)(ncand > 0 ? ncand : 1) * sizeof(cand_t));
        int32_t *keep = (int32_t *)malloc((size_t)k * sizeof(int32_t));
        if (!c || !keep) {
            free(c); free(keep);
#pragma omp atomic write
            failed = 1;
            continue;
        }
        for (int j = 0; j < ncand; ++j) {
            c[j].f = fu[j];
            c[j].idx = j;
        }
        qsort(c, (size_t)ncand, sizeof(cand_t), cand_cmp);
        for (int i = 0; i < nkey; ++i)
            keep[i] = c[i].idx;
        qsort(keep, (size_t)nkey, sizeof(int32_t), int_cmp);
        for (int i = 0; i < w; ++i)
            keep[nkey + i] = n - w + i;
        /* survivors move to the front, in order; keep[i] >= i so a forward
         * walk never overwrites a row it still has to read */
        for (int i = 0; i < k; ++i) {
            int s = keep[i];
            if (s != i) {
                memmove(Ku + (size_t)i * rb, Ku + (size_t)s * rb, rb);
                memmove(Vu + (size_t)i * rb, Vu + (size_t)s * rb, rb);
                fu[i] = fu[s];
                pu[i] = pu[s];
            }
            if (kept_idx) kept_idx[(size_t)u * k + i] = s;
        }
        len[u] = k;
        free(c);
        free(keep);
    }
    return failed ? -2 : 0;
}
