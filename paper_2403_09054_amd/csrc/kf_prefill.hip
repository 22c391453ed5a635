// Prompt-phase scoring of Keyformer for gfx950 (Sec. 3.4, Algorithm 1 prompt
// branch): for every unit
//     x_ij = scale*<Q_i,K_j> - slope*(i-j),  j <= i
//     z_i  = softmax_j((x_ij + zeta_ij)/tau)                 (Eq. 4, Eq. 11)
//     f[j] = sum_{i>=j} z_ij
// The logits are a dense n x n contraction: they are produced 32x32 tiles at a
// time on the matrix cores (MFMA).  The normaliser of row i must be known before
// any z_ij can be summed down a column, so two passes are made, each
// re-computing the logits instead of storing n^2 values:
//   pass 1  (row statistics)  computes the transposed tile K_tile * Q_tile^T so
//           that a lane owns ONE query and sees 16 of the tile's 32 keys: the
//           running max / sum of the row stay in the lane's registers.  Result:
//           c_i = log2(sum_j 2^(y2_ij)), y2 = log2(e)*(x+zeta)/tau, and the
//           row's noise key.
//   pass 2  (column sums)     computes Q_tile * K_tile^T so that a lane owns ONE
//           key and sees 16 of the tile's 32 queries: z_ij = 2^(y2_ij - c_i) is
//           added into the lane's column sum.
// Per logit the work is one 32-bit hash, two logarithms and one exponential;
// that, not the MFMA rate, bounds the kernel, so the per-logit instruction count
// is what is trimmed.  With the Gumbel adjustment (the method; the other
// adjustments keep the plain form): pass 1 sums every term against a reference
// exponent instead of searching each tile's maximum first -- the reference
// starts at the row's own diagonal term (so the sum cannot vanish), follows the
// sum's exponent upwards tile by tile, and a tile whose sum overflows is summed
// again against a higher reference; pass 1 leaves the row normaliser already
// combined with the adjustment's constant part; kernels built for "no position
// bias" drop that term.
#include "kf_device.h"
#include "kf_internal.h"

namespace kf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kPrefillThreads = 256;  // 4 waves, 32 queries (pass 1) or keys (pass 2) each
constexpr int kTile = 32;

// One "group" = the 16 bytes a lane loads from a row: it feeds one bf16 MFMA
// (K = 16: 8 elements from each half of the wave) or four fp32 MFMAs (K = 2).
// Both operands use the same assignment of k indices to (wave half, element),
// so the contraction runs over every k exactly once.
template <typename T>
struct Mma;
template <>
struct Mma<bf16_t> {
    static __device__ __forceinline__ f32x16 group(const uint4& a, const uint4& b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
template <>
struct Mma<f16_t> {
    static __device__ __forceinline__ f32x16 group(const uint4& a, const uint4& b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<float> {
    static __device__ __forceinline__ f32x16 group(const uint4& a, const uint4& b, f32x16 c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
        return c;
    }
};

// Workgroup -> (unit, block of 128 rows).  Consecutive workgroup ids are dealt
// round-robin to the chip's 8 XCDs, each with an L2 of its own; the blocks of
// one unit re-read the same K / Q rows, so all blocks of a unit are given ids
// that are equal modulo 8 and therefore share one L2.
constexpr int kXcds = 8;
__device__ __forceinline__ void unit_and_block(int nblk, int64_t& u, int& blk) {
    const unsigned xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    u = (int64_t)(local / nblk) * kXcds + xcd;
    blk = (int)(local % nblk);
}

// Row of the 32x32 accumulator tile that register r of this lane holds
// (the column is lane % 32).
__device__ __forceinline__ int acc_row(int r, int half) { return (r >> 2) * 8 + half * 4 + (r & 3); }

// y2 = log2(e) * (x + zeta)/tau for one logit, x = scale*acc - slope*dist.
// Gumbel (the method's adjustment) is the fast path: one hash, two hardware
// logarithms; zeta*log2(e) = -(log2(t) + log2(ln 2)) with t = -log2(u).
struct LogitParams {
    float sc1;      // scale * log2(e) / tau
    float slope1;   // slope * log2(e) / tau
    float inv_tau;
    float gz;       // -log2(ln 2) / tau : the constant part of the Gumbel term
    float c1;       // log2(e) / tau
    int noise;
};
__device__ __forceinline__ float logit2_gumbel(const LogitParams& lp, float acc, float dist, uint32_t hash_in) {
    const float l2t = hw_log2(neg_log2_uniform(mix32(hash_in)));
    return fmaf(acc, lp.sc1, fmaf(dist, -lp.slope1, fmaf(l2t, -lp.inv_tau, lp.gz)));
}
__device__ __forceinline__ float logit2_other(const LogitParams& lp, float acc, float dist, uint32_t rkey,
                                              uint32_t k_pos) {
    return fmaf(acc, lp.sc1, fmaf(dist, -lp.slope1, zeta_log2e(lp.noise, rkey, k_pos) * lp.inv_tau));
}

// ------------------------------------------------------------------ streamed tiles through LDS
// The four waves of a workgroup work on four 32-row groups of the SAME 128-row
// block and walk the same sequence of 32-row tiles of the other operand.  That
// tile is fetched once per workgroup (each thread a few 16-byte pieces, fully
// coalesced), parked in LDS and read from there as MFMA operands -- a quarter of
// the L2 traffic and D/4 fewer registers per lane than every wave loading its
// own copy, which is what lets more than two waves per SIMD overlap the MFMAs
// of one with the transcendental epilogue of another.  Two buffers; one
// barrier per tile.  Rows are padded by 16 bytes so that the 32 rows a wave
// reads in one instruction spread over the banks.
template <typename T, int D>
struct TileStage {
    static constexpr int kRowBytes = D * (int)sizeof(T);
    static constexpr int kPitch = kRowBytes + 16;                 // bytes between rows in LDS
    static constexpr int kPieces = kTile * kRowBytes / 16;        // 16-byte pieces of a tile
    static constexpr int NP = kPieces / kPrefillThreads;          // pieces per thread (1, 2 or 4)
    static constexpr int PPR = kRowBytes / 16;                    // pieces per row
    static constexpr int kBufBytes = kTile * kPitch;
    static_assert(kPieces % kPrefillThreads == 0, "a tile is a whole number of pieces per thread");

    // rows [row0, row0+32) of `rows` (clamped to n-1) -> registers
    static __device__ __forceinline__ void fetch(const T* rows, int row0, int n, uint4 (&reg)[NP]) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int p = threadIdx.x + i * kPrefillThreads;
            const int r = min(row0 + p / PPR, n - 1);
            reg[i] = *(const uint4*)((const char*)rows + (size_t)r * kRowBytes + (p % PPR) * 16);
        }
    }
    static __device__ __forceinline__ void park(char* buf, const uint4 (&reg)[NP]) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int p = threadIdx.x + i * kPrefillThreads;
            *(uint4*)(buf + (p / PPR) * kPitch + (p % PPR) * 16) = reg[i];
        }
    }
    // the 16 bytes lane (row n0, half) feeds MFMA group g
    static __device__ __forceinline__ uint4 operand(const char* buf, int n0, int half, int g) {
        return *(const uint4*)(buf + n0 * kPitch + (2 * g + half) * 16);
    }
};

// ------------------------------------------------------------------ pass 1
// <q, k> over the elements of the 16-byte pieces a and b
template <typename T>
__device__ __forceinline__ float dot_piece(const uint4& x, const uint4& y) {
    constexpr int EPV = ElemTraits<T>::kPerVec;
    float xf[EPV], yf[EPV];
    unpack16<T>(x, xf);
    unpack16<T>(y, yf);
    float d = 0.0f;
#pragma unroll
    for (int e = 0; e < EPV; ++e) d = fmaf(xf[e], yf[e], d);
    return d;
}

// Sum over this lane's 16 logits of a tile of 2^(y2 - reference), Gumbel adjustment; `base` is the
// adjustment's constant part less the reference (and the position bias of the lane's first key).  MASK: keep only the keys up to `room` places behind the
// lane's first one (the tile crosses the diagonal).
template <bool BIAS, bool MASK>
__device__ __forceinline__ float tile_sum(const LogitParams& lp, const f32x16& acc, float base, uint32_t rkey,
                                          uint32_t kmul, int room) {
    float ssum = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ro = (r >> 2) * 8 + (r & 3);
        const float l2t = hw_log2(neg_log2_uniform(mix32(rkey ^ (kmul + (uint32_t)ro * kKposMul))));
        // position bias -slope*(dist0 - ro): its dist0 part rides in `base`, the ro part is a literal multiple
        const float t = fmaf(l2t, -lp.inv_tau, BIAS ? fmaf(lp.slope1, (float)ro, base) : base);
        const float e = hw_exp2(fmaf(acc[r], lp.sc1, t));
        ssum += (!MASK || ro <= room) ? e : 0.0f;
    }
    return ssum;
}

// GUMBEL: the method's adjustment, trimmed form; otherwise any adjustment, plain form.  BIAS: slopes given.
template <typename T, int D, bool GUMBEL, bool BIAS>
__global__ void __launch_bounds__(kPrefillThreads) prefill_rowstats_kernel(const PrefillArgs a, int nblk, int64_t units) {
    constexpr int EPV = ElemTraits<T>::kPerVec;
    constexpr int NG = D / (2 * EPV);
    using Stage = TileStage<T, D>;
    __shared__ __attribute__((aligned(16))) char kbuf[2][Stage::kBufBytes];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n0 = lane & 31, half = lane >> 5;
    int64_t u;
    int blk;
    unit_and_block(nblk, u, blk);
    if (u >= units) return;  // workgroup-uniform
    const int rb = nblk - 1 - blk;  // longest rows first
    const int h = (int)(u % a.H), b = (int)((u / a.H) % a.B), l = a.layer0 + (int)(u / ((int64_t)a.H * a.B));
    const int n = a.seq_n ? a.seq_n[b] : a.n;  // this sequence's prompt length; rows n..a.n-1 are padding
    // workgroup-uniform exits: a length out of range (the second pass reports it), a block inside the padding
    if (n < 1 || n > a.n || rb * (4 * kTile) >= n) return;
    const int i0 = rb * (4 * kTile) + wv * kTile;
    const bool active = i0 < n;  // wave-uniform; inactive waves still fetch tiles and meet the barriers
    const int i = i0 + n0;
    const T* Qu = (const T*)a.Q + (size_t)u * a.n * D;
    const T* Ku = (const T*)a.K + (size_t)(u / a.G) * a.cap * D;  // G query heads read one cached head

    uint4 bq[NG];
    {
        const T* row = Qu + (size_t)min(i, n - 1) * D + half * EPV;
#pragma unroll
        for (int g = 0; g < NG; ++g) bq[g] = *(const uint4*)(row + g * 2 * EPV);
    }
    const bool rnd = (a.noise == kNoiseGumbel || a.noise == kNoiseGaussian);
    const uint32_t rkey = rnd ? row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)h), (uint32_t)i) : 0u;
    LogitParams lp;
    lp.c1 = a.inv_tau * kLog2e;
    lp.sc1 = a.scale * lp.c1;
    lp.slope1 = (BIAS ? a.slopes[h] : 0.0f) * lp.c1;
    lp.inv_tau = a.inv_tau;
    lp.gz = -kLog2Ln2 * a.inv_tau;
    lp.noise = a.noise;
    // key position of accumulator register r is jb + half*4 + (r>>2)*8 + (r&3); its hash input
    // is rkey ^ (k_pos * kKposMul): the lane part of the product is formed once
    const uint32_t kmul_lane = (uint32_t)(half * 4) * kKposMul;

    float M = -INFINITY, Ssum = 0.0f;
    if constexpr (GUMBEL) {
        // Reference exponent of the row's sum: its own diagonal term y2_ii, formed here from the query's and the
        // key's elements this lane holds (both halves of the wave added up).  It is a term of the sum, so the
        // sum against it cannot vanish however far below it the others lie.
        const T* krow = Ku + (size_t)min(i, n - 1) * D + half * EPV;
        float dot = 0.0f;
#pragma unroll
        for (int g = 0; g < NG; ++g) dot += dot_piece<T>(bq[g], *(const uint4*)(krow + g * 2 * EPV));
        dot += __shfl_xor(dot, 32, kWave);
        M = logit2_gumbel(lp, dot, 0.0f, rkey ^ ((uint32_t)i * kKposMul));
    }
    const int jt_end = min(i0 + kTile - 1, n - 1) / kTile;                      // this wave's last key tile
    const int jt_last = min(rb * (4 * kTile) + 4 * kTile - 1, n - 1) / kTile;   // the workgroup's
    uint4 stage[Stage::NP];
    Stage::fetch(Ku, 0, n, stage);
    Stage::park(kbuf[0], stage);
    __syncthreads();
    for (int jt = 0; jt <= jt_last; ++jt) {
        // the next tile (the last one again at the end: rows stay in range), in flight during this tile's work
        Stage::fetch(Ku, min(jt + 1, jt_last) * kTile, n, stage);
        if (active && jt <= jt_end) {
            const char* kb = kbuf[jt & 1];
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int g = 0; g < NG; ++g) acc = Mma<T>::group(Stage::operand(kb, n0, half, g), bq[g], acc);
            const int jb = jt * kTile;
            const int jl = jb + half * 4;                       // first key of this lane in the tile
            const uint32_t kmul = (uint32_t)jb * kKposMul + kmul_lane;
            const float dist0 = (float)(i - jl);
            if constexpr (GUMBEL) {
                // every term against the reference as it stands, (gz - M) folded into the chain: no search for the
                // tile's maximum, no subtraction per logit.  A later, larger logit just gives a term above one.
                const bool diag = jb + kTile - 1 > i0;  // the tile crosses the diagonal for some lane: causal mask
                for (int attempt = 0;; ++attempt) {
                    const float base = BIAS ? fmaf(dist0, -lp.slope1, lp.gz - M) : lp.gz - M;
                    const float ssum = diag ? tile_sum<BIAS, true>(lp, acc, base, rkey, kmul, i - jl)
                                            : tile_sum<BIAS, false>(lp, acc, base, rkey, kmul, 0);
                    const float Snew = Ssum + ssum;
                    // a sum beyond fp32 in some lane (a logit 2^120 above its row's reference): that lane raises its
                    // reference and the wave sums the tile again (the other lanes arrive at the same sums as
                    // before); bounded, so that NaN inputs end as NaN
                    const bool over = !(Snew < 0x1p120f);
                    if (__any(over) && attempt < 64) {
                        if (over) {
                            M += 100.0f;
                            Ssum *= 0x1p-100f;
                        }
                        continue;
                    }
                    Ssum = Snew;
                    break;
                }
                // the reference follows the sum's exponent (exact: a power of two)
                if (Ssum > 0x1p40f) {
                    const int sh = (int)(__float_as_uint(Ssum) >> 23) - 127;
                    M += (float)sh;
                    Ssum = __uint_as_float(__float_as_uint(Ssum) - ((uint32_t)sh << 23));
                }
            } else {
            float y2[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ro = (r >> 2) * 8 + (r & 3);
                y2[r] = logit2_other(lp, acc[r], dist0 - (float)ro, rkey, (uint32_t)(jl + ro));
            }
            if (jb + kTile - 1 > i0) {  // the tile crosses the diagonal for some lane: causal mask
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ro = (r >> 2) * 8 + (r & 3);
                    y2[r] = (jl + ro <= i) ? y2[r] : -INFINITY;
                }
            }
            float tmax = y2[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, y2[r]);
            const float Mn = fmaxf(M, tmax);
            if (Mn > -INFINITY) {
                float ssum = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) ssum += hw_exp2(y2[r] - Mn);
                Ssum = Ssum * hw_exp2(M - Mn) + ssum;
                M = Mn;
            }
            }
        }
        if (jt < jt_last) Stage::park(kbuf[(jt + 1) & 1], stage);
        __syncthreads();
    }
    if (!active) return;
    // the two halves of the wave hold disjoint key subsets of the same query
    const float M2 = __shfl_xor(M, 32, kWave), S2 = __shfl_xor(Ssum, 32, kWave);
    const float Mt = fmaxf(M, M2);
    const float St = (M > -INFINITY ? Ssum * hw_exp2(M - Mt) : 0.0f) + (M2 > -INFINITY ? S2 * hw_exp2(M2 - Mt) : 0.0f);
    if (half == 0 && i < n) {
        // log2 of the row's normaliser; the trimmed second pass wants it subtracted from the adjustment's
        // constant part, so that is what is left for it
        const float c = Mt + hw_log2(St);
        a.ws_c[(size_t)u * a.n_pad + i] = GUMBEL ? lp.gz - c : c;
        a.ws_r[(size_t)u * a.n_pad + i] = rkey;
    }
}

// ------------------------------------------------------------------ pass 2
template <typename T, int D, bool GUMBEL, bool BIAS>
__global__ void __launch_bounds__(kPrefillThreads) prefill_colsum_kernel(const PrefillArgs a, int nblk, int64_t units) {
    constexpr int EPV = ElemTraits<T>::kPerVec;
    constexpr int NG = D / (2 * EPV);
    using Stage = TileStage<T, D>;
    __shared__ __attribute__((aligned(16))) char qbuf[2][Stage::kBufBytes];
    __shared__ __attribute__((aligned(16))) float cbuf[2][kTile];     // the tile's row normalisers ...
    __shared__ __attribute__((aligned(16))) uint32_t rbuf[2][kTile];  // ... and row noise keys
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n0 = lane & 31, half = lane >> 5;
    int64_t u;
    int cb;  // longest columns (lowest keys) first
    unit_and_block(nblk, u, cb);
    if (u >= units) return;  // workgroup-uniform
    const int h = (int)(u % a.H), b = (int)((u / a.H) % a.B);
    const int n = a.seq_n ? a.seq_n[b] : a.n;  // this sequence's prompt length; rows n..a.n-1 are padding
    const bool first_of_group = (u % a.G) == 0;
    if (n < 1 || n > a.n) {  // workgroup-uniform: the unit is skipped and counted
        if (cb == 0 && threadIdx.x == 0 && first_of_group) atomicAdd(a.ws_err, 1);
        return;
    }
    if (cb == 0 && threadIdx.x == 0 && first_of_group) a.len[u / a.G] = n;
    if (cb * (4 * kTile) >= n) return;  // workgroup-uniform: the block lies in the padding
    const int j0 = cb * (4 * kTile) + wv * kTile;
    const bool active = j0 < n;  // wave-uniform; inactive waves still fetch tiles and meet the barriers
    const int j = j0 + n0;
    const T* Qu = (const T*)a.Q + (size_t)u * a.n * D;
    const T* Ku = (const T*)a.K + (size_t)(u / a.G) * a.cap * D;  // G query heads read one cached head

    uint4 bk[NG];
    {
        const T* row = Ku + (size_t)min(j, n - 1) * D + half * EPV;
#pragma unroll
        for (int g = 0; g < NG; ++g) bk[g] = *(const uint4*)(row + g * 2 * EPV);
    }
    LogitParams lp;
    lp.c1 = a.inv_tau * kLog2e;
    lp.sc1 = a.scale * lp.c1;
    lp.slope1 = (BIAS ? a.slopes[h] : 0.0f) * lp.c1;
    lp.inv_tau = a.inv_tau;
    lp.gz = -kLog2Ln2 * a.inv_tau;
    lp.noise = a.noise;
    const uint32_t kmul = (uint32_t)j * kKposMul;  // this lane's key in every hash
    const float* wc = a.ws_c + (size_t)u * a.n_pad;
    const uint32_t* wr = a.ws_r + (size_t)u * a.n_pad;

    float colsum = 0.0f;
    const int it_begin = j0 / kTile;                    // this wave's first query tile (the diagonal one)
    const int it_first = cb * 4, it_end = (n - 1) / kTile;  // the workgroup's range of query tiles
    // a tile's 32 row statistics ride with the tile: one wave fetches them (n_pad covers whole tiles)
    uint4 stage[Stage::NP];
    float c_st = 0.0f;
    uint32_t r_st = 0u;
    auto fetch_stats = [&](int it) {
        if (threadIdx.x < kTile) {
            c_st = wc[it * kTile + threadIdx.x];
            r_st = wr[it * kTile + threadIdx.x];
        }
    };
    auto park_stats = [&](int buf) {
        if (threadIdx.x < kTile) {
            cbuf[buf][threadIdx.x] = c_st;
            rbuf[buf][threadIdx.x] = r_st;
        }
    };
    // The query tiles are walked from the LAST one down: every column block of a unit then starts at the same
    // tile and the blocks, which run at the same time on one XCD, ask its L2 for the same rows at about the
    // same time (walking up, each block starts at its own diagonal and the L2 sees 16 unrelated streams:
    // 2.7 GB instead of 1.0 GB fetched on the GPT-J-shaped workload).
    Stage::fetch(Qu, it_end * kTile, n, stage);
    fetch_stats(it_end);
    Stage::park(qbuf[0], stage);
    park_stats(0);
    __syncthreads();
    for (int it = it_end; it >= it_first; --it) {
        const int cur = (it_end - it) & 1;
        // the next tile (the first one again at the end: rows stay in range), in flight during this tile's work
        Stage::fetch(Qu, max(it - 1, it_first) * kTile, n, stage);
        fetch_stats(max(it - 1, it_first));
        if (active && it >= it_begin) {
            const char* qb = qbuf[cur];
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int g = 0; g < NG; ++g) acc = Mma<T>::group(Stage::operand(qb, n0, half, g), bk[g], acc);
            const int ib = it * kTile;
            const bool edge = (ib < j0 + kTile) || (ib + kTile > n);  // crosses the diagonal or the end of the prompt
            float z[16];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int ir = ib + q4 * 8 + half * 4;  // 4 consecutive query rows
                const float4 c4 = *(const float4*)&cbuf[cur][q4 * 8 + half * 4];
                const uint4 r4 = *(const uint4*)&rbuf[cur][q4 * 8 + half * 4];
                const float cs[4] = {c4.x, c4.y, c4.z, c4.w};
                const uint32_t rs[4] = {r4.x, r4.y, r4.z, r4.w};
                const float dist0 = (float)(ir - j);
                if constexpr (GUMBEL) {
                    // cs holds (adjustment's constant part - row normaliser): z = 2^(x2 - log2(t)/tau + cs)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float l2t = hw_log2(neg_log2_uniform(mix32(rs[e] ^ kmul)));
                        float t = fmaf(l2t, -lp.inv_tau, cs[e]);
                        if (BIAS) t = fmaf(dist0 + (float)e, -lp.slope1, t);
                        z[q4 * 4 + e] = hw_exp2(fmaf(acc[q4 * 4 + e], lp.sc1, t));
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float y = logit2_other(lp, acc[q4 * 4 + e], dist0 + (float)e, rs[e], (uint32_t)j);
                        z[q4 * 4 + e] = hw_exp2(y - cs[e]);
                    }
                }
            }
            if (edge) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = ib + (r >> 2) * 8 + half * 4 + (r & 3);
                    z[r] = (i >= j && i < n) ? z[r] : 0.0f;
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) colsum += z[r];
        }
        if (it > it_first) {
            Stage::park(qbuf[cur ^ 1], stage);
            park_stats(cur ^ 1);
        }
        __syncthreads();
    }
    if (!active) return;
    colsum += __shfl_xor(colsum, 32, kWave);
    if (half == 0 && j < n) {
        // one query head per cached head: the column sum is the score; else the heads' sums are
        // added up by the launch that follows
        if (a.G == 1) a.score[(size_t)u * a.cap + j] = colsum;
        else a.ws_f[(size_t)u * a.n_pad + j] = colsum;
        if (first_of_group) a.pos[(size_t)(u / a.G) * a.cap + j] = j;
    }
}

// Grouped-query attention: the score of a cached head is the sum of its query heads' column sums
// (added in head order, so the result does not depend on scheduling).
__global__ void __launch_bounds__(256) prefill_group_sum_kernel(const PrefillArgs a, int64_t kv_units) {
    const int64_t u = blockIdx.x;
    const int j = blockIdx.y * 256 + threadIdx.x;
    if (u >= kv_units) return;
    const int hkv = a.H / a.G, b = (int)((u / hkv) % a.B);
    const int n = a.seq_n ? a.seq_n[b] : a.n;
    if (n > a.n || j >= n) return;
    float s = 0.0f;
    for (int g = 0; g < a.G; ++g) s += a.ws_f[((size_t)u * a.G + g) * a.n_pad + j];
    a.score[(size_t)u * a.cap + j] = s;
}

template <typename T, int D>
static hipError_t launch_prefill_t(const PrefillArgs& a, int64_t U, hipStream_t st) {
    const int nblk = (a.n + 4 * kTile - 1) / (4 * kTile);
    const int64_t groups = (U + kXcds - 1) / kXcds;  // units are dealt to XCDs in groups of 8
    const dim3 grid((unsigned)(groups * kXcds * nblk)), block(kPrefillThreads);
    // four builds of each pass: the Gumbel adjustment in the trimmed form or any adjustment in the plain form,
    // with or without the position-bias term
    const bool gum = a.noise == kNoiseGumbel, bias = a.slopes != nullptr;
    if (gum && bias) hipLaunchKernelGGL((prefill_rowstats_kernel<T, D, true, true>), grid, block, 0, st, a, nblk, U);
    else if (gum) hipLaunchKernelGGL((prefill_rowstats_kernel<T, D, true, false>), grid, block, 0, st, a, nblk, U);
    else if (bias) hipLaunchKernelGGL((prefill_rowstats_kernel<T, D, false, true>), grid, block, 0, st, a, nblk, U);
    else hipLaunchKernelGGL((prefill_rowstats_kernel<T, D, false, false>), grid, block, 0, st, a, nblk, U);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (gum && bias) hipLaunchKernelGGL((prefill_colsum_kernel<T, D, true, true>), grid, block, 0, st, a, nblk, U);
    else if (gum) hipLaunchKernelGGL((prefill_colsum_kernel<T, D, true, false>), grid, block, 0, st, a, nblk, U);
    else if (bias) hipLaunchKernelGGL((prefill_colsum_kernel<T, D, false, true>), grid, block, 0, st, a, nblk, U);
    else hipLaunchKernelGGL((prefill_colsum_kernel<T, D, false, false>), grid, block, 0, st, a, nblk, U);
    e = hipGetLastError();
    if (e != hipSuccess || a.G == 1) return e;
    hipLaunchKernelGGL(prefill_group_sum_kernel, dim3((unsigned)(U / a.G), (unsigned)((a.n + 255) / 256)), dim3(256), 0,
                       st, a, U / a.G);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs& a, int64_t U, int32_t d, int32_t dtype, hipStream_t stream) {
    if (dtype == KF_BF16) {
        if (d == 64) return launch_prefill_t<bf16_t, 64>(a, U, stream);
        if (d == 128) return launch_prefill_t<bf16_t, 128>(a, U, stream);
        if (d == 256) return launch_prefill_t<bf16_t, 256>(a, U, stream);
    } else if (dtype == KF_F16) {
        if (d == 64) return launch_prefill_t<f16_t, 64>(a, U, stream);
        if (d == 128) return launch_prefill_t<f16_t, 128>(a, U, stream);
        if (d == 256) return launch_prefill_t<f16_t, 256>(a, U, stream);
    } else {
        if (d == 64) return launch_prefill_t<float, 64>(a, U, stream);
        if (d == 128) return launch_prefill_t<float, 128>(a, U, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace kf
