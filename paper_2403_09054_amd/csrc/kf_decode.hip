// Fused decode step of Keyformer for gfx950: append, logits, attention and
// score accumulation in one kernel, K and V each streamed from HBM once.
//
// Per unit (one layer/batch/head cache) the step is (Algorithm 1 else-branch):
//   append the new token;  x_j = scale*<q,K_j> - slope*(q_pos - pos_j)   (Eq. 1)
//   out = sum_j softmax(x)_j V_j                                          (attention)
//   f_j += softmax((x + zeta)/tau)_j                                      (Eq. 4, Eq. 11, Sec. 3.3.2)
//
// Work decomposition: a unit's m tokens are cut into S contiguous splits, one
// workgroup each.  A workgroup streams its K rows (16 bytes per lane, a row
// spread over D*sizeof(T)/16 adjacent lanes so that every wave-wide load is one
// contiguous kilobyte), applies position bias and logit adjustment to the
// logits as they come out of the dot products (the vector units have time to
// spare while the next rows are in flight) and keeps both adjusted logit rows
// in LDS; between the streams only the exponentials and the two softmaxes'
// sums remain, formed while the first V tile is already in flight; then it
// streams its V rows.  With S == 1 it finishes the unit itself.  With S > 1 it leaves a
// partial record (un-normalised output, local max and sum of both softmaxes,
// un-normalised score increments) and a second, tiny launch merges the records
// of each unit.  (Merging inside the first launch, by the last split to arrive,
// needs device-scope fences; on this multi-die part every such fence writes
// back an L2 and the kernel ran 6x slower, so the merge is a launch of its own.)
#include "kf_device.h"
#include "kf_internal.h"
#include "kf_merge.h"

namespace kf {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeThreadsBig = 512;   // 4 or 8 query heads, one split: a workgroup with up to most of a CU's LDS
constexpr int kDecodeRedWaves = 4;       // rows of LDS in which a workgroup's waves fold their partial outputs
constexpr int kDecodeMaxChunk = 4096;   // tokens per split the LDS arrays are sized for
constexpr int kDecodeMinBlocks = 1024;  // workgroups wanted on the chip
constexpr int kComputeUnits = 256;                      // MI355X
constexpr int kDecodeBlockOverheadTokens = 48;          // fixed cost of a workgroup, in tokens' worth of time
constexpr int kDecodeMinChunk = 128;
constexpr size_t kDecodeLdsBudget = 65536 - 1024;       // dynamic LDS of a split workgroup
constexpr size_t kDecodeLdsPair = 81920 - 1024;         // ... of a single-split workgroup: two fit a CU's 160 KB
constexpr int kDecodeSingleMinUnits = 320;              // units from which one workgroup per unit fills the chip
constexpr size_t kDecodeLdsWhole = 163840 - 2048;       // ... of a workgroup that has a CU to itself
constexpr size_t kDecodeBigMinLogits8 = 36 * 1024;      // logit bytes from which 8 query heads take the 8-wave workgroup
constexpr size_t kDecodeBigMinLogits4 = 24 * 1024;      // ... 4 query heads
constexpr size_t kDecodeBigMinLogitsSplit = 16 * 1024;  // ... a split of either (few units: few, large workgroups)
constexpr int kDecodeMinBlocksGrouped = 256;            // workgroups wanted on the chip with 4 or 8 query heads
constexpr int kDecodeBigMinUnits = 256;                 // units from which one such workgroup per unit fills the chip

constexpr int kDecodeUnroll = 4;  // 16-byte loads a lane keeps in flight per tile (2 and 8 measured within 2 %)

// ---- lane-group sums without LDS traffic ---------------------------------
// A row's partial dot products sit in LPR adjacent lanes.  The data-parallel
// primitive moves (quad permutes, half-row and row mirrors) fold 16 lanes in
// four single-cycle adds; a 32-lane row needs one more exchange across the two
// 16-lane rows.  Every lane of the group ends up with the group's sum.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int LPR>
__device__ __forceinline__ float group_sum(float p) {
    static_assert(LPR == 8 || LPR == 16 || LPR == 32, "row spans 8, 16 or 32 lanes");
    p += dpp_move<0xB1>(p);   // quad_perm [1,0,3,2]
    p += dpp_move<0x4E>(p);   // quad_perm [2,3,0,1]
    p += dpp_move<0x141>(p);  // row_half_mirror: the other quad of the 8 lanes
    if (LPR >= 16) p += dpp_move<0x140>(p);  // row_mirror: the other 8 lanes of the row
    if (LPR >= 32)
        p += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, p), 0x401F));  // lane ^ 16
    return p;
}

// ---- <q, K_row piece> for the 16 bytes a lane holds ------------------------
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
template <typename T>
struct QueryPiece;
template <>
struct QueryPiece<float> {
    float q[4];
    __device__ __forceinline__ void load(const uint4& r) { unpack16<float>(r, q); }
    __device__ __forceinline__ float dot(const uint4& k) const {
        float p = __uint_as_float(k.x) * q[0];
        p = fmaf(__uint_as_float(k.y), q[1], p);
        p = fmaf(__uint_as_float(k.z), q[2], p);
        p = fmaf(__uint_as_float(k.w), q[3], p);
        return p;
    }
};
template <>
struct QueryPiece<bf16_t> {
    uint4 q;  // eight bf16, kept packed: products of bf16 pairs are accumulated in fp32
    __device__ __forceinline__ void load(const uint4& r) { q = r; }
    __device__ __forceinline__ float dot(const uint4& k) const {
        float p = 0.0f;
        p = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.x), __builtin_bit_cast(bf16x2_t, q.x), p, false);
        p = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.y), __builtin_bit_cast(bf16x2_t, q.y), p, false);
        p = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.z), __builtin_bit_cast(bf16x2_t, q.z), p, false);
        p = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, k.w), __builtin_bit_cast(bf16x2_t, q.w), p, false);
        return p;
    }
};

// One step of a reduce-scatter over lane groups O lanes apart: a lane keeps one half of its values, sends
// the other half to its partner and adds what the partner sends -- half the exchanges of folding every value
// both ways, and afterwards the halves are spread over the two groups.
template <int N, int O>
__device__ __forceinline__ void halve(const float (&in)[N], float (&out)[N / 2], int lane) {
    static_assert(O == 8 || O == 16 || O == 32, "partner distances of a wave's rows");
    const bool up = (lane & O) != 0;
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
        const float keep = up ? in[N / 2 + i] : in[i];
        const float send = up ? in[i] : in[N / 2 + i];
        float recv;
        if constexpr (O == 8) recv = dpp_move<0x128>(send);  // row_ror:8
        else if constexpr (O == 16)
            recv = __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, send), 0x401F));
        else recv = __shfl_xor(send, 32, kWave);
        out[i] = keep + recv;
    }
}

// Wave-wide max / sum: the data-parallel moves fold a 16-lane row, two exchanges through the LDS crossbar
// (lane ^ 16, lane ^ 32) fold the four rows.  Every lane ends up with the result.
__device__ __forceinline__ float wave_max_fast(float v) {
    v = fmaxf(v, dpp_move<0xB1>(v));
    v = fmaxf(v, dpp_move<0x4E>(v));
    v = fmaxf(v, dpp_move<0x141>(v));
    v = fmaxf(v, dpp_move<0x140>(v));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F)));
    return fmaxf(v, __shfl_xor(v, 32, kWave));
}
__device__ __forceinline__ float wave_sum_fast(float v) {
    v = group_sum<32>(v);
    return v + __shfl_xor(v, 32, kWave);
}

typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
template <>
struct QueryPiece<f16_t> {
    uint4 q;  // eight halves, kept packed: products of half pairs are accumulated in fp32
    __device__ __forceinline__ void load(const uint4& r) { q = r; }
    __device__ __forceinline__ float dot(const uint4& k) const {
        float p = 0.0f;
        p = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, k.x), __builtin_bit_cast(f16x2_t, q.x), p, false);
        p = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, k.y), __builtin_bit_cast(f16x2_t, q.y), p, false);
        p = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, k.z), __builtin_bit_cast(f16x2_t, q.z), p, false);
        p = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, k.w), __builtin_bit_cast(f16x2_t, q.w), p, false);
        return p;
    }
};

// Block-wide sums of N values at once.  `red` holds N*NT/64 + N floats.  With few values and waves every
// thread folds the waves' results itself (one pair of barriers); with many (8 query heads, 8 waves: 128 LDS
// reads per thread that way) N threads fold them once and publish the N results.
template <int NT, int N>
__device__ __forceinline__ void block_sum_n(float (&v)[N], float* red) {
    constexpr int NW = NT / 64;
    constexpr bool kTwoLevel = N * NW > 32;
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = kTwoLevel ? wave_sum_fast(v[i]) : wave_sum(v[i]);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) red[N * (threadIdx.x >> 6) + i] = v[i];
    }
    __syncthreads();
    if constexpr (kTwoLevel) {
        float* res = red + N * NW;
        if (threadIdx.x < N) {
            float r = red[threadIdx.x];
#pragma unroll
            for (int w = 1; w < NW; ++w) r += red[N * w + threadIdx.x];
            res[threadIdx.x] = r;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = res[i];
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            float r = red[i];
#pragma unroll
            for (int w = 1; w < NW; ++w) r += red[N * w + i];
            v[i] = r;
        }
    }
}

// Logits of a query group on the matrix cores.  With 8 bf16 query heads per
// cached head the logits are a small dense contraction, rows x head dimension x
// heads, and the lane-group reductions of the vector form cost more registers
// and issue slots than the chip has to spare (4 heads still run faster in the
// vector form: 64 % against 58 % of the HBM peak measured).  A wave multiplies a tile of 16 key rows (A operand: lane l holds eight
// consecutive elements of row l%16, the l/16-th eight of every 32) by the query
// group padded to 16 heads (B operand, same element assignment, kept in
// registers), D/32 MFMAs per tile, and lane l receives the logits of rows
// 4*(l/16) .. +3 for head l%16.  No dot products, no lane-group reductions.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <typename T, int G>
struct MfmaLogits {
    static constexpr bool value = false;
};
template <int G>
struct MfmaLogits<bf16_t, G> {
    static constexpr bool value = (G >= 8);
};
template <int G>
struct MfmaLogits<f16_t, G> {
    static constexpr bool value = (G >= 8);
};
// acc += A (16 rows x 32) * B (32 x 16 columns), eight 16-bit elements of each per lane
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
template <typename T>
__device__ __forceinline__ f32x4_t mfma_16x16x32(const uint4& a, const uint4& b, f32x4_t acc);
template <>
__device__ __forceinline__ f32x4_t mfma_16x16x32<bf16_t>(const uint4& a, const uint4& b, f32x4_t acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x4_t mfma_16x16x32<f16_t>(const uint4& a, const uint4& b, f32x4_t acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), acc, 0, 0, 0);
}

// Attention output of a query group on the matrix cores.  The contraction of out[g][c] = sum_j p[g][j]*V[j][c]
// runs over the tokens, and an MFMA lane must hold eight consecutive contraction elements -- but a coalesced
// load gives a lane eight consecutive COLUMNS of one token.  So the contraction index is widened to the pair
// (token, column within the lane's eight): with rows of 256 bytes a wave-wide load is four tokens x 16 lanes,
// which read as the B operand of a 16x16x32 MFMA is B[k = (token, e)][n = lane's piece] = V[token][8n + e] --
// the loaded registers as they are, no transposition.  The A operand carries the weights with a Kronecker
// delta, A[m = (head, e')][k = (token, e)] = p[head][token] * (e == e'), so that C[(head, e')][n] =
// sum_token p[head][token] * V[token][8n + e']: 16 rows of A are two heads x eight column offsets, four MFMAs
// cover the eight heads, and a lane's A operand is one weight in one fixed 16-bit slot, zeros elsewhere.
// Seven eighths of the matrix work multiply zeros, on units that idle otherwise; against 64 multiply-adds
// per 16 bytes on the vector units it leaves them eight byte-permutes per MFMA pair.  Weights enter as
// bf16, so each is split in two terms (the upper 16 bits and the upper 16 bits of the rest: 2^-16
// relative), one MFMA each; they wait in LDS already split and packed.
template <typename T, int D, int G>
struct MfmaPV {
    static constexpr bool value = false;
};
template <>
struct MfmaPV<bf16_t, 128, 8> {
    static constexpr bool value = true;
};
// weight p in [0, 1] -> (p rounded to bf16) | (the rest, rounded to bf16) >> 16: the two terms add up to p within
// 2^-18 relative (round to nearest even on the bit patterns; the rest is exact in fp32 and may be negative)
__device__ __forceinline__ uint32_t bf16_bits_rne(float x) {
    const uint32_t b = __float_as_uint(x);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
}
__device__ __forceinline__ uint32_t split_weight(float p) {
    const uint32_t hi = bf16_bits_rne(p);
    return hi | (bf16_bits_rne(p - __uint_as_float(hi)) >> 16);
}
__device__ __forceinline__ float joined_weight(uint32_t w) {
    return __uint_as_float(w & 0xFFFF0000u) + __uint_as_float(w << 16);
}

// One workgroup streams the cache rows [j0, j1) of one cached head ("unit") once
// and serves the G query heads that read it (G = 1: ordinary multi-head
// attention; G > 1: grouped-query attention, query head hq = h*G + g).
template <typename T, int D, int NT, int G>
__device__ __forceinline__ void decode_block(const DecodeArgs& a) {
    constexpr int EPV = ElemTraits<T>::kPerVec;  // elements per 16-byte vector
    constexpr int LPR = D / EPV;                 // lanes that share one row
    constexpr int RPW = kWave / LPR;             // rows per wave-wide load
    constexpr int NW = NT / kWave;
    constexpr int RPB = RPW * NW;                // rows per block-wide load
    // independent loads in flight per lane (8 query heads: registers are short; one instead of two costs the
    // 8-wave workgroup 15-20 %, four do not fit)
    constexpr int UNR = (G >= 8 && !MfmaPV<T, D, G>::value) ? 2 : kDecodeUnroll;
    constexpr int TILE = RPB * UNR;              // rows per tile of the workgroup
    constexpr int PW = D + 4;                    // floats in a partial record
    constexpr bool BIG = NW > kDecodeRedWaves;  // the 8-wave workgroup: one split, 4 or 8 query heads, up to most of a CU's LDS
    constexpr bool PVM = MfmaPV<T, D, G>::value;  // attention output on the matrix cores
    constexpr size_t ROWB = (size_t)D * sizeof(T);
    static_assert(LPR <= 32 && D <= NT, "row must fit half a wave, output a block");

    extern __shared__ float smem[];
    const int CS = a.chunk + 1;        // logits of the split's rows (+1: the new token)
    float* xs = smem;                  // [G][CS] logits, then attention weights
    float* ys = smem + G * CS;         // [G][CS] perturbed logits / tau, then their exponentials
    float* red_o = smem + ((2 * G * CS + 3) & ~3);  // [NW][G*D] output partials, 16-byte aligned (not BIG)
    __shared__ __attribute__((aligned(16))) float red_s[2 * G * (NW + 2)];
    __shared__ float stat[4 * G];      // per query head: max x, sum p, max y, sum e
    __shared__ unsigned long long evict_min[NW];  // whole-step launch: per-wave smallest (score, position) pack
    __shared__ int evict_slot;
    __shared__ float new_score;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int sub = lane / LPR, cl = lane % LPR;
    const int S = a.S;
    const int64_t u = blockIdx.x / S;
    const int s = blockIdx.x % S;
    const int h = (int)(u % a.H), b = (int)((u / a.H) % a.B), l = a.layer0 + (int)(u / ((int64_t)a.H * a.B));

    // query position and temperature of this step: from the host, or from the device step counter
    // (same fp32 operations, in the same order, as the host's schedule function)
    int q_pos = a.q_pos;
    float inv_tau = a.inv_tau;
    if (a.step) {
        const int t = max(*a.step, 1);  // decode steps count from 1 (0 is the prompt iteration)
        q_pos = a.n0 + t - 1;
        inv_tau = 1.0f / schedule_tau(a.tau_init, a.dtau, min(t, a.T));  // IEEE division, as on the host
    }
    if (a.seq_q_pos) q_pos = a.seq_q_pos[b];  // a batch whose sequences are at different steps
    if (a.seq_tau) inv_tau = 1.0f / a.seq_tau[b];
    const int len0 = a.len[u];
    const int m = len0 + 1;
    if (len0 < 0 || len0 >= a.cap || len0 > S * a.chunk) {
        // no room for the new token (or a launch shaped for fewer tokens):
        // leave the unit alone and report it
        if (s == 0) {
            for (int c = tid; c < G * D; c += NT) a.out[u * G * D + c] = 0.0f;
            if (tid == 0) {
                atomicAdd(a.ws_err, 1);
                a.ws_m[u] = 0;  // tokens scored in this unit by this launch: none
                // whole-step launch: the selection would have refused this unit as well (slot layout,
                // more than one token over budget) and reported it on its own
                if (a.fuse_k > 0 && len0 > a.fuse_k + 1) atomicAdd(a.ws_err, 1);
            }
        }
        return;
    }
    // The split streams cache rows [j0, j1).  The new token never comes from the
    // cache: the last split takes its key and value from k_new / v_new and keeps
    // its logit in the LDS slot behind its own rows.
    const int j0 = s * a.chunk;
    const int j1 = min(len0, j0 + a.chunk);
    const int cnt_c = max(j1 - j0, 0);
    const bool owner = (s == S - 1);
    const int cnt = cnt_c + (owner ? 1 : 0);

    const char* Ku = (const char*)a.K + (size_t)u * a.cap * ROWB;
    const char* Vu = (const char*)a.V + (size_t)u * a.cap * ROWB;
    const T* qu = (const T*)a.q + (size_t)u * G * D;
    const char* knew = (const char*)a.k_new + (size_t)u * ROWB;
    const char* vnew = (const char*)a.v_new + (size_t)u * ROWB;
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;

    // Whole-step launch (S == 1): a unit exactly one token over its budget evicts in this launch, and the
    // new token then goes straight into the freed slot instead of being appended first.
    const bool over = a.fuse_k > 0 && m > a.fuse_k;
    const bool evict_here = over && m == a.fuse_k + 1;

    // ---- append: the last split stores the new row (nobody reads it back in this launch)
    if (owner && !evict_here) {
        if (wv == 0 && lane < LPR) ((uint4*)(a.K))[((size_t)u * a.cap + len0) * LPR + lane] = ((const uint4*)knew)[lane];
        if (wv == 1 && lane < LPR) ((uint4*)(a.V))[((size_t)u * a.cap + len0) * LPR + lane] = ((const uint4*)vnew)[lane];
        if (tid == 2 * kWave) pu[len0] = q_pos;
    }

    // This lane's piece of row (base + i*RPB + sub) sits at lane_off + base*ROWB + i*RPB*ROWB.
    const size_t lane_off = (size_t)sub * ROWB + (size_t)cl * 16;
    const int base0 = j0 + wv * RPW;
    // a tile starting at `base` is "plain" (no bounds checks) if all its rows are below j1
    auto plain = [&](int base) { return base + (UNR - 1) * RPB + RPW <= j1; };
    auto load_plain = [&](const char* rows, int base, uint4(&raw)[UNR]) {
        const char* p = rows + (size_t)base * ROWB + lane_off;
#pragma unroll
        for (int i = 0; i < UNR; ++i) raw[i] = stream_load((const uint4*)(p + (size_t)i * RPB * ROWB));
    };
    auto load_edge = [&](const char* rows, int base, uint4(&raw)[UNR]) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int j = base + i * RPB + sub;
            raw[i] = make_uint4(0u, 0u, 0u, 0u);
            if (j < j1) raw[i] = stream_load((const uint4*)(rows + (size_t)j * ROWB + (size_t)cl * 16));
        }
    };
    auto load_tile = [&](const char* rows, int base, uint4(&raw)[UNR]) {
        if (plain(base)) load_plain(rows, base, raw);
        else load_edge(rows, base, raw);
    };

    // ---- phase 1: stream K (next tile in flight while this one is reduced), logits into LDS
    uint4 cur[UNR], nxt[UNR];
    const bool rnd_l = (a.noise == kNoiseGumbel || a.noise == kNoiseGaussian);
    if constexpr (MfmaLogits<T, G>::value) {
        if constexpr (D >= 128) {
            // Rows of 256 bytes and more.  An MFMA row slot holds a QUARTER of a cache row: slot i = 4*r + s
            // is row r of a group of four rows, pieces {s, 4+s, 8+s, 12+s} (16 bytes each) of every 256 bytes.
            // Lane (i, kb) then loads piece 4*kb + s of row r: four adjacent lanes read 64 contiguous bytes,
            // the 64 lanes of a load instruction four whole 256-byte row parts -- every cache line is asked
            // for once, by one instruction (with a whole row per slot a line is split over two instructions
            // and adjacent lanes sit 256 bytes apart: the K stream ran 28 us per 2048-token unit against
            // 20 us for the V stream).  The B operand's column j = 4*g' + s' carries head g' of a group of
            // four, restricted to the pieces of class s'; of the 16x16 products only those with s = s' are
            // wanted, and their sum over s is the logit of (row r, head g') -- two MFMAs (two head groups) per
            // four rows, twice the matrix work of the plain layout, on units that idle anyway.
            constexpr int KS = D / 128;  // 256-byte parts of a row = MFMA k-steps
            const int i4 = lane & 15, kb = lane >> 4, r4 = i4 >> 2, s4 = i4 & 3;
            uint4 bq[2][KS];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    bq[hh][ks] = ((const uint4*)(qu + (size_t)(hh * 4 + r4) * D))[16 * ks + 4 * kb + s4];
            }
            // After the MFMAs lane (j = i4, kb) holds, in register reg, the product of slot 4*kb + reg with
            // column j: the wanted one is reg = s4 (row kb of the group, head r4 of the head group); the four
            // lanes of a quad add theirs up.  A step is 16 rows (four groups) x 8 heads = 128 logits per
            // wave: lane s4 of a quad keeps those of row group s4, i.e. ONE row and the heads r4, r4 + 4, and
            // applies position bias and logit adjustment to them right here, while the next rows are in
            // flight -- the statistics pass after the K stream shrinks to the running maxima kept per lane.
            static_assert(G == 8, "two head groups of four");
            float slope_l[2];
            uint32_t rkey_l[2];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int hq = h * G + hh * 4 + r4;
                slope_l[hh] = a.slopes ? a.slopes[hq] : 0.0f;
                rkey_l[hh] = rnd_l ? row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)hq), (uint32_t)q_pos) : 0u;
            }
            float mx_l[2] = {-INFINITY, -INFINITY}, my_l[2] = {-INFINITY, -INFINITY};
            // rows past the split re-read its last row (the address stays inside the cache); their logits are dropped
            auto load_rows = [&](int base, uint4(&raw)[4][KS], int& pos1) {
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int row = min(base + wv * 16 + rg * 4 + r4, j1 - 1);
                    const uint4* p = (const uint4*)(Ku + (size_t)row * ROWB) + 4 * kb + s4;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) raw[rg][ks] = stream_load(p + 16 * ks);
                }
                pos1 = pu[min(base + wv * 16 + s4 * 4 + kb, j1 - 1)];
            };
            auto logits_of = [&](int base, const uint4(&raw)[4][KS], int pos1) {
                float v[2] = {0.0f, 0.0f};
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
                            acc = mfma_16x16x32<T>(raw[rg][ks], bq[hh][ks], acc);
                        float t = s4 == 0 ? acc[0] : s4 == 1 ? acc[1] : s4 == 2 ? acc[2] : acc[3];
                        t += dpp_move<0xB1>(t);  // the quad's four classes
                        t += dpp_move<0x4E>(t);
                        if (s4 == rg) v[hh] = t;
                    }
                }
                const int row = base + wv * 16 + s4 * 4 + kb;
                if (row < j1) {
                    const int dist = a.new_pos ? (len0 - row) : (q_pos - pos1);
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        // base-2 domain: x2 = log2(e)*x, y2 = log2(e)*(x + zeta)/tau
                        const float x = (v[hh] * a.scale - slope_l[hh] * (float)dist) * kLog2e;
                        const float y = (x + zeta_log2e(a.noise, rkey_l[hh], (uint32_t)pos1)) * inv_tau;
                        xs[(hh * 4 + r4) * CS + row - j0] = x;
                        ys[(hh * 4 + r4) * CS + row - j0] = y;
                        mx_l[hh] = fmaxf(mx_l[hh], x);
                        my_l[hh] = fmaxf(my_l[hh], y);
                    }
                }
            };
            if (cnt_c > 0) {
                uint4 kcur[4][KS], knxt[4][KS];
                int pcur, pnxt;
                int base = j0;
                load_rows(base, kcur, pcur);
                while (base + NW * 16 < j1) {
                    load_rows(base + NW * 16, knxt, pnxt);
                    logits_of(base, kcur, pcur);
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) kcur[rg][ks] = knxt[rg][ks];
                    }
                    pcur = pnxt;
                    base += NW * 16;
                }
                logits_of(base, kcur, pcur);
            }
            // the 16 lanes of a head pair (quad x four 16-lane rows) fold their maxima; row NW of the table
            // takes the new token's own logits (distance 0: no position bias), or nothing
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                float mx = mx_l[hh], my = my_l[hh];
                mx = fmaxf(mx, dpp_move<0xB1>(mx));
                my = fmaxf(my, dpp_move<0xB1>(my));
                mx = fmaxf(mx, dpp_move<0x4E>(mx));
                my = fmaxf(my, dpp_move<0x4E>(my));
                mx = fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, mx), 0x401F)));
                my = fmaxf(my, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, my), 0x401F)));
                mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
                my = fmaxf(my, __shfl_xor(my, 32, kWave));
                if (kb == 0 && s4 == 0) {
                    red_s[2 * G * wv + 2 * (hh * 4 + r4)] = mx;
                    red_s[2 * G * wv + 2 * (hh * 4 + r4) + 1] = my;
                }
            }
        } else {
            constexpr int KK = D / 32;  // MFMAs (and 16-byte loads per lane) per 16-row tile
            const int mrow = lane & 15, c4 = lane >> 4;
            uint4 bq[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {  // heads G..15 of the padded group are zero
                bq[kk] = ((const uint4*)(qu + (size_t)min(mrow, G - 1) * D))[kk * 4 + c4];
                if (mrow >= G) bq[kk] = make_uint4(0u, 0u, 0u, 0u);
            }
            // The MFMA leaves lane (mrow, c4) with the logits of head mrow for rows 4*c4 .. +3, and nothing of use
            // in the lanes of the padding heads (mrow >= G).  Those take rows 4*c4+2, +3 over from lane mrow-8
            // (one data-parallel move each), so that all 64 lanes apply position bias and logit adjustment to two
            // logits each, right here, while the next rows are in flight: the vector units idle during the K
            // stream, and the statistics pass after it (one more sweep over all G x rows logits, with the
            // workgroup's memory pipeline empty) shrinks to the two running maxima kept per lane.
            static_assert(G == 8, "the padding half of the 16 MFMA columns takes half of the real heads' rows");
            const int g_l = mrow & (G - 1), r_l = (mrow >= G) ? 2 : 0;
            const int hq_l = h * G + g_l;
            const float slope_l = a.slopes ? a.slopes[hq_l] : 0.0f;
            const uint32_t rkey_l = rnd_l ? row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)hq_l), (uint32_t)q_pos) : 0u;
            float mx_l = -INFINITY, my_l = -INFINITY;
            // rows past the split re-read its last row (the address stays inside the cache); their logits are dropped
            auto load_rows = [&](int base, uint4(&raw)[KK], int(&pos2)[2]) {
                const int row = min(base + wv * 16 + mrow, j1 - 1);  // a wave's 16 rows of the workgroup's NW*16
                const uint4* p = (const uint4*)(Ku + (size_t)row * ROWB) + c4;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) raw[kk] = stream_load(p + kk * 4);
#pragma unroll
                for (int r = 0; r < 2; ++r) pos2[r] = pu[min(base + wv * 16 + c4 * 4 + r_l + r, j1 - 1)];
            };
            auto logits_of = [&](int base, const uint4(&raw)[KK], const int(&pos2)[2]) {
                f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
                    acc = mfma_16x16x32<T>(raw[kk], bq[kk], acc);
                const float from2 = dpp_move<0x118>(acc[2]), from3 = dpp_move<0x118>(acc[3]);  // row_shr:8
                const float v[2] = {mrow >= G ? from2 : acc[0], mrow >= G ? from3 : acc[1]};
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int row = base + wv * 16 + c4 * 4 + r_l + r;
                    if (row < j1) {
                        const int dist = a.new_pos ? (len0 - row) : (q_pos - pos2[r]);
                        // base-2 domain: x2 = log2(e)*x, y2 = log2(e)*(x + zeta)/tau
                        const float x = (v[r] * a.scale - slope_l * (float)dist) * kLog2e;
                        const float y = (x + zeta_log2e(a.noise, rkey_l, (uint32_t)pos2[r])) * inv_tau;
                        xs[g_l * CS + row - j0] = x;
                        ys[g_l * CS + row - j0] = y;
                        mx_l = fmaxf(mx_l, x);
                        my_l = fmaxf(my_l, y);
                    }
                }
            };
            if (cnt_c > 0) {
                uint4 kcur[KK], knxt[KK];
                int pcur[2], pnxt[2];
                int base = j0;
                load_rows(base, kcur, pcur);
                while (base + NW * 16 < j1) {
                    load_rows(base + NW * 16, knxt, pnxt);
                    logits_of(base, kcur, pcur);
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) kcur[kk] = knxt[kk];
                    pcur[0] = pnxt[0];
                    pcur[1] = pnxt[1];
                    base += NW * 16;
                }
                logits_of(base, kcur, pcur);
            }
            // the eight lanes of a head (mrow, mrow+8 in each of the four 16-lane rows) fold their maxima; row NW of
            // the table takes the new token's own logits (distance 0: no position bias), or nothing
            mx_l = fmaxf(mx_l, dpp_move<0x128>(mx_l));  // row_ror:8
            my_l = fmaxf(my_l, dpp_move<0x128>(my_l));
            mx_l = fmaxf(mx_l, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, mx_l), 0x401F)));
            my_l = fmaxf(my_l, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, my_l), 0x401F)));
            mx_l = fmaxf(mx_l, __shfl_xor(mx_l, 32, kWave));
            my_l = fmaxf(my_l, __shfl_xor(my_l, 32, kWave));
            if (lane < G) {
                red_s[2 * G * wv + 2 * lane] = mx_l;
                red_s[2 * G * wv + 2 * lane + 1] = my_l;
            }
        }
    } else {
        QueryPiece<T> qp[G];
#pragma unroll
        for (int g = 0; g < G; ++g) qp[g].load(((const uint4*)(qu + (size_t)g * D))[cl]);

        // After the lane-group sums every lane of a row holds all G x UNR logits of its row group.  Lane cl
        // keeps those numbered cl, cl + LPR, ...: number v is head v % G (always cl % G: one head per lane) of
        // the tile's load v / G.  It applies position bias and logit adjustment to them right here, while the
        // next tile is in flight -- the vector units have time to spare during the K stream, and the statistics
        // pass after it (one more sweep over all logits with the memory pipeline empty, all workgroups of a
        // small launch at the same time) shrinks to the two running maxima kept per lane.
        constexpr int NV = G * UNR, VPL = (NV + LPR - 1) / LPR;
        static_assert(LPR % G == 0, "a lane's logits belong to one head");
        const int g_l = cl % G, i_l = cl / G;
        const int hq_l = h * G + g_l;
        const float slope_l = a.slopes ? a.slopes[hq_l] : 0.0f;
        const uint32_t rkey_l = rnd_l ? row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)hq_l), (uint32_t)q_pos) : 0u;
        float mx_l = -INFINITY, my_l = -INFINITY;
        int pcur[VPL], pnxt[VPL];
        // positions of this lane's rows of the tile at `base` (rows past the split: its last row, dropped later)
        auto load_pos = [&](int base, int(&ps)[VPL]) {
#pragma unroll
            for (int r = 0; r < VPL; ++r) {
                const int i = i_l + r * (LPR / G);
                ps[r] = (i < UNR) ? pu[min(base + i * RPB + sub, j1 - 1)] : 0;
            }
        };
        auto logits_of = [&](int base, const int(&ps)[VPL]) {
            float p[G][UNR];
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int i = 0; i < UNR; ++i) p[g][i] = qp[g].dot(cur[i]);
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int i = 0; i < UNR; ++i) p[g][i] = group_sum<LPR>(p[g][i]);
            }
#pragma unroll
            for (int r = 0; r < VPL; ++r) {
                const int i_r = i_l + r * (LPR / G);
                float v = 0.0f;
#pragma unroll
                for (int g = 0; g < G; ++g) {
#pragma unroll
                    for (int i = 0; i < UNR; ++i) v = (g == g_l && i == i_r) ? p[g][i] : v;
                }
                const int j = base + i_r * RPB + sub;
                if (i_r < UNR && j < j1) {
                    const int dist = a.new_pos ? (len0 - j) : (q_pos - ps[r]);
                    // base-2 domain: x2 = log2(e)*x, y2 = log2(e)*(x + zeta)/tau
                    const float x = (v * a.scale - slope_l * (float)dist) * kLog2e;
                    const float y = (x + zeta_log2e(a.noise, rkey_l, (uint32_t)ps[r])) * inv_tau;
                    xs[g_l * CS + j - j0] = x;
                    ys[g_l * CS + j - j0] = y;
                    mx_l = fmaxf(mx_l, x);
                    my_l = fmaxf(my_l, y);
                }
            }
        };
        {
            int base = base0;
            if (base < j1) {
                load_tile(Ku, base, cur);
                load_pos(base, pcur);
            }
            // steady state: the next tile needs no bounds checks, so the loop body is
            // branch-free and only the older tile's loads are waited for
            while (plain(base + TILE)) {
                load_plain(Ku, base + TILE, nxt);
                load_pos(base + TILE, pnxt);
                logits_of(base, pcur);
#pragma unroll
                for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
#pragma unroll
                for (int r = 0; r < VPL; ++r) pcur[r] = pnxt[r];
                base += TILE;
            }
            while (base < j1) {  // the last one or two tiles of the split
                if (base + TILE < j1) {
                    load_edge(Ku, base + TILE, nxt);
                    load_pos(base + TILE, pnxt);
                }
                logits_of(base, pcur);
#pragma unroll
                for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
#pragma unroll
                for (int r = 0; r < VPL; ++r) pcur[r] = pnxt[r];
                base += TILE;
            }
        }
        // per head, the wave's maxima; row NW of the table takes the new token's own logits, or nothing
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mx = wave_max_fast(g == g_l ? mx_l : -INFINITY);
            const float my = wave_max_fast(g == g_l ? my_l : -INFINITY);
            if (lane == 0) {
                red_s[2 * G * wv + 2 * g] = mx;
                red_s[2 * G * wv + 2 * g + 1] = my;
            }
        }
    }
    // the new token's own logits (distance 0: no position bias)
    if (wv == 0) {
        const uint4 kv = ((const uint4*)knew)[cl];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            QueryPiece<T> qg;
            qg.load(((const uint4*)(qu + (size_t)g * D))[cl]);
            const float p = group_sum<LPR>(qg.dot(kv));
            if (lane == 0) {
                float x = -INFINITY, y = -INFINITY;
                if (owner) {
                    const int hq = h * G + g;
                    const uint32_t rk = rnd_l ? row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)hq), (uint32_t)q_pos) : 0u;
                    x = (p * a.scale) * kLog2e;
                    y = (x + zeta_log2e(a.noise, rk, (uint32_t)q_pos)) * inv_tau;
                    xs[g * CS + cnt_c] = x;
                    ys[g * CS + cnt_c] = y;
                }
                red_s[2 * G * NW + 2 * g] = x;
                red_s[2 * G * NW + 2 * g + 1] = y;
            }
        }
    }
    // first V tile: in flight while the softmax statistics are formed
    if (base0 < j1) load_tile(Vu, base0, cur);
    __syncthreads();

    // ---- phase 1.5: position bias, logit adjustment, the two softmaxes' statistics
    float mxy[2 * G];
    {
        // adjusted in the K stream; the waves' maxima (and the new token's logits) wait in red_s
        float* res = red_s + 2 * G * (NW + 1);
        if (tid < 2 * G) {
            float r = red_s[tid];
#pragma unroll
            for (int w2 = 1; w2 <= NW; ++w2) r = fmaxf(r, red_s[2 * G * w2 + tid]);
            res[tid] = r;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2 * G; ++i) mxy[i] = res[i];
    }
    float spe[2 * G];
#pragma unroll
    for (int i = 0; i < 2 * G; ++i) spe[i] = 0.0f;
    for (int t = tid; t < cnt; t += NT) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float p = hw_exp2(xs[g * CS + t] - mxy[2 * g]);
            const float e = hw_exp2(ys[g * CS + t] - mxy[2 * g + 1]);
            xs[g * CS + t] = PVM ? __uint_as_float(split_weight(p)) : p;
            ys[g * CS + t] = e;
            spe[2 * g] += p;
            spe[2 * g + 1] += e;
        }
    }
    block_sum_n<NT, 2 * G>(spe, red_s);  // its barriers also publish the attention weights in xs
    if (tid == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            stat[4 * g + 0] = mxy[2 * g];
            stat[4 * g + 1] = spe[2 * g];
            stat[4 * g + 2] = mxy[2 * g + 1];
            stat[4 * g + 3] = spe[2 * g + 1];
        }
    }
    // (The score increments in ys are written out after the V stream: stores issued here
    // would have to drain before the first V tile could be consumed.)

    // ---- phase 2: stream V, weighted sum
    float acc[G][EPV];
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[g][e] = 0.0f;
    }
    // matrix-core form: lane (piece cl, row sub) feeds A row cl = (head 2*mf + cl/8, column offset cl%8) and
    // receives C rows 4*sub .. +3 = (head 2*mf + sub/2, column offsets 4*(sub%2) .. +3) of column piece cl
    f32x4_t cacc[PVM ? 4 : 1];
    uint32_t sel_hi[4], sel_lo[4];  // byte selectors that put a weight's term into this lane's slot of A
#pragma unroll
    for (int q = 0; q < (PVM ? 4 : 1); ++q) cacc[q] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bool mine = q == ((cl & 7) >> 1), upper = (cl & 1) != 0;
        sel_hi[q] = !mine ? 0x0C0C0C0Cu : upper ? 0x03020C0Cu : 0x0C0C0302u;
        sel_lo[q] = !mine ? 0x0C0C0C0Cu : upper ? 0x01000C0Cu : 0x0C0C0100u;
    }
    auto weigh = [&](int base) {
        if constexpr (PVM) {
            const uint32_t* xw = (const uint32_t*)xs + (cl >> 3) * CS - j0;
            // The matrix cores do not round their fp32 accumulation to nearest: over the hundreds of dependent
            // MFMAs of a long unit that grows into a bias of 1e-4 of the sum.  So a tile's eight MFMAs start
            // from zero and the tile's sums are added to the running ones on the vector units.
            f32x4_t tacc[4];
#pragma unroll
            for (int mf = 0; mf < 4; ++mf) tacc[mf] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int i = 0; i < UNR; ++i) {
                const int j = base + i * RPB + sub;
#pragma unroll
                for (int mf = 0; mf < 4; ++mf) {
                    const uint32_t w = (j < j1) ? xw[2 * mf * CS + j] : 0u;
                    uint4 ah, al;
                    ah.x = __builtin_amdgcn_perm(w, w, sel_hi[0]);
                    ah.y = __builtin_amdgcn_perm(w, w, sel_hi[1]);
                    ah.z = __builtin_amdgcn_perm(w, w, sel_hi[2]);
                    ah.w = __builtin_amdgcn_perm(w, w, sel_hi[3]);
                    al.x = __builtin_amdgcn_perm(w, w, sel_lo[0]);
                    al.y = __builtin_amdgcn_perm(w, w, sel_lo[1]);
                    al.z = __builtin_amdgcn_perm(w, w, sel_lo[2]);
                    al.w = __builtin_amdgcn_perm(w, w, sel_lo[3]);
                    tacc[mf] = mfma_16x16x32<T>(ah, cur[i], tacc[mf]);
                    tacc[mf] = mfma_16x16x32<T>(al, cur[i], tacc[mf]);
                }
            }
#pragma unroll
            for (int mf = 0; mf < 4; ++mf) cacc[mf] += tacc[mf];
            return;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int j = base + i * RPB + sub;
            float vvals[EPV];
            unpack16<T>(cur[i], vvals);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = (j < j1) ? xs[g * CS + j - j0] : 0.0f;
#pragma unroll
                for (int e = 0; e < EPV; ++e) acc[g][e] = fmaf(p, vvals[e], acc[g][e]);
            }
        }
    };
    {
        int base = base0;
        while (plain(base + TILE)) {
            load_plain(Vu, base + TILE, nxt);
            weigh(base);
#pragma unroll
            for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
            base += TILE;
        }
        while (base < j1) {
            if (base + TILE < j1) load_edge(Vu, base + TILE, nxt);
            weigh(base);
#pragma unroll
            for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
            base += TILE;
        }
    }
    if constexpr (PVM) {
        if (owner && wv == 0) {  // the new token's value row, into the accumulators as the MFMAs lay them out
            static_assert(!PVM || sizeof(T) == 2, "four 16-bit columns per accumulator register group");
            const uint2 hv = ((const uint2*)vnew)[2 * cl + (sub & 1)];  // columns 8*cl + 4*(sub%2) .. +3
            const float v4[4] = {bf16_lo(hv.x), bf16_hi(hv.x), bf16_lo(hv.y), bf16_hi(hv.y)};
#pragma unroll
            for (int mf = 0; mf < 4; ++mf) {
                const float p = joined_weight(((const uint32_t*)xs)[(2 * mf + (sub >> 1)) * CS + cnt_c]);
#pragma unroll
                for (int r = 0; r < 4; ++r) cacc[mf][r] = fmaf(p, v4[r], cacc[mf][r]);
            }
        }
    } else if (owner && wv == 0 && sub == 0) {  // the new token's value row
        float vvals[EPV];
        unpack16<T>(((const uint4*)vnew)[cl], vvals);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float p = xs[g * CS + cnt_c];
#pragma unroll
            for (int e = 0; e < EPV; ++e) acc[g][e] = fmaf(p, vvals[e], acc[g][e]);
        }
    }
    // Partial outputs of the waves meet in LDS.  Few accumulators per lane: the rows of one wave-wide load
    // (RPW lane groups) are folded with exchanges, lane group 0 stores.  Many (4 or 8 query heads): the fold is a
    // reduce-scatter, every lane group ends up with 1/RPW of the sums and stores those.  The 8-wave
    // workgroup stores later, into the logit area, once nobody reads logits any more (see below).
    constexpr int HV = G * EPV / RPW;  // sums a lane holds after the reduce-scatter
    constexpr bool RS = G >= 4;        // many accumulators per lane: reduce-scatter fold
    float fin[RS ? HV : 1];
    int off = 0;
    auto store_fin = [&](float* row) {  // this lane's sums -> its places in a [G][D] row of partial outputs
        if constexpr (PVM) {  // the MFMAs summed over the lane groups already: 16 sums per lane, each (head, column) once
#pragma unroll
            for (int mf = 0; mf < 4; ++mf)
                *(float4*)&row[(2 * mf + (sub >> 1)) * D + cl * EPV + 4 * (sub & 1)] =
                    make_float4(cacc[mf][0], cacc[mf][1], cacc[mf][2], cacc[mf][3]);
        } else if constexpr (RS) {
#pragma unroll
            for (int i4 = 0; i4 < HV / 4; ++i4) {
                const int fi = off + 4 * i4;
                *(float4*)&row[(fi / EPV) * D + cl * EPV + (fi % EPV)] =
                    make_float4(fin[4 * i4], fin[4 * i4 + 1], fin[4 * i4 + 2], fin[4 * i4 + 3]);
            }
        } else if (sub == 0) {  // folded over the lane groups with exchanges: group 0 has the sums
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) row[g * D + cl * EPV + e] = acc[g][e];
            }
        }
    };
    if constexpr (PVM) {
        if constexpr (!BIG) {
            store_fin(red_o + (size_t)wv * G * D);
            __syncthreads();  // red_o and stat are complete
        }
    } else if constexpr (RS) {
        constexpr int N = G * EPV;
        static_assert(HV % 4 == 0, "a lane group ends up with whole 16-byte pieces of output rows");
        float flat[N];
#pragma unroll
        for (int i = 0; i < N; ++i) flat[i] = acc[i / EPV][i % EPV];
        off = (lane & 32) ? N / 2 : 0;
        if constexpr (RPW == 2) {
            halve<N, 32>(flat, fin, lane);
        } else if constexpr (RPW == 4) {
            float t1[N / 2];
            halve<N, 32>(flat, t1, lane);
            halve<N / 2, 16>(t1, fin, lane);
            off += (lane & 16) ? HV : 0;
        } else {
            static_assert(RPW == 8, "2, 4 or 8 rows per wave-wide load");
            float t1[N / 2], t2[N / 4];
            halve<N, 32>(flat, t1, lane);
            halve<N / 2, 16>(t1, t2, lane);
            halve<N / 4, 8>(t2, fin, lane);
            off += ((lane & 16) ? N / 4 : 0) + ((lane & 8) ? HV : 0);
        }
        if constexpr (!BIG) {
            store_fin(red_o + (size_t)wv * G * D);
            __syncthreads();  // red_o and stat are complete
        }
    } else {
#pragma unroll
        for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) acc[g][e] += __shfl_xor(acc[g][e], o, kWave);
            }
        }
        if constexpr (!BIG) {
            store_fin(red_o + (size_t)wv * G * D);
            __syncthreads();  // red_o and stat are complete
        }
    }
    if (S == 1) {
        // the whole unit is here: accumulate the normalised score increment of all its query heads
        // The 8-wave workgroup has had no barrier since thread 0 published stat[]: a wave that found no V rows
        // of its own (a launch shaped for many more tokens than the unit holds) would read it too early.
        if constexpr (BIG && G >= 8) __syncthreads();
        float inv[G];
#pragma unroll
        for (int g = 0; g < G; ++g) inv[g] = 1.0f / (G >= 8 ? stat[4 * g + 3] : spe[2 * g + 1]);  // many heads: not kept in registers across the V stream
        float* we = a.ws_e + (size_t)u * G * a.cap;
        // whole-step launch: this lane's smallest candidate, as (order-preserving score key, ~position):
        // the lowest score leaves, the highest position among equal scores (lower positions are kept)
        unsigned long long best = ~0ull;
        int best_slot = -1;
        for (int t = tid; t < cnt; t += NT) {
            const int slot = (t == cnt_c) ? len0 : j0 + t;
            float df = 0.0f;
#pragma unroll
            for (int g = 0; g < G; ++g) df = fmaf(ys[g * CS + t], inv[g], df);
            if (evict_here) {
                // the scores are needed at once: read, add, keep the sum for the selection
                float f_new = df;
                int pj = q_pos;
                if (t == cnt_c) {
                    new_score = df;
                } else {
                    f_new = fu[slot] + df;
                    fu[slot] = f_new;
                    pj = pu[slot];
                }
                if (pj <= q_pos - a.fuse_w) {  // outside the recent window: a candidate
                    const unsigned long long pack = ((unsigned long long)float_key(f_new) << 32) | (uint32_t)(~(uint32_t)pj);
                    if (pack < best) {
                        best = pack;
                        best_slot = slot;
                    }
                }
                continue;
            }
            // existing scores take the increment as a fire-and-forget atomic add at the L2: no load,
            // no round trip (one add per address and launch, so the result is the plain fp32 sum)
            if (a.shared) we[slot] = df;  // summed over the layers by the launch that follows
            else if (t == cnt_c) fu[slot] = df;
            else unsafeAtomicAdd(&fu[slot], df);
        }
        const float* orows = red_o;
        if constexpr (BIG) {
            // 8 waves' partial outputs (32 KB and more) take the place of the logits: every wave is past the
            // V stream (attention weights in xs) and the loop above (increments in ys) after this barrier
            __syncthreads();
            store_fin(smem + (size_t)wv * G * D);
            __syncthreads();
            orows = smem;
        }
        for (int c = tid; c < G * D; c += NT) {
            float o_c = 0.0f;
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2) o_c += orows[w2 * G * D + c];
            a.out[u * G * D + c] = o_c / stat[4 * (c / D) + 1];
        }
        if (!evict_here) {
            if (tid == 0) {
                a.len[u] = m;
                if (a.shared) a.ws_m[u] = m;
                if (over) atomicAdd(a.ws_err, 1);  // more than one token over budget: appended, not evicted, reported
            }
            if (a.fuse_idx && !over) {  // within budget: untouched, identity then -1 padding
                int32_t* idx = a.fuse_idx + (size_t)u * a.fuse_k;
                for (int i = tid; i < a.fuse_k; i += NT) idx[i] = i < m ? i : -1;
            }
            return;
        }
        // ---- eviction by this workgroup (slot layout): the candidate with the smallest score leaves
        const unsigned long long mine = best;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long t2 = __shfl_xor(best, o, kWave);
            best = t2 < best ? t2 : best;
        }
        if (lane == 0) evict_min[wv] = best;
        if (tid == 0) evict_slot = -1;
        __syncthreads();  // also orders the score stores above before the one into the freed slot
        unsigned long long gbest = evict_min[0];
#pragma unroll
        for (int i = 1; i < NW; ++i) gbest = evict_min[i] < gbest ? evict_min[i] : gbest;
        // positions are unique, so exactly one lane's own candidate carries the winning pack
        if (gbest != ~0ull && mine == gbest) evict_slot = best_slot;
        __syncthreads();
        const int e = evict_slot;
        const int k = a.fuse_k;
        if (e < 0) {
            // nothing lies outside the window (positions not consecutive at the recent end): append after
            // all, leave the unit one over budget and report it, as the selection launch would
            if (wv == 0 && lane < LPR) ((uint4*)(a.K))[((size_t)u * a.cap + len0) * LPR + lane] = ((const uint4*)knew)[lane];
            if (wv == 1 && lane < LPR) ((uint4*)(a.V))[((size_t)u * a.cap + len0) * LPR + lane] = ((const uint4*)vnew)[lane];
            if (tid == 2 * kWave) {
                pu[len0] = q_pos;
                fu[len0] = new_score;
                a.len[u] = m;
                atomicAdd(a.ws_err, 1);
            }
            return;
        }
        if (e != len0) {  // e == len0: the new token itself leaves (only without a recent window)
            if (wv == 0 && lane < LPR) ((uint4*)(a.K))[((size_t)u * a.cap + e) * LPR + lane] = ((const uint4*)knew)[lane];
            if (wv == 1 && lane < LPR) ((uint4*)(a.V))[((size_t)u * a.cap + e) * LPR + lane] = ((const uint4*)vnew)[lane];
            if (tid == 2 * kWave) {
                pu[e] = q_pos;
                fu[e] = new_score;
            }
        }
        if (a.fuse_idx) {  // survivors by pre-compaction slot: the new token counts as slot k
            int32_t* idx = a.fuse_idx + (size_t)u * k;
            for (int i = tid; i < k; i += NT) idx[i] = (i == e) ? k : i;
        }
        if (tid == 0) a.len[u] = k;
        return;
    }
    // ---- S > 1: leave the un-normalised increments and a partial record per query head for the merge
    {
        float* we = a.ws_e + (size_t)u * G * a.cap;
        for (int t = tid; t < cnt; t += NT) {
            const int slot = (t == cnt_c) ? len0 : j0 + t;
#pragma unroll
            for (int g = 0; g < G; ++g) we[(size_t)g * a.cap + slot] = ys[g * CS + t];
        }
    }
    if (owner && tid == 0) a.ws_m[u] = m;  // tokens scored in this unit: the merge reads the length from here
    const float* orows = red_o;
    if constexpr (BIG) {  // as above: the waves' partial outputs take the place of the logits
        __syncthreads();
        store_fin(smem + (size_t)wv * G * D);
        __syncthreads();
        orows = smem;
    }
    float* part = a.ws_part + ((size_t)u * S + s) * G * PW;
    for (int c = tid; c < G * D; c += NT) {
        float o_c = 0.0f;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) o_c += orows[w2 * G * D + c];
        part[(c / D) * PW + (c % D)] = o_c;
    }
    if (tid < 4 * G) part[(tid >> 2) * PW + D + (tid & 3)] = stat[tid];
}

// (The 8-wave workgroup is compiled for four waves per SIMD, i.e. two per CU -- at most 128 registers per lane: with a few more its
// medium-length units lose the second workgroup that overlaps their statistics and folds, 67 -> 48 % of peak.)
template <typename T, int D, int NT, int G>
__global__ void __launch_bounds__(NT, NT >= 512 ? 4 : 1) decode_kernel(const DecodeArgs a) {
    decode_block<T, D, NT, G>(a);
    // Whole-step launch with the step number in device memory: every workgroup read the number when it
    // started, so the one that finishes last may move it on (and clears the ticket counter for the next launch).
    if (a.step_inc && threadIdx.x == 0) {
        if (atomicAdd(a.ws_ticket, 1) == (int)gridDim.x - 1) {
            *a.ws_ticket = 0;
            *a.step_inc += 1;
        }
    }
}

// Merge kernel, launched after the split kernel: gridDim.y workgroups per unit share the token range of
// the score update (each re-derives the few per-split weights); the first also writes the outputs.  The
// unit's token count comes from the split kernel's record, not from len, which the first workgroup updates.
template <int D, int NT, int G>
__global__ void __launch_bounds__(NT) decode_merge_kernel(const DecodeArgs a) {
    __shared__ float w_p[G * kDecodeMaxSplits], w_e[G * kDecodeMaxSplits];
    const int64_t u = blockIdx.x;
    const int m = a.ws_m[u];
    if (m <= 0) {  // skipped by the split kernel
        // the selection may still evict from this unit (it is full): its slices' minima come from the scores as they are
        const int n = a.len[u];
        if (a.pre_slices > 0 && !a.shared && n == a.pre_k + 1) {
            const int per = ((n + (int)gridDim.y - 1) / (int)gridDim.y + NT - 1) / NT * NT;
            const int j_begin = (int)blockIdx.y * per;
            scan_slice_min<NT>(a, u, n, j_begin, j_begin + per, (int)blockIdx.y);
        }
        return;
    }
    const int per = ((m + (int)gridDim.y - 1) / (int)gridDim.y + NT - 1) / NT * NT;
    const int j_begin = (int)blockIdx.y * per;
    merge_unit<D, NT, G>(a, u, m - 1, w_p, w_e, j_begin, j_begin + per, blockIdx.y == 0, (int)blockIdx.y);
}

// Shared score function (the paper's ablation of one score for all layers,
// Sec. 4.4.1): every layer's contribution to token j of sequence/head bh is
// summed in layer order, and every layer's copy of the score takes the same
// sum, so all copies stay bit-identical and all layers evict the same tokens.
constexpr int kShareThreads = 256;
__global__ void __launch_bounds__(kShareThreads) share_kernel(const ShareArgs a) {
    const int bh = blockIdx.x;
    const int j = blockIdx.y * kShareThreads + threadIdx.x;
    const int m = a.m[bh];
    bool same = true;
    for (int l = 1; l < a.L; ++l) same = same && (a.m[(size_t)l * a.BH + bh] == m);
    if (!same) {  // layers that hold different token counts cannot share a score: leave them, report
        if (j == 0 && blockIdx.z == 0) atomicAdd(a.ws_err, 1);
        return;
    }
    if (j >= m || m > a.cap) return;  // m == 0: the decode launch skipped (and reported) these units
    const size_t stride = (size_t)a.BH * a.cap, at = (size_t)bh * a.cap + j;
    if (a.inc) {
        // decode: a workgroup per layer (gridDim.z = L); each adds up all layers' increments itself, in layer
        // order (every copy gets the same bits), and updates its own layer's score.  A unit's increments sit
        // inc_unit floats apart (one row per query head, the sum in the first).
        float s = 0.0f;
        int l = 0;
        for (; l + 4 <= a.L; l += 4) {  // four loads in flight
            const float v0 = a.inc[((size_t)(l + 0) * a.BH + bh) * a.inc_unit + j];
            const float v1 = a.inc[((size_t)(l + 1) * a.BH + bh) * a.inc_unit + j];
            const float v2 = a.inc[((size_t)(l + 2) * a.BH + bh) * a.inc_unit + j];
            const float v3 = a.inc[((size_t)(l + 3) * a.BH + bh) * a.inc_unit + j];
            s = (((s + v0) + v1) + v2) + v3;
        }
        for (; l < a.L; ++l) s += a.inc[((size_t)l * a.BH + bh) * a.inc_unit + j];
        float* f = a.score + (size_t)blockIdx.z * stride + at;
        *f = (j == m - 1) ? s : *f + s;  // m-1: the token appended by this step
        return;
    }
    // prompt: the layers' scores are summed in place, so one thread owns a token in every layer
    float s = 0.0f;
    for (int l = 0; l < a.L; ++l) s += a.score[l * stride + at];
    for (int l = 0; l < a.L; ++l) a.score[l * stride + at] = s;
}

hipError_t launch_share(const ShareArgs& a, hipStream_t stream) {
    const dim3 grid((unsigned)a.BH, (unsigned)((a.cap + kShareThreads - 1) / kShareThreads), a.inc ? (unsigned)a.L : 1u);
    hipLaunchKernelGGL(share_kernel, grid, dim3(kShareThreads), 0, stream, a);
    return hipGetLastError();
}

// -------------------------------------------------------------------- host
static int rows_per_block(int32_t d, int32_t dtype) {
    const int epv = dtype == KF_F32 ? 4 : 8;
    const int lpr = d / epv;
    return (kWave / lpr) * (kDecodeThreads / kWave);
}

static size_t decode_lds_bytes(int32_t G, int64_t chunk, int32_t d) {
    return (size_t)(2 * G * (chunk + 1) + 3 + kDecodeRedWaves * G * d) * sizeof(float);
}
// ... of the 8-wave workgroup: its waves' partial outputs reuse the logit area
static size_t decode_lds_bytes_big(int32_t G, int64_t chunk, int32_t d) {
    const size_t logits = (size_t)(2 * G * (chunk + 1) + 3) * sizeof(float);
    const size_t outs = (size_t)(kDecodeThreadsBig / kWave) * G * d * sizeof(float);
    return logits > outs ? logits : outs;
}

// Chooses the number of splits S of a unit's token range.
//
// One workgroup per unit (S = 1) is the fastest shape whenever it is possible:
// the unit is finished by the workgroup that streamed it -- no increments and
// partial records through memory, no merge launch -- which measures 6-15 %
// faster than any split (gptj 82 vs 89 us, long 790 vs 875 us).  It needs the
// unit's 2*G logit rows in LDS -- twice per CU for the 4-wave workgroup, once
// (up to most of a CU's 160 KB) for the 8-wave workgroup that takes the units
// beyond that and the longer ones with 4 or 8 query heads (16 k tokens with one
// head: 87 % of the HBM peak against 75 % in splits) -- and enough units to
// fill the chip (at 256 units of one head a split wins again).
//
// Otherwise the launch is bandwidth bound and every workgroup does the same
// amount of work, so what matters is how evenly U*S workgroups spread over the
// compute units: the cost of a candidate is the number of workgroups the
// busiest unit gets times the tokens (plus a fixed per-workgroup overhead) each
// of them streams.  Candidates that leave the chip with too few workgroups to
// hide memory latency are skipped when a better filled one exists.  With G
// query heads per unit a split workgroup keeps G logit rows in LDS, so its
// chunk is at most 1/G of the single-head maximum.
// Enough workgroups per unit that each walks at most ~8 strides of the token range.
int32_t decode_merge_slices(int32_t S, int32_t chunk) {
    const int64_t tokens = (int64_t)S * chunk;
    int64_t slices = (tokens + 8 * kDecodeThreads - 1) / (8 * kDecodeThreads);
    if (slices > 16) slices = 16;
    if (slices < 1) slices = 1;
    return (int32_t)slices;
}

DecodePlan plan_decode(int64_t U, int32_t m, int32_t d, int32_t dtype, int32_t G) {
    DecodePlan p;
    const int rpb = rows_per_block(d, dtype);
    const int64_t rows = m > 1 ? m - 1 : 1;  // cache rows; the new token rides with the last split
    if ((G == 4 || (G == 8 && dtype != KF_F32)) && U >= kDecodeBigMinUnits) {
        // one workgroup per unit, up to one per CU with the unit's 2 x G logit rows in most of the CU's LDS
        const int64_t chunk = (rows + rpb - 1) / rpb * rpb;
        if (decode_lds_bytes_big(G, chunk, d) <= kDecodeLdsWhole) {
            p.S = 1;
            p.chunk = (int32_t)chunk;
            p.lds_bytes = decode_lds_bytes_big(G, chunk, d);
            return p;
        }
    }
    if (G <= 4 && U >= kDecodeSingleMinUnits) {
        const int64_t chunk = (rows + rpb - 1) / rpb * rpb;
        if (decode_lds_bytes(G, chunk, d) <= kDecodeLdsPair) {
            p.S = 1;
            p.chunk = (int32_t)chunk;
            p.lds_bytes = decode_lds_bytes(G, chunk, d);
            return p;
        }
        if (decode_lds_bytes_big(G, chunk, d) <= kDecodeLdsWhole) {  // one 8-wave workgroup per CU
            p.S = 1;
            p.chunk = (int32_t)chunk;
            p.lds_bytes = decode_lds_bytes_big(G, chunk, d);
            return p;
        }
    }
    // LDS of a split workgroup: within 64 KB less the small static arrays
    const int lds_rows = (int)((kDecodeLdsBudget - 3 * sizeof(float) - (size_t)kDecodeRedWaves * G * d * sizeof(float)) /
                               (2 * G * sizeof(float))) - 1;
    int max_chunk = kDecodeMaxChunk / G;
    if (lds_rows < max_chunk) max_chunk = lds_rows / rpb * rpb;
    if (G == 4 || (G == 8 && dtype != KF_F32)) {
        // these splits run in 8-wave workgroups whose partial outputs reuse the logit area: rows up to two
        // such workgroups per CU (8 heads, 9830 tokens: 20 splits of 496 rows 39 %, 10 of 992 rows 47 % of peak)
        max_chunk = 2 * kDecodeMaxChunk / G;
        while (max_chunk > rpb && decode_lds_bytes_big(G, max_chunk, d) > kDecodeLdsPair) max_chunk -= rpb;
    }
    const int min_chunk = kDecodeMinChunk < max_chunk ? kDecodeMinChunk : max_chunk;
    int64_t s_hi = (m + min_chunk - 1) / min_chunk;
    int64_t s_lo = (rows + max_chunk - 1) / max_chunk;  // the new token takes no cache row
    if (s_hi > kDecodeMaxSplits) s_hi = kDecodeMaxSplits;
    if (s_lo < 1) s_lo = 1;
    if (s_hi < s_lo) s_hi = s_lo;
    // 4 and 8 query heads: a workgroup's fixed work (statistics and folds of G heads, G partial records) is
    // large, so few units are cut into few, long splits for 8-wave workgroups, one per CU (8 cached heads x
    // 8 sequences x 2048 tokens, 8 query heads each: 16 splits of 128 rows 73 us, 4 of 512 rows 52 us)
    const int64_t min_blocks = (G >= 4) ? kDecodeMinBlocksGrouped : kDecodeMinBlocks;
    int64_t best_S = s_lo;
    double best_cost = 0.0;
    bool best_filled = false;
    for (int64_t S = s_lo; S <= s_hi && S <= s_lo + 63; ++S) {
        int64_t chunk = (rows + S - 1) / S;
        chunk = (chunk + rpb - 1) / rpb * rpb;
        if (chunk > max_chunk) continue;  // rounding up to whole block-wide loads overshot: take more splits
        const int64_t blocks = U * S;
        const int64_t per_cu = (blocks + kComputeUnits - 1) / kComputeUnits;
        const double cost = (double)per_cu * (double)(chunk + kDecodeBlockOverheadTokens);
        const bool filled = blocks >= min_blocks;
        if (best_cost == 0.0 || (filled && !best_filled) || (filled == best_filled && cost < best_cost)) {
            best_S = S;
            best_cost = cost;
            best_filled = filled;
        }
    }
    int64_t chunk = (rows + best_S - 1) / best_S;
    chunk = (chunk + rpb - 1) / rpb * rpb;
    p.S = (int32_t)best_S;
    p.chunk = (int32_t)chunk;
    p.lds_bytes = decode_lds_bytes(G, chunk, d);
    return p;
}

template <typename T, int D, int G>
static hipError_t launch_decode_g(const DecodeArgs& a, int64_t U, size_t lds, hipStream_t st, bool merge) {
    const dim3 grid((unsigned)(U * a.S)), block(kDecodeThreads);
    if constexpr (G == 4 || (G == 8 && MfmaLogits<T, G>::value)) {
        // One split with 4 or 8 query heads: short units keep the 4-wave workgroup (three or more fit a CU),
        // longer ones take 8 waves (two per CU while the logits stay under ~75 KB, then one with most of the CU's
        // LDS).  Measured at 2048 units, d = 128, 8 heads: 512 tokens 51 % (4 waves) vs 49 % (8) vs 36 % (16 waves);
        // 1024 tokens 49 / 62 / 49 %; 2048 tokens - / 62 / 58 %.  4 heads: 512 tokens 67 % (4 waves) vs 63 % (8);
        // 1024 tokens 71 / 74.5 %; 2048 tokens 73-78 / 80 %.  Splits (few units) take the 8 waves from 16 KB
        // of logits on: 64 units x 4 splits of 512 rows, 8 heads 61 -> 52 us, 4 heads 43 -> 39 us.
        const size_t logits = (size_t)2 * G * (a.chunk + 1) * sizeof(float);
        const size_t big_from = a.S > 1 ? kDecodeBigMinLogitsSplit : (G == 8 ? kDecodeBigMinLogits8 : kDecodeBigMinLogits4);
        if (logits > big_from) {
            const size_t lds_big = decode_lds_bytes_big(G, a.chunk, D);
            if (lds_big > kDecodeLdsWhole) return hipErrorInvalidValue;
            hipLaunchKernelGGL((decode_kernel<T, D, kDecodeThreadsBig, G>), grid, dim3(kDecodeThreadsBig), lds_big, st, a);
            hipError_t e2 = hipGetLastError();
            if (e2 == hipSuccess && a.S > 1 && merge) {
                const int32_t slices = decode_merge_slices(a.S, a.chunk);
                hipLaunchKernelGGL((decode_merge_kernel<D, kDecodeThreads, G>), dim3((unsigned)U, (unsigned)slices), block, 0, st, a);
                e2 = hipGetLastError();
            }
            return e2;
        }
    }
    lds = decode_lds_bytes(G, a.chunk, D);  // what this workgroup shape needs for the plan's chunk
    if constexpr (G <= 2) {
        if (a.S == 1 && lds > kDecodeLdsPair) {  // a unit too long for two workgroups per CU: one of 8 waves
            const size_t lds_big = decode_lds_bytes_big(G, a.chunk, D);
            if (lds_big > kDecodeLdsWhole) return hipErrorInvalidValue;
            hipLaunchKernelGGL((decode_kernel<T, D, kDecodeThreadsBig, G>), grid, dim3(kDecodeThreadsBig), lds_big, st, a);
            return hipGetLastError();
        }
    }
    if (lds > kDecodeLdsPair) return hipErrorInvalidValue;
    hipLaunchKernelGGL((decode_kernel<T, D, kDecodeThreads, G>), grid, block, lds, st, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.S > 1 && merge) {
        const int32_t slices = decode_merge_slices(a.S, a.chunk);
        hipLaunchKernelGGL((decode_merge_kernel<D, kDecodeThreads, G>), dim3((unsigned)U, (unsigned)slices), block, 0, st, a);
        e = hipGetLastError();
    }
    return e;
}

template <typename T, int D>
static hipError_t launch_decode_t(const DecodeArgs& a, int64_t U, size_t lds, hipStream_t st, bool merge) {
    switch (a.G) {
        case 1: return launch_decode_g<T, D, 1>(a, U, lds, st, merge);
        case 2: return launch_decode_g<T, D, 2>(a, U, lds, st, merge);
        case 4: return launch_decode_g<T, D, 4>(a, U, lds, st, merge);
        case 8: return launch_decode_g<T, D, 8>(a, U, lds, st, merge);
        default: return hipErrorInvalidValue;
    }
}

static hipError_t launch_decode_any(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                                    hipStream_t stream, bool merge) {
    if (a.S > kDecodeMaxSplits) return hipErrorInvalidValue;
    if (dtype == KF_BF16) {
        if (d == 64) return launch_decode_t<bf16_t, 64>(a, U, lds_bytes, stream, merge);
        if (d == 128) return launch_decode_t<bf16_t, 128>(a, U, lds_bytes, stream, merge);
        if (d == 256) return launch_decode_t<bf16_t, 256>(a, U, lds_bytes, stream, merge);
    } else if (dtype == KF_F16) {
        if (d == 64) return launch_decode_t<f16_t, 64>(a, U, lds_bytes, stream, merge);
        if (d == 128) return launch_decode_t<f16_t, 128>(a, U, lds_bytes, stream, merge);
        if (d == 256) return launch_decode_t<f16_t, 256>(a, U, lds_bytes, stream, merge);
    } else {
        if (d == 64) return launch_decode_t<float, 64>(a, U, lds_bytes, stream, merge);
        if (d == 128) return launch_decode_t<float, 128>(a, U, lds_bytes, stream, merge);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_decode(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                         hipStream_t stream) {
    return launch_decode_any(a, U, d, dtype, lds_bytes, stream, true);
}

hipError_t launch_decode_split(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                               hipStream_t stream) {
    return launch_decode_any(a, U, d, dtype, lds_bytes, stream, false);
}

}  // namespace kf
