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
// contiguous kilobyte), keeps the logits in LDS, forms the two softmaxes'
// local statistics while its first V tile is already in flight, then streams
// its V rows.  With S == 1 it finishes the unit itself.  With S > 1 it leaves a
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
constexpr int kDecodeMaxChunk = 4096;   // tokens per split the LDS arrays are sized for
constexpr int kDecodeMinBlocks = 1024;  // workgroups wanted on the chip
constexpr int kComputeUnits = 256;                      // MI355X
constexpr int kDecodeBlockOverheadTokens = 48;          // fixed cost of a workgroup, in tokens' worth of time
constexpr int kDecodeMinChunk = 128;

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

// Block-wide max / sum of two values at once (one pair of barriers).
template <int NT>
__device__ __forceinline__ void block_max2(float& x, float& y, float* red /* [2*NT/64] */) {
    x = wave_max(x);
    y = wave_max(y);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        red[2 * (threadIdx.x >> 6)] = x;
        red[2 * (threadIdx.x >> 6) + 1] = y;
    }
    __syncthreads();
    x = red[0];
    y = red[1];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) {
        x = fmaxf(x, red[2 * i]);
        y = fmaxf(y, red[2 * i + 1]);
    }
}
template <int NT>
__device__ __forceinline__ void block_sum2(float& x, float& y, float* red) {
    x = wave_sum(x);
    y = wave_sum(y);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        red[2 * (threadIdx.x >> 6)] = x;
        red[2 * (threadIdx.x >> 6) + 1] = y;
    }
    __syncthreads();
    x = red[0];
    y = red[1];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) {
        x += red[2 * i];
        y += red[2 * i + 1];
    }
}

template <typename T, int D, int NT>
__global__ void __launch_bounds__(NT) decode_kernel(const DecodeArgs a) {
    constexpr int EPV = ElemTraits<T>::kPerVec;  // elements per 16-byte vector
    constexpr int LPR = D / EPV;                 // lanes that share one row
    constexpr int RPW = kWave / LPR;             // rows per wave-wide load
    constexpr int NW = NT / kWave;
    constexpr int RPB = RPW * NW;                // rows per block-wide load
    constexpr int UNR = kDecodeUnroll;             // independent loads in flight per lane
    constexpr int TILE = RPB * UNR;              // rows per tile of the workgroup
    constexpr int PW = D + 4;                    // floats in a partial record
    constexpr size_t ROWB = (size_t)D * sizeof(T);
    static_assert(LPR <= 32 && D <= NT, "row must fit half a wave, output a block");

    extern __shared__ float smem[];
    float* xs = smem;                // [chunk+1] logits, then attention weights (+1: the new token)
    float* ys = smem + a.chunk + 1;  // [chunk+1] perturbed logits / tau, then their exponentials
    float* red_o = ys + a.chunk + 1; // [NW][D] per-wave output partials
    __shared__ float red_s[2 * NW];

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
    const int len0 = a.len[u];
    const int m = len0 + 1;
    if (len0 < 0 || len0 >= a.cap || len0 > S * a.chunk) {
        // no room for the new token (or a launch shaped for fewer tokens):
        // leave the unit alone and report it
        if (s == 0) {
            if (tid < D) a.out[u * D + tid] = 0.0f;
            if (tid == 0) {
                atomicAdd(a.ws_err, 1);
                if (a.shared) a.ws_m[u] = 0;
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
    const T* qu = (const T*)a.q + (size_t)u * D;
    const char* knew = (const char*)a.k_new + (size_t)u * ROWB;
    const char* vnew = (const char*)a.v_new + (size_t)u * ROWB;
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;

    // ---- append: the last split stores the new row (nobody reads it back in this launch)
    if (owner) {
        if (wv == 0 && lane < LPR) ((uint4*)(a.K))[((size_t)u * a.cap + len0) * LPR + lane] = ((const uint4*)knew)[lane];
        if (wv == 1 && lane < LPR) ((uint4*)(a.V))[((size_t)u * a.cap + len0) * LPR + lane] = ((const uint4*)vnew)[lane];
        if (tid == 2 * kWave) pu[len0] = q_pos;
    }

    QueryPiece<T> qp;
    qp.load(((const uint4*)qu)[cl]);

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
    auto logits_of = [&](int base) {
        float p[UNR];
#pragma unroll
        for (int i = 0; i < UNR; ++i) p[i] = qp.dot(cur[i]);
#pragma unroll
        for (int i = 0; i < UNR; ++i) p[i] = group_sum<LPR>(p[i]);
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int j = base + i * RPB + sub;
            if (cl == 0 && j < j1) xs[j - j0] = p[i] * a.scale;
        }
    };
    {
        int base = base0;
        if (base < j1) load_tile(Ku, base, cur);
        // steady state: the next tile needs no bounds checks, so the loop body is
        // branch-free and only the older tile's loads are waited for
        while (plain(base + TILE)) {
            load_plain(Ku, base + TILE, nxt);
            logits_of(base);
#pragma unroll
            for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
            base += TILE;
        }
        while (base < j1) {  // the last one or two tiles of the split
            if (base + TILE < j1) load_edge(Ku, base + TILE, nxt);
            logits_of(base);
#pragma unroll
            for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
            base += TILE;
        }
    }
    if (owner && wv == 0) {  // the new token's own logit (distance 0: no position bias)
        const float p = group_sum<LPR>(qp.dot(((const uint4*)knew)[cl]));
        if (lane == 0) xs[cnt_c] = p * a.scale;
    }
    // first V tile: in flight while the softmax statistics are formed
    if (base0 < j1) load_tile(Vu, base0, cur);
    __syncthreads();

    // ---- phase 1.5: position bias, logit adjustment, the two softmaxes' statistics
    const float slope = a.slopes ? a.slopes[h] : 0.0f;
    uint32_t rkey = 0;
    if (a.noise == kNoiseGumbel || a.noise == kNoiseGaussian)
        rkey = row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)h), (uint32_t)q_pos);
    float mx = -INFINITY, my = -INFINITY;
    for (int t = tid; t < cnt; t += NT) {
        const int pj = (t == cnt_c) ? q_pos : pu[j0 + t];  // t == cnt_c: the new token
        // base-2 domain: x2 = log2(e)*x, y2 = log2(e)*(x + zeta)/tau
        const int dist = a.new_pos ? (len0 - (j0 + t)) : (q_pos - pj);  // the new token: 0 either way
        const float x = (xs[t] - slope * (float)((t == cnt_c) ? 0 : dist)) * kLog2e;
        const float y = (x + zeta_log2e(a.noise, rkey, (uint32_t)pj)) * inv_tau;
        xs[t] = x;
        ys[t] = y;
        mx = fmaxf(mx, x);
        my = fmaxf(my, y);
    }
    block_max2<NT>(mx, my, red_s);
    float sp = 0.0f, se = 0.0f;
    for (int t = tid; t < cnt; t += NT) {
        const float p = hw_exp2(xs[t] - mx);
        const float e = hw_exp2(ys[t] - my);
        xs[t] = p;
        ys[t] = e;
        sp += p;
        se += e;
    }
    block_sum2<NT>(sp, se, red_s);  // its barriers also publish the attention weights in xs
    // (The score increments in ys are written out after the V stream: stores issued here
    // would have to drain before the first V tile could be consumed.)

    // ---- phase 2: stream V, weighted sum
    float acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = 0.0f;
    auto weigh = [&](int base) {
        float p[UNR];
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int j = base + i * RPB + sub;
            p[i] = (j < j1) ? xs[j - j0] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            float vvals[EPV];
            unpack16<T>(cur[i], vvals);
#pragma unroll
            for (int e = 0; e < EPV; ++e) acc[e] = fmaf(p[i], vvals[e], acc[e]);
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
    if (owner && wv == 0 && sub == 0) {  // the new token's value row
        float vvals[EPV];
        unpack16<T>(((const uint4*)vnew)[cl], vvals);
        const float p = xs[cnt_c];
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[e] = fmaf(p, vvals[e], acc[e]);
    }
    // rows of one wave-wide load live in different lane groups: fold them
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
    }
    if (sub == 0) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) red_o[wv * D + cl * EPV + e] = acc[e];
    }
    __syncthreads();
    float o_c = 0.0f;
    if (tid < D) {
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) o_c += red_o[w2 * D + tid];
    }

    if (S == 1) {
        // the whole unit is here: accumulate the normalised score increment
        const float inv = 1.0f / se;
        float* we = a.ws_e + (size_t)u * a.cap;
        for (int t = tid; t < cnt; t += NT) {
            const int slot = (t == cnt_c) ? len0 : j0 + t;
            // existing scores take the increment as a fire-and-forget atomic add at the L2: no load,
            // no round trip (one add per address and launch, so the result is the plain fp32 sum)
            if (a.shared) we[slot] = ys[t] * inv;  // summed over the layers by the launch that follows
            else if (t == cnt_c) fu[slot] = ys[t] * inv;
            else unsafeAtomicAdd(&fu[slot], ys[t] * inv);
        }
        if (tid < D) a.out[u * D + tid] = o_c / sp;
        if (tid == 0) {
            a.len[u] = m;
            if (a.shared) a.ws_m[u] = m;
        }
        return;
    }
    {
        float* we = a.ws_e + (size_t)u * a.cap;
        for (int t = tid; t < cnt; t += NT) we[(t == cnt_c) ? len0 : j0 + t] = ys[t];
    }

    // ---- S > 1: leave a partial record for the merge
    float* part = a.ws_part + ((size_t)u * S + s) * PW;
    if (tid < D) part[tid] = o_c;
    if (tid == 0) {
        part[D + 0] = mx;
        part[D + 1] = sp;
        part[D + 2] = my;
        part[D + 3] = se;
    }
}

// Merge kernel: one workgroup per unit, launched after the split kernel.
template <int D, int NT>
__global__ void __launch_bounds__(NT) decode_merge_kernel(const DecodeArgs a) {
    __shared__ float red_s[NT / kWave];
    __shared__ float w_p[kDecodeMaxSplits], w_e[kDecodeMaxSplits];
    const int64_t u = blockIdx.x;
    const int len0 = a.len[u];
    if (len0 < 0 || len0 >= a.cap || len0 > a.S * a.chunk) return;  // skipped by the split kernel too
    merge_unit<D, NT>(a, u, len0, red_s, w_p, w_e);
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
        if (j == 0) atomicAdd(a.ws_err, 1);
        return;
    }
    if (j >= m || m > a.cap) return;  // m == 0: the decode launch skipped (and reported) these units
    const size_t stride = (size_t)a.BH * a.cap, at = (size_t)bh * a.cap + j;
    const float* src = a.inc ? a.inc : a.score;
    float s = 0.0f;
    for (int l = 0; l < a.L; ++l) s += src[l * stride + at];
    const bool fresh = !a.inc || j == m - 1;  // prompt scores, or the token appended by this step
    for (int l = 0; l < a.L; ++l) {
        float* f = a.score + l * stride + at;
        *f = fresh ? s : *f + s;
    }
}

hipError_t launch_share(const ShareArgs& a, hipStream_t stream) {
    const dim3 grid((unsigned)a.BH, (unsigned)((a.cap + kShareThreads - 1) / kShareThreads));
    hipLaunchKernelGGL(share_kernel, grid, dim3(kShareThreads), 0, stream, a);
    return hipGetLastError();
}

// -------------------------------------------------------------------- host
static int rows_per_block(int32_t d, int32_t dtype) {
    const int epv = dtype == KF_F32 ? 4 : 8;
    const int lpr = d / epv;
    return (kWave / lpr) * (kDecodeThreads / kWave);
}

// Chooses the number of splits S.  The launch is bandwidth bound and every
// workgroup does the same amount of work, so what matters is how evenly U*S
// workgroups spread over the compute units: the cost of a candidate is the
// number of workgroups the busiest unit gets times the tokens (plus a fixed
// per-workgroup overhead) each of them streams.  Candidates that leave the chip
// with too few workgroups to hide memory latency are skipped when a better
// filled one exists.
DecodePlan plan_decode(int64_t U, int32_t m, int32_t d, int32_t dtype) {
    DecodePlan p;
    const int rpb = rows_per_block(d, dtype);
    const int64_t rows = m > 1 ? m - 1 : 1;  // cache rows; the new token rides with the last split
    int64_t s_hi = (m + kDecodeMinChunk - 1) / kDecodeMinChunk;
    int64_t s_lo = (m + kDecodeMaxChunk - 1) / kDecodeMaxChunk;
    if (s_hi > kDecodeMaxSplits) s_hi = kDecodeMaxSplits;
    if (s_lo < 1) s_lo = 1;
    if (s_hi < s_lo) s_hi = s_lo;
    int64_t best_S = s_lo;
    double best_cost = 0.0;
    bool best_filled = false;
    for (int64_t S = s_lo; S <= s_hi && S <= s_lo + 63; ++S) {
        int64_t chunk = (rows + S - 1) / S;
        chunk = (chunk + rpb - 1) / rpb * rpb;
        const int64_t blocks = U * S;
        const int64_t per_cu = (blocks + kComputeUnits - 1) / kComputeUnits;
        const double cost = (double)per_cu * (double)(chunk + kDecodeBlockOverheadTokens);
        const bool filled = blocks >= kDecodeMinBlocks;
        if (S == s_lo || (filled && !best_filled) || (filled == best_filled && cost < best_cost)) {
            best_S = S;
            best_cost = cost;
            best_filled = filled;
        }
    }
    int64_t chunk = (rows + best_S - 1) / best_S;
    chunk = (chunk + rpb - 1) / rpb * rpb;
    p.S = (int32_t)best_S;
    p.chunk = (int32_t)chunk;
    p.lds_bytes = (size_t)(2 * (chunk + 1) + (kDecodeThreads / kWave) * d) * sizeof(float);
    return p;
}

template <typename T, int D>
static hipError_t launch_decode_t(const DecodeArgs& a, int64_t U, size_t lds, hipStream_t st, bool merge) {
    const dim3 grid((unsigned)(U * a.S)), block(kDecodeThreads);
    hipLaunchKernelGGL((decode_kernel<T, D, kDecodeThreads>), grid, block, lds, st, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.S > 1 && merge) {
        hipLaunchKernelGGL((decode_merge_kernel<D, kDecodeThreads>), dim3((unsigned)U), block, 0, st, a);
        e = hipGetLastError();
    }
    return e;
}

static hipError_t launch_decode_any(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                                    hipStream_t stream, bool merge) {
    if (a.chunk > kDecodeMaxChunk || a.S > kDecodeMaxSplits) return hipErrorInvalidValue;
    if (dtype == KF_BF16) {
        if (d == 64) return launch_decode_t<bf16_t, 64>(a, U, lds_bytes, stream, merge);
        if (d == 128) return launch_decode_t<bf16_t, 128>(a, U, lds_bytes, stream, merge);
        if (d == 256) return launch_decode_t<bf16_t, 256>(a, U, lds_bytes, stream, merge);
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
