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

namespace kf {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeMaxChunk = 4096;   // tokens per split the LDS arrays are sized for
constexpr int kDecodeMaxSplits = 256;   // <= kDecodeThreads: one thread per split in the merge
#ifndef KF_DECODE_MIN_BLOCKS
#define KF_DECODE_MIN_BLOCKS 1024
#endif
constexpr int kDecodeMinBlocks = KF_DECODE_MIN_BLOCKS;  // workgroups wanted on the chip
constexpr int kComputeUnits = 256;                      // MI355X
constexpr int kDecodeBlockOverheadTokens = 48;          // fixed cost of a workgroup, in tokens' worth of time
constexpr int kDecodeMinChunk = 128;

#ifndef KF_DECODE_UNROLL
#define KF_DECODE_UNROLL 4
#endif

// Merges the S partial records of unit u: rescales every split's un-normalised
// output and score increments to the unit-wide maxima, normalises, accumulates
// the scores and publishes the new length.  Called by a whole workgroup.
template <int D, int NT>
__device__ __forceinline__ void merge_unit(const DecodeArgs& a, int64_t u, int len0, float* red_s, float* w_p,
                                           float* w_e) {
    constexpr int PW = D + 4;
    const int tid = threadIdx.x, S = a.S, m = len0 + 1;
    const float* parts = a.ws_part + (size_t)u * S * PW;
    float* fu = a.score + (size_t)u * a.cap;
    float pmx = -INFINITY, psp = 0.0f, pmy = -INFINITY, pse = 0.0f;
    if (tid < S) {
        const float* r = parts + (size_t)tid * PW + D;
        pmx = r[0];
        psp = r[1];
        pmy = r[2];
        pse = r[3];
    }
    const float Mx = block_max<NT>(pmx, red_s);
    const float My = block_max<NT>(pmy, red_s);
    const float wp = (psp > 0.0f) ? expf(pmx - Mx) : 0.0f;  // empty splits weigh nothing
    const float we_ = (pse > 0.0f) ? expf(pmy - My) : 0.0f;
    const float sumP = block_sum<NT>(wp * psp, red_s);
    const float sumE = block_sum<NT>(we_ * pse, red_s);
    if (tid < S) {
        w_p[tid] = wp;
        w_e[tid] = we_;
    }
    __syncthreads();
    if (tid < D) {
        float o = 0.0f;
        for (int ss = 0; ss < S; ++ss) o = fmaf(w_p[ss], parts[(size_t)ss * PW + tid], o);
        a.out[u * D + tid] = o / sumP;
    }
    const float* we = a.ws_e + (size_t)u * a.cap;
    const float inv = 1.0f / sumE;
    for (int j = tid; j < m; j += NT) {
        const float prev = (j == len0) ? 0.0f : fu[j];
        fu[j] = prev + we[j] * (w_e[j / a.chunk] * inv);
    }
    if (tid == 0) a.len[u] = m;
}

template <typename T, int D, int NT>
__global__ void __launch_bounds__(NT) decode_kernel(const DecodeArgs a) {
    constexpr int EPV = ElemTraits<T>::kPerVec;  // elements per 16-byte vector
    constexpr int LPR = D / EPV;                 // lanes that share one row
    constexpr int RPW = kWave / LPR;             // rows per wave-wide load
    constexpr int NW = NT / kWave;
    constexpr int RPB = RPW * NW;                // rows per block-wide load
    constexpr int UNR = KF_DECODE_UNROLL;        // independent loads in flight per lane
    constexpr int PW = D + 4;                    // floats in a partial record
    static_assert(LPR <= kWave && D <= NT, "row must fit a wave, output a block");

    extern __shared__ float smem[];
    float* xs = smem;                // [chunk] logits, then attention weights
    float* ys = smem + a.chunk;      // [chunk] perturbed logits / tau, then their exponentials
    float* red_o = ys + a.chunk;     // [NW][D] per-wave output partials
    __shared__ float red_s[NW];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int sub = lane / LPR, cl = lane % LPR;
    const int S = a.S;
    const int64_t u = blockIdx.x / S;
    const int s = blockIdx.x % S;
    const int h = (int)(u % a.H), b = (int)((u / a.H) % a.B), l = a.layer0 + (int)(u / ((int64_t)a.H * a.B));

    const int len0 = a.len[u];
    const int m = len0 + 1;
    if (len0 < 0 || len0 >= a.cap || m > S * a.chunk) {
        // no room for the new token (or a launch shaped for fewer tokens):
        // leave the unit alone and report it
        if (s == 0) {
            if (tid < D) a.out[u * D + tid] = 0.0f;
            if (tid == 0) atomicAdd(a.ws_err, 1);
        }
        return;
    }
    const int j0 = s * a.chunk;
    const int j1 = min(m, j0 + a.chunk);
    const int cnt = max(j1 - j0, 0);

    const T* Ku = (const T*)a.K + (size_t)u * a.cap * D;
    const T* Vu = (const T*)a.V + (size_t)u * a.cap * D;
    const T* qu = (const T*)a.q + (size_t)u * D;
    const T* knew = (const T*)a.k_new + (size_t)u * D;
    const T* vnew = (const T*)a.v_new + (size_t)u * D;
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;

    // ---- append: the split that owns slot len0 stores the new row.  The row is
    // not read back from the cache in this launch (the streams below take it
    // from k_new / v_new), so no ordering is needed.
    if (len0 >= j0 && len0 < j1) {
        if (wv == 0 && lane < LPR)
            ((uint4*)((T*)a.K + ((size_t)u * a.cap + len0) * D))[lane] = ((const uint4*)knew)[lane];
        if (wv == 1 && lane < LPR)
            ((uint4*)((T*)a.V + ((size_t)u * a.cap + len0) * D))[lane] = ((const uint4*)vnew)[lane];
        if (tid == 2 * kWave) pu[len0] = a.q_pos;
    }

    // ---- query slice of this lane
    float qv[EPV];
    {
        const uint4 r = ((const uint4*)qu)[cl];
        unpack16<T>(r, qv);
    }

    // Loads one tile (UNR block-wide loads) of this lane's 16-byte pieces; the
    // slot of the new token is served from the call's own k_new / v_new row.
    auto load_tile = [&](const T* rows, const T* fresh, int base, uint4(&raw)[UNR]) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int j = base + i * RPB + sub;
            if (j < j1) {
                const T* row = (j == len0) ? fresh : rows + (size_t)j * D;
                raw[i] = ((const uint4*)row)[cl];
            } else {
                raw[i] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    };
    constexpr int TILE = RPB * UNR;
    const int base0 = j0 + wv * RPW;

    // ---- phase 1: stream K (next tile in flight while this one is reduced), logits into LDS
    uint4 cur[UNR], nxt[UNR];
    if (base0 < j1) load_tile(Ku, knew, base0, cur);
    for (int base = base0; base < j1; base += TILE) {
        if (base + TILE < j1) load_tile(Ku, knew, base + TILE, nxt);
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            float kvals[EPV];
            unpack16<T>(cur[i], kvals);
            float p = 0.0f;
#pragma unroll
            for (int e = 0; e < EPV; ++e) p = fmaf(kvals[e], qv[e], p);
#pragma unroll
            for (int o = LPR / 2; o > 0; o >>= 1) p += __shfl_xor(p, o, kWave);
            const int j = base + i * RPB + sub;
            if (cl == 0 && j < j1) xs[j - j0] = p * a.scale;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
    }
    // first V tile: in flight while the softmax statistics are formed
    if (base0 < j1) load_tile(Vu, vnew, base0, cur);
    __syncthreads();

    // ---- phase 1.5: position bias, logit adjustment, the two softmaxes' statistics
    const float slope = a.slopes ? a.slopes[h] : 0.0f;
    uint32_t rkey = 0;
    if (a.noise == kNoiseGumbel || a.noise == kNoiseGaussian)
        rkey = row_key(unit_key(a.seeds[b], (uint32_t)l, (uint32_t)h), (uint32_t)a.q_pos);
    float mx = -INFINITY, my = -INFINITY;
    for (int t = tid; t < cnt; t += NT) {
        const int j = j0 + t;
        const int pj = (j == len0) ? a.q_pos : pu[j];
        const float x = xs[t] - slope * (float)(a.q_pos - pj);
        const float y = (x + zeta_of(a.noise, rkey, (uint32_t)pj)) * a.inv_tau;
        xs[t] = x;
        ys[t] = y;
        mx = fmaxf(mx, x);
        my = fmaxf(my, y);
    }
    mx = block_max<NT>(mx, red_s);
    my = block_max<NT>(my, red_s);
    float sp = 0.0f, se = 0.0f;
    for (int t = tid; t < cnt; t += NT) {
        const float p = expf(xs[t] - mx);
        const float e = expf(ys[t] - my);
        xs[t] = p;
        ys[t] = e;
        sp += p;
        se += e;
    }
    sp = block_sum<NT>(sp, red_s);
    se = block_sum<NT>(se, red_s);
    if (S == 1) {
        // the whole unit is here: accumulate the normalised score increment
        const float inv = 1.0f / se;
        for (int t = tid; t < cnt; t += NT) {
            const float prev = (t == len0) ? 0.0f : fu[t];
            fu[t] = prev + ys[t] * inv;
        }
    } else {
        float* we = a.ws_e + (size_t)u * a.cap;
        for (int t = tid; t < cnt; t += NT) we[j0 + t] = ys[t];
    }
    __syncthreads();  // attention weights of all threads are in xs

    // ---- phase 2: stream V, weighted sum
    float acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = 0.0f;
    for (int base = base0; base < j1; base += TILE) {
        if (base + TILE < j1) load_tile(Vu, vnew, base + TILE, nxt);
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int j = base + i * RPB + sub;
            const float p = (j < j1) ? xs[j - j0] : 0.0f;
            float vvals[EPV];
            unpack16<T>(cur[i], vvals);
#pragma unroll
            for (int e = 0; e < EPV; ++e) acc[e] = fmaf(p, vvals[e], acc[e]);
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) cur[i] = nxt[i];
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
        if (tid < D) a.out[u * D + tid] = o_c / sp;
        if (tid == 0) a.len[u] = m;
        return;
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
    if (len0 < 0 || len0 >= a.cap || len0 + 1 > a.S * a.chunk) return;  // skipped by the split kernel too
    merge_unit<D, NT>(a, u, len0, red_s, w_p, w_e);
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
    int64_t s_hi = (m + kDecodeMinChunk - 1) / kDecodeMinChunk;
    int64_t s_lo = (m + kDecodeMaxChunk - 1) / kDecodeMaxChunk;
    if (s_hi > kDecodeMaxSplits) s_hi = kDecodeMaxSplits;
    if (s_lo < 1) s_lo = 1;
    if (s_hi < s_lo) s_hi = s_lo;
    int64_t best_S = s_lo;
    double best_cost = 0.0;
    bool best_filled = false;
    for (int64_t S = s_lo; S <= s_hi && S <= s_lo + 63; ++S) {
        int64_t chunk = (m + S - 1) / S;
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
    int64_t chunk = (m + best_S - 1) / best_S;
    chunk = (chunk + rpb - 1) / rpb * rpb;
    p.S = (int32_t)best_S;
    p.chunk = (int32_t)chunk;
    p.lds_bytes = (size_t)(2 * chunk + (kDecodeThreads / kWave) * d) * sizeof(float);
    return p;
}

template <typename T, int D>
static hipError_t launch_decode_t(const DecodeArgs& a, int64_t U, size_t lds, hipStream_t st) {
    const dim3 grid((unsigned)(U * a.S)), block(kDecodeThreads);
    hipLaunchKernelGGL((decode_kernel<T, D, kDecodeThreads>), grid, block, lds, st, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.S > 1) {
        hipLaunchKernelGGL((decode_merge_kernel<D, kDecodeThreads>), dim3((unsigned)U), block, 0, st, a);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_decode(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                         hipStream_t stream) {
    if (a.chunk > kDecodeMaxChunk) return hipErrorInvalidValue;
    if (dtype == KF_BF16) {
        if (d == 64) return launch_decode_t<bf16_t, 64>(a, U, lds_bytes, stream);
        if (d == 128) return launch_decode_t<bf16_t, 128>(a, U, lds_bytes, stream);
        if (d == 256) return launch_decode_t<bf16_t, 256>(a, U, lds_bytes, stream);
    } else {
        if (d == 64) return launch_decode_t<float, 64>(a, U, lds_bytes, stream);
        if (d == 128) return launch_decode_t<float, 128>(a, U, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace kf
