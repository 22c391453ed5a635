// Merge of a unit's split-wise partial results of the decode kernel; shared by
// the stand-alone merge kernel and the fused step-tail kernel.
#pragma once
#include "kf_device.h"
#include "kf_internal.h"

namespace kf {

constexpr int kDecodeMaxSplits = 256;  // one thread per split in the merge: <= threads of the merging workgroup

// Merges the S partial records of unit u (one per split and query head):
// rescales every split's un-normalised output and score increments to the
// head-wide maxima, normalises, accumulates the scores (summed over the unit's
// G query heads) and publishes the new length.  Called by a whole workgroup.
// w_p, w_e: LDS, G*S floats each.
// The workgroup handles tokens [j_begin, j_end) of the score update; the `lead`
// workgroup of a unit also writes the attention outputs and the new length.
template <int D, int NT, int G>
__device__ __forceinline__ void merge_unit(const DecodeArgs& a, int64_t u, int len0, float* red_s, float* w_p,
                                           float* w_e, int j_begin, int j_end, bool lead) {
    constexpr int PW = D + 4;
    const int tid = threadIdx.x, S = a.S, m = len0 + 1;
    const float* parts = a.ws_part + (size_t)u * S * G * PW;
    float* fu = a.score + (size_t)u * a.cap;
    float inv[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float pmx = -INFINITY, psp = 0.0f, pmy = -INFINITY, pse = 0.0f;
        if (tid < S) {
            const float* r = parts + ((size_t)tid * G + g) * PW + D;
            pmx = r[0];
            psp = r[1];
            pmy = r[2];
            pse = r[3];
        }
        const float Mx = block_max<NT>(pmx, red_s);
        const float My = block_max<NT>(pmy, red_s);
        // statistics are kept in the base-2 domain (logits times log2 e)
        const float wp = (psp > 0.0f) ? hw_exp2(pmx - Mx) : 0.0f;  // empty splits weigh nothing
        const float we_ = (pse > 0.0f) ? hw_exp2(pmy - My) : 0.0f;
        const float sumP = block_sum<NT>(wp * psp, red_s);
        const float sumE = block_sum<NT>(we_ * pse, red_s);
        if (tid < S) {
            w_p[g * S + tid] = wp;
            w_e[g * S + tid] = we_;
        }
        __syncthreads();
        if (lead && tid < D) {
            float o = 0.0f;
            for (int ss = 0; ss < S; ++ss) o = fmaf(w_p[g * S + ss], parts[((size_t)ss * G + g) * PW + tid], o);
            a.out[(u * G + g) * D + tid] = o / sumP;
        }
        inv[g] = 1.0f / sumE;
    }
    float* we = a.ws_e + (size_t)u * G * a.cap;
    for (int j = j_begin + tid; j < min(j_end, m); j += NT) {
        const int split = (j == len0) ? S - 1 : j / a.chunk;  // the new token belongs to the last split
        float df = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) df = fmaf(we[(size_t)g * a.cap + j], w_e[g * S + split] * inv[g], df);
        if (a.shared) we[j] = df;  // summed over the layers by the launch that follows
        else if (j == len0) fu[j] = df;
        else unsafeAtomicAdd(&fu[j], df);  // fire-and-forget add at the L2 (one per address: the plain fp32 sum)
    }
    if (lead && tid == 0) a.len[u] = m;
}

}  // namespace kf
