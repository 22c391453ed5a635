// Merge of a unit's split-wise partial results of the decode kernel; shared by
// the stand-alone merge kernel and the fused step-tail kernel.
#pragma once
#include "kf_device.h"
#include "kf_internal.h"

namespace kf {

constexpr int kDecodeMaxSplits = 256;  // a wave merges one head's records: this many / 64 per lane, in registers

// Merges the S partial records of unit u (one per split and query head):
// rescales every split's un-normalised output and score increments to the
// head-wide maxima, normalises, accumulates the scores (summed over the unit's
// G query heads) and publishes the new length.  Called by a whole workgroup.
// w_p, w_e: LDS, G*S floats each.
// The workgroup handles tokens [j_begin, j_end) of the score update; the `lead`
// workgroup of a unit also writes the attention outputs and the new length.
template <int D, int NT, int G>
__device__ __forceinline__ void merge_unit(const DecodeArgs& a, int64_t u, int len0, float* w_p, float* w_e, int j_begin,
                                           int j_end, bool lead) {
    constexpr int PW = D + 4;
    const int tid = threadIdx.x, S = a.S, m = len0 + 1;
    const float* parts = a.ws_part + (size_t)u * S * G * PW;
    float* fu = a.score + (size_t)u * a.cap;
    // Per-head statistics: one wave per query head (heads beyond the wave count take turns), each lane
    // holding the records of splits lane, lane+64, ...; wave-wide reductions only, so the G heads cost
    // no workgroup barrier and their record loads are all in flight at once.
    constexpr int NW = NT / kWave, SP = kDecodeMaxSplits / kWave;
    __shared__ float inv_p[G];
    const int wave = tid / kWave, lane = tid % kWave;
    for (int g = wave; g < G; g += NW) {
        float pmx[SP], psp[SP], pmy[SP], pse[SP];
#pragma unroll
        for (int i = 0; i < SP; ++i) {
            const int ss = lane + i * kWave;
            pmx[i] = -INFINITY, psp[i] = 0.0f, pmy[i] = -INFINITY, pse[i] = 0.0f;
            if (ss < S) {
                const float4 r = *reinterpret_cast<const float4*>(parts + ((size_t)ss * G + g) * PW + D);
                pmx[i] = r.x, psp[i] = r.y, pmy[i] = r.z, pse[i] = r.w;
            }
        }
        float mx = pmx[0], my = pmy[0];
#pragma unroll
        for (int i = 1; i < SP; ++i) mx = fmaxf(mx, pmx[i]), my = fmaxf(my, pmy[i]);
        const float Mx = wave_max(mx), My = wave_max(my);
        // statistics are kept in the base-2 domain (logits times log2 e)
        float wp[SP], we_[SP], sp = 0.0f, se = 0.0f;
#pragma unroll
        for (int i = 0; i < SP; ++i) {
            wp[i] = (psp[i] > 0.0f) ? hw_exp2(pmx[i] - Mx) : 0.0f;  // empty splits weigh nothing
            we_[i] = (pse[i] > 0.0f) ? hw_exp2(pmy[i] - My) : 0.0f;
            sp = fmaf(wp[i], psp[i], sp);
            se = fmaf(we_[i], pse[i], se);
        }
        const float sumP = wave_sum(sp), invE = 1.0f / wave_sum(se);
#pragma unroll
        for (int i = 0; i < SP; ++i) {
            const int ss = lane + i * kWave;
            if (ss < S) {
                w_p[g * S + ss] = wp[i];
                w_e[g * S + ss] = we_[i] * invE;
            }
        }
        if (lane == 0) inv_p[g] = 1.0f / sumP;
    }
    __syncthreads();
    if (lead) {
        for (int idx = tid; idx < G * D; idx += NT) {
            const int g = idx / D, t = idx % D;
            float o = 0.0f;
            for (int ss = 0; ss < S; ++ss) o = fmaf(w_p[g * S + ss], parts[((size_t)ss * G + g) * PW + t], o);
            a.out[(u * G + g) * D + t] = o * inv_p[g];
        }
    }
    float* we = a.ws_e + (size_t)u * G * a.cap;
    for (int j = j_begin + tid; j < min(j_end, m); j += NT) {
        const int split = (j == len0) ? S - 1 : j / a.chunk;  // the new token belongs to the last split
        float df = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) df = fmaf(we[(size_t)g * a.cap + j], w_e[g * S + split], df);
        if (a.shared) we[j] = df;  // summed over the layers by the launch that follows
        else if (j == len0) fu[j] = df;
        else unsafeAtomicAdd(&fu[j], df);  // fire-and-forget add at the L2 (one per address: the plain fp32 sum)
    }
    if (lead && tid == 0) a.len[u] = m;
}

}  // namespace kf
