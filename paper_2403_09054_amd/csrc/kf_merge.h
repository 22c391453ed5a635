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
// Smallest eviction candidate of a slice of tokens, as the selection's candidate scan forms it: the pack
// orders by score, then (equal scores) the higher slot -- ordered layout -- or the higher position -- slot
// layout -- leaves first.
struct SliceMin {
    unsigned long long best = ~0ull;
    int slot = -1;
    __device__ __forceinline__ void take(float f, int j, int tie) {
        const unsigned long long pack = ((unsigned long long)float_key(f) << 32) | (uint32_t)(~(uint32_t)tie);
        if (pack < best) {
            best = pack;
            slot = j;
        }
    }
};

// The workgroup's smallest candidate goes to entry `slice` of the unit's table.  Called by a whole workgroup.
template <int NT>
__device__ __forceinline__ void publish_slice_min(const DecodeArgs& a, int64_t u, int slice, SliceMin mine) {
    __shared__ unsigned long long wmin_s[NT / kWave];
    __shared__ int wslot_s[NT / kWave];
    const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
    unsigned long long best = mine.best;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long t = __shfl_xor(best, o, kWave);
        best = t < best ? t : best;
    }
    // slots and positions are unique: one lane of the wave owns the wave's minimum
    const unsigned long long owner = __ballot(mine.best == best && best != ~0ull);
    const int wslot = __shfl(mine.slot, owner ? __ffsll((long long)owner) - 1 : 0, kWave);
    if (lane == 0) {
        wmin_s[wv] = best;
        wslot_s[wv] = owner ? wslot : -1;
    }
    __syncthreads();
    if (tid == 0) {
        unsigned long long g = wmin_s[0];
        int gs = wslot_s[0];
        for (int i = 1; i < NT / kWave; ++i)
            if (wmin_s[i] < g) {
                g = wmin_s[i];
                gs = wslot_s[i];
            }
        a.pre_min[(size_t)u * a.pre_slices + slice] = g;
        a.pre_slot[(size_t)u * a.pre_slices + slice] = gs;
    }
}

// The same table entry for a unit the decode launch skipped (it is full; the selection may still evict
// from it): the candidates among slots [j_begin, j_end) of its n entries, from the scores as they are.
template <int NT>
__device__ __forceinline__ void scan_slice_min(const DecodeArgs& a, int64_t u, int n, int j_begin, int j_end, int slice) {
    const bool by_pos = a.pre_layout == KF_LAYOUT_SLOT;
    const float* fu = a.score + (size_t)u * a.cap;
    const int32_t* pu = a.pos + (size_t)u * a.cap;
    const int newest = by_pos ? pu[n - 1] : 0;
    SliceMin smin;
    for (int j = j_begin + (int)threadIdx.x; j < min(j_end, n); j += NT) {
        const int pj = by_pos ? pu[j] : 0;
        if (by_pos ? (pj <= newest - a.pre_w) : (j < n - a.pre_w)) smin.take(fu[j], j, by_pos ? pj : j);
    }
    publish_slice_min<NT>(a, u, slice, smin);
}

template <int D, int NT, int G>
__device__ __forceinline__ void merge_unit(const DecodeArgs& a, int64_t u, int len0, float* w_p, float* w_e, int j_begin,
                                           int j_end, bool lead, int slice = 0) {
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
    float* we = a.ws_e + (size_t)u * G * a.cap;
    // with pre_slices the finished scores are also searched for the slice's smallest eviction candidate
    // (only a unit exactly one token over the budget is looked at by the selection launch)
    const bool pre = a.pre_slices > 0 && m == a.pre_k + 1;
    const bool by_pos = a.pre_layout == KF_LAYOUT_SLOT;
    const int32_t* pu = a.pos + (size_t)u * a.cap;
    const int newest = (pre && by_pos) ? pu[len0] : 0;
    // Loads first, arithmetic after: a loop that waits for each of its loads in turn costs a trip to memory per
    // split and per token stride (32 splits: the output alone took 11 us).  A thread has kMergeTok tokens of the
    // score update and kMergeRec split records of an output element in flight at a time, and the first tokens
    // are asked for before the outputs are formed.  The order of every sum is the sequential one.
    constexpr int kMergeTok = 4, kMergeRec = 8;
    const int jmax = min(j_end, m);
    float tw[kMergeTok][G], tf[kMergeTok];
    int tp[kMergeTok];
    auto load_tokens = [&](int jb) {
#pragma unroll
        for (int i = 0; i < kMergeTok; ++i) {
            const int j = jb + i * NT;
            const bool ok = j < jmax;
#pragma unroll
            for (int g = 0; g < G; ++g) tw[i][g] = ok ? we[(size_t)g * a.cap + j] : 0.0f;
            tf[i] = (ok && pre && j != len0) ? fu[j] : 0.0f;
            tp[i] = (ok && pre && by_pos) ? pu[j] : 0;
        }
    };
    int jb = j_begin + tid;
    if (jb < jmax) load_tokens(jb);
    if (lead) {
        for (int idx = tid; idx < G * D; idx += NT) {
            const int g = idx / D, t = idx % D;
            const float* pr = parts + (size_t)g * PW + t;
            float o = 0.0f;
            for (int s0 = 0; s0 < S; s0 += kMergeRec) {
                float v[kMergeRec];
#pragma unroll
                for (int i = 0; i < kMergeRec; ++i) v[i] = (s0 + i < S) ? pr[(size_t)(s0 + i) * G * PW] : 0.0f;
#pragma unroll
                for (int i = 0; i < kMergeRec; ++i) o = fmaf((s0 + i < S) ? w_p[g * S + s0 + i] : 0.0f, v[i], o);
            }
            a.out[(u * G + g) * D + t] = o * inv_p[g];
        }
    }
    SliceMin smin;
    while (jb < jmax) {
#pragma unroll
        for (int i = 0; i < kMergeTok; ++i) {
            const int j = jb + i * NT;
            if (j >= jmax) break;
            const int split = (j == len0) ? S - 1 : j / a.chunk;  // the new token belongs to the last split
            float df = 0.0f;
#pragma unroll
            for (int g = 0; g < G; ++g) df = fmaf(tw[i][g], w_e[g * S + split], df);
            if (a.shared) we[j] = df;  // summed over the layers by the launch that follows
            else if (pre) {
                const float f_new = (j == len0) ? df : tf[i] + df;  // one add per address, as below
                fu[j] = f_new;
                if (by_pos ? (tp[i] <= newest - a.pre_w) : (j < m - a.pre_w)) smin.take(f_new, j, by_pos ? tp[i] : j);
            } else if (j == len0) fu[j] = df;
            else unsafeAtomicAdd(&fu[j], df);  // fire-and-forget add at the L2 (one per address: the plain fp32 sum)
        }
        jb += kMergeTok * NT;
        if (jb < jmax) load_tokens(jb);
    }
    if (pre) publish_slice_min<NT>(a, u, slice, smin);
    if (lead && tid == 0) a.len[u] = m;
}

}  // namespace kf
