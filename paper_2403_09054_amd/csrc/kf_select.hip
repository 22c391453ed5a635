// Key-token selection and in-place, order-preserving KV compaction for gfx950.
//
// Per unit (Algorithm 1: S_w, S_key, S_k):  keep the last w slots and the k-w
// slots of [0, len-w) with the largest accumulated score, equal scores resolved
// toward the lower slot; move the survivors' K, V, score and pos rows to slots
// [0,k) in their original order; len = k.
//
// One workgroup per unit.
//   select   radix select on order-preserving uint32 keys of the scores: four
//            8-bit passes with an LDS histogram find the (k-w)-th largest key T
//            and how many candidates equal to T still fit.
//   rank     one ordered sweep over the candidates: a candidate survives if its
//            key is above T, or equals T and fewer than `need` equal keys
//            precede it (lower slot wins).  Ballot/popcount prefix counts give
//            each survivor its destination; the source slots are written to a
//            dense index list.
//   compact  rows are gathered front to back in tiles: a tile's sources are
//            read into registers, the workgroup synchronises, then the tile's
//            destinations are written.  Every source lies at or after its
//            destination, so a tile never overwrites a row a later tile still
//            has to read.  Rows that stay where they are are not touched.
#include "kf_device.h"
#include "kf_internal.h"

namespace kf {

constexpr int kSelectThreads = 512;
constexpr int kSelectGroups = 4;  // row groups a thread holds in registers per tile

template <int NT>
__global__ void __launch_bounds__(NT) select_kernel(const SelectArgs a) {
    constexpr int NW = NT / kWave;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_bin, s_rem;
    __shared__ uint32_t wtot[NW][2];
    __shared__ int s_first;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t u = blockIdx.x;
    const int n = a.len[u];
    const int k = a.k, w = a.w;
    int32_t* idx = a.idx + (size_t)u * k;

    if (n <= k) {  // under budget: nothing leaves
        for (int i = tid; i < k; i += NT) idx[i] = (i < n) ? i : -1;
        return;
    }
    const int ncand = n - w, nkey = k - w;
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;

    // ---- select: threshold key T = the nkey-th largest candidate key
    uint32_t T = 0xFFFFFFFFu, need = 0;
    if (nkey > 0) {
        uint32_t prefix = 0, mask = 0, remaining = (uint32_t)nkey;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int j = tid; j < ncand; j += NT) {
                const uint32_t key = float_key(fu[j]);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid < kWave) {
                // lane owns bins [4*lane, 4*lane+4); count of keys in higher bins first
                uint32_t c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) c[i] = hist[tid * 4 + i];
                const uint32_t tot = c[0] + c[1] + c[2] + c[3];
                uint32_t incl = tot;  // becomes the sum over lanes >= this one
#pragma unroll
                for (int o = 1; o < kWave; o <<= 1) {
                    const uint32_t t = __shfl_down(incl, o, kWave);
                    if (tid + o < kWave) incl += t;
                }
                uint32_t above = incl - tot;
#pragma unroll
                for (int i = 3; i >= 0; --i) {
                    if (above < remaining && remaining <= above + c[i]) {
                        s_bin = (uint32_t)(tid * 4 + i);
                        s_rem = remaining - above;
                    }
                    above += c[i];
                }
            }
            __syncthreads();
            prefix |= s_bin << shift;
            mask |= 0xFFu << shift;
            remaining = s_rem;
        }
        T = prefix;
        need = remaining;  // how many candidates equal to T survive (lowest slots first)
    }

    // ---- rank: ordered sweep, destination of every survivor
    if (tid == 0) s_first = k;
    __syncthreads();
    uint32_t run_gt = 0, run_eq = 0;
    for (int base = 0; base < ncand; base += NT) {
        const int j = base + tid;
        bool gt = false, eq = false;
        if (j < ncand && nkey > 0) {
            const uint32_t key = float_key(fu[j]);
            gt = key > T;
            eq = key == T;
        }
        const unsigned long long bg = __ballot(gt), be = __ballot(eq);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (lane == 0) {
            wtot[wv][0] = (uint32_t)__popcll(bg);
            wtot[wv][1] = (uint32_t)__popcll(be);
        }
        __syncthreads();
        uint32_t gt_before = run_gt + (uint32_t)__popcll(bg & below);
        uint32_t eq_before = run_eq + (uint32_t)__popcll(be & below);
        uint32_t tg = 0, te = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if (i < wv) {
                gt_before += wtot[i][0];
                eq_before += wtot[i][1];
            }
            tg += wtot[i][0];
            te += wtot[i][1];
        }
        const bool keep = gt || (eq && eq_before < need);
        if (keep) {
            const uint32_t dst = gt_before + min(eq_before, need);
            if (dst < (uint32_t)nkey) idx[dst] = j;  // always true; keeps a logic error in bounds
        } else if (j < ncand) {
            atomicMin(&s_first, j);  // first slot that changes occupant
        }
        run_gt += tg;
        run_eq += te;
        __syncthreads();
    }
    for (int i = tid; i < w; i += NT) idx[nkey + i] = ncand + i;  // the recent window
    __syncthreads();  // idx and s_first are complete for the whole workgroup

    // ---- compact: front-to-back gather through registers
    const int PPR = a.row_bytes >> 4;  // 16-byte pieces per row
    const int rpp = NT / PPR;          // rows per pass of the workgroup
    const int R = rpp * kSelectGroups; // rows per tile
    const int piece = tid % PPR, rsub = tid / PPR;
    uint4* Kb = (uint4*)((char*)a.K + (size_t)u * a.cap * a.row_bytes);
    uint4* Vb = (uint4*)((char*)a.V + (size_t)u * a.cap * a.row_bytes);
    for (int t0 = s_first; t0 < k; t0 += R) {
        uint4 rk[kSelectGroups], rv[kSelectGroups];
        int src[kSelectGroups];
#pragma unroll
        for (int g = 0; g < kSelectGroups; ++g) {
            const int i = t0 + g * rpp + rsub;
            src[g] = (i < k) ? idx[i] : -1;
            if (src[g] >= n) src[g] = -1;  // cannot happen; never read past the unit
            if (src[g] >= 0 && src[g] != i) {
                rk[g] = Kb[(size_t)src[g] * PPR + piece];
                rv[g] = Vb[(size_t)src[g] * PPR + piece];
            }
        }
        float fv = 0.0f;
        int pv = 0, ssrc = -1;
        const int si = t0 + tid;
        if (tid < R && si < k) {
            ssrc = idx[si];
            if (ssrc >= n) ssrc = -1;
            if (ssrc >= 0) {
                fv = fu[ssrc];
                pv = pu[ssrc];
            }
        }
        // the loads above must have returned before any thread overwrites a row
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#pragma unroll
        for (int g = 0; g < kSelectGroups; ++g) {
            const int i = t0 + g * rpp + rsub;
            if (src[g] >= 0 && src[g] != i) {
                Kb[(size_t)i * PPR + piece] = rk[g];
                Vb[(size_t)i * PPR + piece] = rv[g];
            }
        }
        if (ssrc >= 0 && ssrc != si) {
            fu[si] = fv;
            pu[si] = pv;
        }
    }
    if (tid == 0) a.len[u] = k;
}

hipError_t launch_select(const SelectArgs& a, int64_t U, hipStream_t stream) {
    const dim3 grid((unsigned)U), block(kSelectThreads);
    hipLaunchKernelGGL((select_kernel<kSelectThreads>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace kf
