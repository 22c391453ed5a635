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
//            (A unit that is exactly one token over budget -- every decode
//            step -- skips both: the token to evict is the candidate with the
//            smallest score, the highest slot among equals, found by one
//            min-reduction; see evict_one.)
//   compact  rows are gathered front to back in tiles: a tile's sources are
//            read into registers, the workgroup synchronises, then the tile's
//            destinations are written.  Every source lies at or after its
//            destination, so a tile never overwrites a row a later tile still
//            has to read.  Rows that stay where they are are not touched.
#include "kf_device.h"
#include "kf_internal.h"
#include "kf_merge.h"

namespace kf {

constexpr int kSelectThreads = 1024;     // ordered layout: many rows move, many waves stream them
constexpr int kSelectThreadsSlot = 512;  // slot layout: one row moves, smaller workgroups finish sooner
constexpr int kSelectGroups = 4;  // row groups a thread holds in registers per tile
constexpr int kShiftDepth = 8;    // independent 16-byte loads a lane keeps in flight while shifting

// One token over budget (len = k+1, the shape of every decode step): evict the
// candidate with the smallest score, the highest slot among equal minima (so
// that lower slots are kept), then close the gap: rows e+1..k move down by one.
//
// The rows that move are the candidates behind the evicted slot (usually a
// handful) and the whole recent window (always, whatever slot is evicted).  The
// window part therefore starts before the evicted slot is known: waves 2.. own
// fixed contiguous ranges of it and have their first rows in flight while the
// min-reduction runs.  A lane owns one 16-byte piece of a row, the two halves of
// a wave take K and V.  A wave walks its range upwards, several rows in flight:
// row i+1 is loaded before row i is stored, loads return in order, and the wave
// is the only writer of its range, so it never overwrites a row it still has to
// read.  The one row it reads from its neighbour's range (the first row above
// its own) is loaded before the barrier; the neighbour stores only after it.
// The candidate part is read completely before that same barrier -- into
// registers when it is short, by a streaming pass of its own when it is long --
// because its last source row is the window part's first destination.
// Waves 0 and 1 shift score and pos the same way, 64 elements per instruction.
// Row loads and stores are non-temporal: the shifted rows are not needed again
// before the next step's full sweep, and leaving them out of the caches shortens
// that sweep (the following decode launch ran 93 -> 83 us on the GPT-J-shaped
// workload, this kernel 47 -> 51 us).
struct RowLane {  // what a lane needs to address its piece of a row
    uint4* base;
    int PPR, RPI, rsub, piece;
    __device__ __forceinline__ uint4* at(int row) const { return base + (size_t)row * PPR + piece; }
};

// Streams dst rows [r0, r1) <- src rows [r0+1, r1+1) of one wave's range.  `first`
// holds the already loaded sources of the range's first G instructions, `last`
// those of its last instruction (the only rows read from beyond the range).
template <int G>
__device__ __forceinline__ void shift_range(const RowLane& L, int r0, int NI, const uint4 (&first)[G], bool has_last,
                                            int last_i, const uint4& last) {
#pragma unroll
    for (int g = 0; g < G; ++g)
        if (g < NI - 1) stream_store(L.at(r0 + g * L.RPI + L.rsub), first[g]);
    for (int ii = G; ii < NI - 1; ii += G) {
        uint4 regs[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            regs[g] = make_uint4(0u, 0u, 0u, 0u);
            if (ii + g < NI - 1) regs[g] = stream_load(L.at(r0 + (ii + g) * L.RPI + L.rsub + 1));
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
            if (ii + g < NI - 1) stream_store(L.at(r0 + (ii + g) * L.RPI + L.rsub), regs[g]);
    }
    if (has_last) stream_store(L.at(last_i), last);
}

// Loads what shift_range needs up front: the first G instructions' sources and the last one's.
template <int G>
__device__ __forceinline__ void preload_range(const RowLane& L, int r0, int r1, int& NI, uint4 (&first)[G],
                                              bool& has_last, int& last_i, uint4& last) {
    NI = r0 < r1 ? (r1 - r0 + L.RPI - 1) / L.RPI : 0;  // wave instructions of this range
    last_i = r0 + (NI - 1) * L.RPI + L.rsub;
    has_last = NI > 0 && last_i < r1;
    last = make_uint4(0u, 0u, 0u, 0u);
    if (has_last) last = stream_load(L.at(last_i + 1));
#pragma unroll
    for (int g = 0; g < G; ++g) {
        first[g] = make_uint4(0u, 0u, 0u, 0u);
        if (g < NI - 1) first[g] = stream_load(L.at(r0 + g * L.RPI + L.rsub + 1));
    }
}

template <int NT>
__device__ __forceinline__ void evict_one(const SelectArgs& a, int64_t u, int n, bool write_idx) {
    constexpr int NW = NT / kWave;
    constexpr int NRW = NW - 2;  // waves that move rows
    constexpr int G = kShiftDepth;
    __shared__ unsigned long long wmin[NW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int k = a.k, w = a.w;
    const int ncand = n - w;
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;

    RowLane L;
    L.PPR = a.row_bytes >> 4;  // 16-byte pieces per row: 8, 16 or 32
    L.RPI = 32 / L.PPR;        // rows per wave instruction (each half of the wave one tensor)
    L.rsub = (lane & 31) / L.PPR;
    L.piece = lane % L.PPR;
    L.base = (uint4*)((char*)((lane >> 5) ? a.V : a.K) + (size_t)u * a.cap * a.row_bytes);
    auto range_of = [&](int lo, int hi, int& r0, int& r1) {  // this wave's share of dst rows [lo, hi)
        int per = (hi - lo + NRW - 1) / NRW;
        per = (per + L.RPI - 1) / L.RPI * L.RPI;
        r0 = min(hi, lo + (wv - 2) * per);
        r1 = min(hi, r0 + per);
    };

    // candidate scores first, so that they return ahead of the row loads issued next
    // smallest (key, -slot): the low word holds ~slot so that the highest slot wins a tie
    unsigned long long best = ~0ull;
    for (int j = tid; j < ncand; j += NT) {
        const unsigned long long pack = ((unsigned long long)float_key(fu[j]) << 32) | (uint32_t)(~(uint32_t)j);
        best = pack < best ? pack : best;
    }

    // ---- window part, dst rows [ncand-1, k): in flight before the evicted slot is known
    const int w_lo = max(ncand - 1, 0);
    int wr0 = 0, wr1 = 0, wNI = 0, wlast_i = 0;
    bool whas_last = false;
    uint4 wfirst[G], wlast = make_uint4(0u, 0u, 0u, 0u);
    if (wv >= 2) {
        range_of(w_lo, k, wr0, wr1);
        preload_range<G>(L, wr0, wr1, wNI, wfirst, whas_last, wlast_i, wlast);
    }

#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long t = __shfl_xor(best, o, kWave);
        best = t < best ? t : best;
    }
    if (lane == 0) wmin[wv] = best;
    __syncthreads();
    best = wmin[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) best = wmin[i] < best ? wmin[i] : best;
    const int e = (int)(~(uint32_t)(best & 0xFFFFFFFFull));  // evicted slot, in [0, ncand)

    if (write_idx) {
        int32_t* idx = a.idx + (size_t)u * k;
        for (int i = tid; i < k; i += NT) idx[i] = i + (i >= e ? 1 : 0);
    }

    // ---- candidate part, dst rows [e, ncand-1)
    const int c = w_lo - e;                 // rows of it (>= 0)
    const bool c_in_regs = c <= NRW * L.RPI;  // one instruction per wave covers it
    uint4 creg = make_uint4(0u, 0u, 0u, 0u);
    int crow = -1;
    if (c > 0 && !c_in_regs) {
        // long: a streaming pass of its own, finished (reads and writes) before the window part stores
        if (wv >= 2) {
            int r0, r1, NI, last_i;
            bool has_last;
            uint4 first[G], last;
            range_of(e, w_lo, r0, r1);
            preload_range<G>(L, r0, r1, NI, first, has_last, last_i, last);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            shift_range<G>(L, r0, NI, first, has_last, last_i, last);
        } else {
            __syncthreads();
        }
    } else if (c > 0 && wv >= 2) {
        const int r = e + (wv - 2) * L.RPI + L.rsub;
        if (r < w_lo) {
            crow = r;
            creg = stream_load(L.at(r + 1));
        }
    }
    // every source row that another wave will overwrite has been read
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    if (wv >= 2) {
        if (crow >= 0) stream_store(L.at(crow), creg);
        shift_range<G>(L, wr0, wNI, wfirst, whas_last, wlast_i, wlast);
    } else {
        // ---- score (wave 0) and pos (wave 1): one wave owns the whole range [e, k)
        uint32_t* arr = wv == 0 ? (uint32_t*)fu : (uint32_t*)pu;
        for (int i0 = e; i0 < k; i0 += kWave * G) {
            uint32_t regs[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int i = i0 + g * kWave + lane;
                regs[g] = 0u;
                if (i < k) regs[g] = arr[i + 1];
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int i = i0 + g * kWave + lane;
                if (i < k) arr[i] = regs[g];
            }
        }
    }
    if (tid == 0) a.len[u] = k;
}

// Candidate scan of long units ahead of the selection launch: workgroup (unit, slice) finds the smallest
// candidate of its slice of a decode-shape unit (len = k+1) -- by slot in the ordered layout (candidates are
// the slots below len-w, equal scores: the higher slot leaves), by position in the slot layout (candidates
// are the entries at least w positions behind the newest, equal scores: the higher position leaves).
constexpr int kPreselThreads = 256;
__global__ void __launch_bounds__(kPreselThreads) presel_kernel(const SelectArgs a, int64_t units) {
    __shared__ unsigned long long wmin_p[kPreselThreads / kWave];
    __shared__ int wslot_p[kPreselThreads / kWave];
    const int64_t u = blockIdx.x % units;  // slice-major ids: every XCD gets slices of every kind
    const int sl = (int)(blockIdx.x / units);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = a.len[u];
    if (n != a.k + 1) return;  // the selection launch does not look at the slices of such a unit
    const float* fu = a.score + (size_t)u * a.cap;
    const int32_t* pu = a.pos + (size_t)u * a.cap;
    const int per = ((n + a.presel - 1) / a.presel + kPreselThreads - 1) / kPreselThreads * kPreselThreads;
    const int j0 = sl * per, j1 = min(n, j0 + per);
    const bool by_pos = a.layout == KF_LAYOUT_SLOT;
    const int newest = by_pos ? pu[n - 1] : 0;
    unsigned long long best = ~0ull;
    int best_slot = -1;
    for (int j = j0 + tid; j < j1; j += kPreselThreads) {
        const int pj = by_pos ? pu[j] : 0;
        const bool cand = by_pos ? (pj <= newest - a.w) : (j < n - a.w);
        if (cand) {
            const unsigned long long pack =
                ((unsigned long long)float_key(fu[j]) << 32) | (uint32_t)(~(uint32_t)(by_pos ? pj : j));
            if (pack < best) {
                best = pack;
                best_slot = j;
            }
        }
    }
    const unsigned long long mine = best;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long t = __shfl_xor(best, o, kWave);
        best = t < best ? t : best;
    }
    // slots and positions are unique: one lane of the wave owns the wave's minimum
    const unsigned long long owner = __ballot(mine == best && best != ~0ull);
    const int wslot = __shfl(best_slot, owner ? __ffsll((long long)owner) - 1 : 0, kWave);
    if (lane == 0) {
        wmin_p[wv] = best;
        wslot_p[wv] = owner ? wslot : -1;
    }
    __syncthreads();
    if (tid == 0) {
        unsigned long long g = wmin_p[0];
        int gs = wslot_p[0];
        for (int i = 1; i < kPreselThreads / kWave; ++i)
            if (wmin_p[i] < g) {
                g = wmin_p[i];
                gs = wslot_p[i];
            }
        a.ws_pmin[(size_t)u * a.presel + sl] = g;
        a.ws_pslot[(size_t)u * a.presel + sl] = gs;
    }
}

// The evicted slot from the slices' minima (every lane gets it), -1 if no slice had a candidate.
__device__ __forceinline__ int presel_pick(const SelectArgs& a, int64_t u) {
    unsigned long long g = ~0ull;
    int gs = -1;
    for (int i = 0; i < a.presel; ++i) {
        const unsigned long long v = a.ws_pmin[(size_t)u * a.presel + i];
        if (v < g) {
            g = v;
            gs = a.ws_pslot[(size_t)u * a.presel + i];
        }
    }
    return gs;
}

// Slot-replacement variant of the same eviction (layout KF_LAYOUT_SLOT): the
// cache is an unordered set of (pos, K, V, score) entries.  The recent window
// is the w largest original positions -- positions are consecutive at the
// recent end, so "pos > newest - w" -- the candidate with the smallest score
// leaves (the highest position among equal minima, the same rule as above
// expressed through pos), and the newest entry (slot k) takes its slot: one row
// moves instead of every row behind the gap.
template <int NT>
__device__ __forceinline__ void evict_one_slot(const SelectArgs& a, int64_t u, int n, bool write_idx) {
    constexpr int NW = NT / kWave;
    __shared__ unsigned long long wmin_s[NW];
    __shared__ int s_slot;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int k = a.k, w = a.w;
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;
    const int newest = pu[n - 1];

    if (!a.presel) {  // else the launch ahead scanned the candidates
        unsigned long long best = ~0ull, mine[2] = {~0ull, ~0ull};
        for (int j = tid, c = 0; j < n; j += NT, ++c) {
            const int pj = pu[j];
            unsigned long long pack = ~0ull;
            if (pj <= newest - w)  // a candidate: outside the recent window
                pack = ((unsigned long long)float_key(fu[j]) << 32) | (uint32_t)(~(uint32_t)pj);
            best = pack < best ? pack : best;
            if (c < 2) mine[c] = pack;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long t = __shfl_xor(best, o, kWave);
            best = t < best ? t : best;
        }
        if (lane == 0) wmin_s[wv] = best;
        if (tid == 0) s_slot = -1;
        __syncthreads();
        best = wmin_s[0];
#pragma unroll
        for (int i = 1; i < NW; ++i) best = wmin_s[i] < best ? wmin_s[i] : best;
        // positions are unique, so exactly one entry carries the winning pack
        if (best != ~0ull) {
            for (int j = tid, c = 0; j < n; j += NT, ++c) {
                unsigned long long pack;
                if (c < 2) {
                    pack = mine[c];
                } else {
                    const int pj = pu[j];
                    pack = (pj <= newest - w)
                               ? (((unsigned long long)float_key(fu[j]) << 32) | (uint32_t)(~(uint32_t)pj))
                               : ~0ull;
                }
                if (pack == best) s_slot = j;
            }
        }
        __syncthreads();
    }
    const int e = a.presel ? presel_pick(a, u) : s_slot;
    if (e < 0) {  // no entry lies outside the window (positions not consecutive at the recent end): report
        if (tid == 0) atomicAdd(a.ws_err, 1);
        return;
    }
    if (write_idx) {
        int32_t* idx = a.idx + (size_t)u * k;
        for (int i = tid; i < k; i += NT) idx[i] = (i == e) ? k : i;
    }
    if (e != k) {  // the newest entry moves into the freed slot
        const int PPR = a.row_bytes >> 4;
        if (tid < 2 * PPR) {
            uint4* base = (uint4*)((char*)(tid < PPR ? a.K : a.V) + (size_t)u * a.cap * a.row_bytes);
            const int piece = tid % PPR;
            base[(size_t)e * PPR + piece] = base[(size_t)k * PPR + piece];
        } else if (tid == 2 * PPR) {
            fu[e] = fu[k];
        } else if (tid == 2 * PPR + 1) {
            pu[e] = newest;
        }
    }
    if (tid == 0) a.len[u] = k;
}

// Decode-shape eviction in the ordered layout, first of two launches ("wide" mode, for workloads whose
// units are too few or too long for one workgroup each to move the rows): find the evicted slot e exactly
// as evict_one does, and save the entries at slots R, 2R, ... behind it.  The second launch gives every
// R-slot chunk of [e, k) to a workgroup of its own; a chunk's last source is the next chunk's first
// destination, and that one entry is read from the copy saved here, so the chunks need no order.
template <int NT>
__device__ __forceinline__ void evict_find(const SelectArgs& a, int64_t u, int n, bool write_idx) {
    constexpr int NW = NT / kWave;
    __shared__ unsigned long long wmin_f[NW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int k = a.k, w = a.w;
    const int ncand = n - w;
    const float* fu = a.score + (size_t)u * a.cap;
    const int32_t* pu = a.pos + (size_t)u * a.cap;
    int e;
    if (a.presel) {
        e = presel_pick(a, u);  // the launch ahead scanned the candidates
    } else {
        unsigned long long best = ~0ull;
        for (int j = tid; j < ncand; j += NT) {
            const unsigned long long pack = ((unsigned long long)float_key(fu[j]) << 32) | (uint32_t)(~(uint32_t)j);
            best = pack < best ? pack : best;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long t = __shfl_xor(best, o, kWave);
            best = t < best ? t : best;
        }
        if (lane == 0) wmin_f[wv] = best;
        __syncthreads();
        best = wmin_f[0];
#pragma unroll
        for (int i = 1; i < NW; ++i) best = wmin_f[i] < best ? wmin_f[i] : best;
        e = (int)(~(uint32_t)(best & 0xFFFFFFFFull));  // evicted slot, in [0, ncand)
    }
    if (write_idx) {
        int32_t* idx = a.idx + (size_t)u * k;
        for (int i = tid; i < k; i += NT) idx[i] = i + (i >= e ? 1 : 0);
    }
    // boundary entries at slots b = (c+1)*R with e < b <= k
    const int R = a.chunk_rows, PPR = a.row_bytes >> 4;
    const int c0 = e / R, c1 = k / R;  // boundaries c0 .. c1-1
    const uint4* Kr = (const uint4*)((const char*)a.K + (size_t)u * a.cap * a.row_bytes);
    const uint4* Vr = (const uint4*)((const char*)a.V + (size_t)u * a.cap * a.row_bytes);
    uint4* brow = (uint4*)((char*)a.ws_brow + (size_t)u * a.nb * 2 * a.row_bytes);
    const int per = 2 * PPR;  // pieces per boundary: the K row, then the V row
    for (int p = tid; p < (c1 - c0) * per; p += NT) {
        const int c = c0 + p / per, q = p % per;
        const int b = (c + 1) * R;
        brow[(size_t)c * per + q] = (q < PPR) ? Kr[(size_t)b * PPR + q] : Vr[(size_t)b * PPR + q - PPR];
    }
    for (int c = c0 + tid; c < c1; c += NT) {
        a.ws_bscore[(size_t)u * a.nb + c] = fu[(c + 1) * R];
        a.ws_bpos[(size_t)u * a.nb + c] = pu[(c + 1) * R];
    }
    if (tid == 0) {
        a.ws_evict[u] = e;
        a.len[u] = k;
    }
}

// Second launch of the wide mode: workgroup (unit u, chunk c) moves entries [max(e, cR)+1, min(k, (c+1)R)]
// down by one slot.  Everything it reads is in registers before its one barrier; its last source, if it is
// the next chunk's first destination, comes from the copy the first launch saved.
constexpr int kWideThreads = 256;
constexpr int kWidePieces = 2048 / kWideThreads;  // 16-byte pieces per thread and tensor
__global__ void __launch_bounds__(kWideThreads) shift_chunk_kernel(const SelectArgs a, int nchunks, int64_t units) {
    // chunk-major: the chunks that have work are the same few of every unit (those behind the evicted slot),
    // and consecutive workgroup ids go round-robin to the 8 XCDs -- unit-major ids would park all the work on
    // the XCDs those chunk numbers map to (measured: half the chip idle, 84 instead of 40 us)
    const int64_t u = blockIdx.x % units;
    const int c = (int)(blockIdx.x / units);
    const int e = a.ws_evict[u];
    if (e < 0) return;
    const int R = a.chunk_rows, k = a.k, PPR = a.row_bytes >> 4;
    const int lo = max(e, c * R), hi = min(k, (c + 1) * R);
    if (lo >= hi) return;
    const int rows = hi - lo, bnd = (c + 1) * R;  // sources lo+1 .. hi; source `bnd` is saved
    const int tid = threadIdx.x;
    uint4* Kr = (uint4*)((char*)a.K + (size_t)u * a.cap * a.row_bytes);
    uint4* Vr = (uint4*)((char*)a.V + (size_t)u * a.cap * a.row_bytes);
    const uint4* brow = (const uint4*)((const char*)a.ws_brow + ((size_t)u * a.nb + c) * 2 * a.row_bytes);
    float* fu = a.score + (size_t)u * a.cap;
    int32_t* pu = a.pos + (size_t)u * a.cap;
    // branch-free: a lane past the chunk's end re-reads the last source, the saved entry is a pointer choice
    uint4 kreg[kWidePieces], vreg[kWidePieces];
#pragma unroll
    for (int i = 0; i < kWidePieces; ++i) {
        const int p = tid + i * kWideThreads;
        const int q = p % PPR;
        const int src = lo + min(p / PPR, rows - 1) + 1;
        const uint4* ks = (src == bnd) ? brow + q : Kr + (size_t)src * PPR + q;
        const uint4* vs = (src == bnd) ? brow + PPR + q : Vr + (size_t)src * PPR + q;
        kreg[i] = stream_load(ks);
        vreg[i] = stream_load(vs);
    }
    float fs = 0.0f;
    int32_t ps = 0;
    if (tid < rows) {
        const int src = lo + tid + 1;
        fs = (src == bnd) ? a.ws_bscore[(size_t)u * a.nb + c] : fu[src];
        ps = (src == bnd) ? a.ws_bpos[(size_t)u * a.nb + c] : pu[src];
    }
    __syncthreads();  // (with its wait for the loads) every source of the chunk is in registers
#pragma unroll
    for (int i = 0; i < kWidePieces; ++i) {
        const int p = tid + i * kWideThreads;
        const int r = p / PPR, q = p % PPR;
        if (r < rows) {
            stream_store(Kr + (size_t)(lo + r) * PPR + q, kreg[i]);
            stream_store(Vr + (size_t)(lo + r) * PPR + q, vreg[i]);
        }
    }
    if (tid < rows) {
        fu[lo + tid] = fs;
        pu[lo + tid] = ps;
    }
}

// Selection and compaction of one unit by one workgroup.
template <int NT>
__device__ __forceinline__ void select_unit(const SelectArgs& a, int64_t u) {
    constexpr int NW = NT / kWave;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_bin, s_rem;
    __shared__ uint32_t wtot[NW][2];
    __shared__ int s_first;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n = a.len[u];
    const int k = a.k, w = a.w;
    int32_t* idx = a.idx + (size_t)u * k;

    if (a.wide && tid == 0) a.ws_evict[u] = -1;  // unless the decode-shape branch below says otherwise
    if (n <= k) {  // under budget: nothing leaves
        if (a.idx_is_output || !a.move)
            for (int i = tid; i < k; i += NT) idx[i] = (i < n) ? i : -1;
        return;
    }
    if (a.layout == KF_LAYOUT_SLOT) {
        if (n == k + 1) {
            evict_one_slot<NT>(a, u, n, a.idx_is_output != 0);
        } else if (tid == 0) {
            atomicAdd(a.ws_err, 1);  // more than one token over budget: not handled in this layout
        }
        return;
    }
    if (n == k + 1 && a.move) {  // decode shape
        if (a.wide) {
            __syncthreads();  // the -1 above is stored before this workgroup's own slot number
            evict_find<NT>(a, u, n, a.idx_is_output != 0);
        } else {
            evict_one<NT>(a, u, n, a.idx_is_output != 0);
        }
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
    if (!a.move) return;  // index list only: the rows are gathered into another cache by gather_kernel

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
            rk[g] = make_uint4(0u, 0u, 0u, 0u);
            rv[g] = make_uint4(0u, 0u, 0u, 0u);
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

// Last launch of a step whose number lives in device memory: one lane moves the
// counter on.  No workgroup of this launch reads the counter, and the next
// step's launches start after this one has drained.
__device__ __forceinline__ void advance_step(const SelectArgs& a) {
    if (a.step_inc && blockIdx.x == 0 && threadIdx.x == 0) *a.step_inc += 1;
}

template <int NT>
__global__ void __launch_bounds__(NT) select_kernel(const SelectArgs a) {
    select_unit<NT>(a, (int64_t)blockIdx.x);
    advance_step(a);
}

// Tail of a fused generation step: merge the decode kernel's split records of
// the unit (attention output, score accumulation, new length), then select and
// compact -- one launch instead of two.
template <int D, int NT, int G>
__global__ void __launch_bounds__(NT) step_tail_kernel(const DecodeArgs d, const SelectArgs a) {
    __shared__ float w_p[G * kDecodeMaxSplits], w_e[G * kDecodeMaxSplits];
    const int64_t u = blockIdx.x;
    const int len0 = d.len[u];
    if (len0 >= 0 && len0 < d.cap && len0 <= d.S * d.chunk) {  // else: skipped by the split kernel too
        merge_unit<D, NT, G>(d, u, len0, w_p, w_e, 0, len0 + 1, true);
        __syncthreads();  // the merged scores and the new length are visible to the whole workgroup
    } else if (d.pre_slices > 0 && len0 == d.pre_k + 1) {
        scan_slice_min<NT>(d, u, len0, 0, len0, 0);  // the selection below takes the evicted slot from the table
        __syncthreads();
    }
    select_unit<NT>(a, u);
    advance_step(a);
}

template <int NT, int G>
static hipError_t launch_step_tail_g(const DecodeArgs& d, const SelectArgs& a, int64_t U, int32_t hd,
                                     hipStream_t stream) {
    const dim3 grid((unsigned)U), block(NT);
    if (hd == 64) hipLaunchKernelGGL((step_tail_kernel<64, NT, G>), grid, block, 0, stream, d, a);
    else if (hd == 128) hipLaunchKernelGGL((step_tail_kernel<128, NT, G>), grid, block, 0, stream, d, a);
    else if (hd == 256) hipLaunchKernelGGL((step_tail_kernel<256, NT, G>), grid, block, 0, stream, d, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int NT>
static hipError_t launch_step_tail_nt(const DecodeArgs& d, const SelectArgs& a, int64_t U, int32_t hd,
                                      hipStream_t stream) {
    switch (d.G) {
        case 1: return launch_step_tail_g<NT, 1>(d, a, U, hd, stream);
        case 2: return launch_step_tail_g<NT, 2>(d, a, U, hd, stream);
        case 4: return launch_step_tail_g<NT, 4>(d, a, U, hd, stream);
        case 8: return launch_step_tail_g<NT, 8>(d, a, U, hd, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_step_tail(const DecodeArgs& d, const SelectArgs& a, int64_t U, int32_t hd, hipStream_t stream) {
    if (a.layout == KF_LAYOUT_SLOT) return launch_step_tail_nt<kSelectThreadsSlot>(d, a, U, hd, stream);
    return launch_step_tail_nt<kSelectThreads>(d, a, U, hd, stream);
}

// Out-of-place compaction: survivor i of unit u (slot idx[u][i] of the source
// cache) goes to slot i of the destination cache.  Source and destination do
// not overlap, so any number of workgroups can share a unit: a workgroup copies
// kGatherRows rows, a lane one 16-byte piece of K or V.
constexpr int kGatherThreads = 256;
constexpr int kGatherRows = 64;

__global__ void __launch_bounds__(kGatherThreads) gather_kernel(const GatherArgs g) {
    const int64_t u = blockIdx.y + (int64_t)blockIdx.z * gridDim.y;
    if (u >= g.units) return;
    const int64_t ud = u + g.dst_unit0;
    const int tid = threadIdx.x;
    const int k = g.k;
    const int32_t* idx = g.idx + (size_t)u * k;
    const int row0 = blockIdx.x * kGatherRows;
    const int PPR = g.row_bytes >> 4;
    const uint4* Ks = (const uint4*)((const char*)g.src_K + (size_t)u * g.src_cap * g.row_bytes);
    const uint4* Vs = (const uint4*)((const char*)g.src_V + (size_t)u * g.src_cap * g.row_bytes);
    uint4* Kd = (uint4*)((char*)g.dst_K + (size_t)ud * g.dst_cap * g.row_bytes);
    uint4* Vd = (uint4*)((char*)g.dst_V + (size_t)ud * g.dst_cap * g.row_bytes);
    const int pieces = kGatherRows * PPR;  // per tensor
    for (int p = tid; p < 2 * pieces; p += kGatherThreads) {
        const int t = p >= pieces, q = t ? p - pieces : p;
        const int i = row0 + q / PPR, piece = q % PPR;
        if (i < k) {
            const int s = idx[i];
            if (s >= 0 && s < g.src_cap) {
                const uint4 v = stream_load((t ? Vs : Ks) + (size_t)s * PPR + piece);
                stream_store((t ? Vd : Kd) + (size_t)i * PPR + piece, v);
            }
        }
    }
    if (tid < kGatherRows) {
        const int i = row0 + tid;
        if (i < k) {
            const int s = idx[i];
            if (s >= 0 && s < g.src_cap) {
                g.dst_score[(size_t)ud * g.dst_cap + i] = g.src_score[(size_t)u * g.src_cap + s];
                g.dst_pos[(size_t)ud * g.dst_cap + i] = g.src_pos[(size_t)u * g.src_cap + s];
            }
        }
    }
    if (blockIdx.x == 0 && tid == 0) g.dst_len[ud] = min(g.src_len[u], k);
}

hipError_t launch_gather(const GatherArgs& g, hipStream_t stream) {
    const unsigned gy = (unsigned)(g.units < 32768 ? g.units : 32768);
    const unsigned gz = (unsigned)((g.units + gy - 1) / gy);
    const dim3 grid((unsigned)((g.k + kGatherRows - 1) / kGatherRows), gy, gz);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(kGatherThreads), 0, stream, g);
    return hipGetLastError();
}

// Beam fork (beam search, one cache per beam): gridDim.x workgroups share the live rows of a destination unit
// and copy them from the parent beam's unit -- a lane one 16-byte piece of K or V at a time, four in flight --
// with their scores and positions.  The parent's row of the batch is only read in this launch (it continues
// itself), so source and destination never meet.  Few, looping workgroups per unit rather than one per 64
// rows: most calls fork few beams or none, and a workgroup that finds nothing to do still costs its launch.
constexpr int kForkDepth = 4;
__global__ void __launch_bounds__(kGatherThreads) fork_kernel(const ForkArgs f) {
    const int64_t u = blockIdx.y + (int64_t)blockIdx.z * gridDim.y;  // destination unit
    const int64_t units = (int64_t)f.L * f.B * f.H;
    if (u >= units) return;
    const int h = (int)(u % f.H), b = (int)((u / f.H) % f.B);
    const int64_t l = u / ((int64_t)f.H * f.B);
    const int pb = f.parent[b];
    if (pb == b) return;
    if (pb < 0 || pb >= f.B || f.parent[pb] != pb) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicAdd(f.ws_err, 1);
        return;
    }
    const int64_t us = (l * f.B + pb) * f.H + h;  // source unit
    const int n = min(max(f.len[us], 0), f.cap);
    if (blockIdx.x == 0 && threadIdx.x == 0) f.len[u] = n;
    const int per = (n + (int)gridDim.x - 1) / (int)gridDim.x;
    const int row0 = (int)blockIdx.x * per, row1 = min(n, row0 + per);
    if (row0 >= row1) return;
    const int tid = threadIdx.x;
    const int PPR = f.row_bytes >> 4;
    const size_t so = (size_t)us * f.cap * PPR + (size_t)row0 * PPR, dof = (size_t)u * f.cap * PPR + (size_t)row0 * PPR;
    const int pieces = (row1 - row0) * PPR;  // per tensor; the rows of a slice are contiguous
    for (int p0 = tid; p0 < 2 * pieces; p0 += kForkDepth * kGatherThreads) {
        uint4 v[kForkDepth];
#pragma unroll
        for (int i = 0; i < kForkDepth; ++i) {
            const int p = p0 + i * kGatherThreads;
            v[i] = make_uint4(0u, 0u, 0u, 0u);
            if (p < 2 * pieces) v[i] = stream_load((p >= pieces ? (const uint4*)f.V + so + (p - pieces) : (const uint4*)f.K + so + p));
        }
#pragma unroll
        for (int i = 0; i < kForkDepth; ++i) {
            const int p = p0 + i * kGatherThreads;
            if (p < 2 * pieces) stream_store((p >= pieces ? (uint4*)f.V + dof + (p - pieces) : (uint4*)f.K + dof + p), v[i]);
        }
    }
    for (int r = row0 + tid; r < row1; r += kGatherThreads) {
        f.score[(size_t)u * f.cap + r] = f.score[(size_t)us * f.cap + r];
        f.pos[(size_t)u * f.cap + r] = f.pos[(size_t)us * f.cap + r];
    }
}

hipError_t launch_fork(const ForkArgs& f, hipStream_t stream) {
    const int64_t units = (int64_t)f.L * f.B * f.H;
    const unsigned gy = (unsigned)(units < 32768 ? units : 32768);
    const unsigned gz = (unsigned)((units + gy - 1) / gy);
    // slices per unit: about 64 KB of rows each, at most 16, fewer when the units alone fill the chip
    const int64_t unit_bytes = 2 * (int64_t)f.cap * f.row_bytes;
    int64_t slices = (unit_bytes + 65535) / 65536;
    if (slices > 16) slices = 16;
    while (slices > 1 && units * slices > 4096) slices >>= 1;
    const dim3 grid((unsigned)slices, gy, gz);
    hipLaunchKernelGGL(fork_kernel, grid, dim3(kGatherThreads), 0, stream, f);
    return hipGetLastError();
}

hipError_t launch_select(const SelectArgs& a, int64_t U, hipStream_t stream) {
    const dim3 grid((unsigned)U);
    if (a.presel && !a.presel_done) {
        hipLaunchKernelGGL(presel_kernel, dim3((unsigned)(U * a.presel)), dim3(kPreselThreads), 0, stream, a, U);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    if (a.layout == KF_LAYOUT_SLOT)
        hipLaunchKernelGGL((select_kernel<kSelectThreadsSlot>), grid, dim3(kSelectThreadsSlot), 0, stream, a);
    else
        hipLaunchKernelGGL((select_kernel<kSelectThreads>), grid, dim3(kSelectThreads), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.wide) e = launch_shift(a, U, stream);
    return e;
}

// Second launch of the two-launch eviction: every chunk of rows behind the evicted slot moves down by one.
hipError_t launch_shift(const SelectArgs& a, int64_t U, hipStream_t stream) {
    const int nchunks = (a.k + a.chunk_rows - 1) / a.chunk_rows;
    hipLaunchKernelGGL(shift_chunk_kernel, dim3((unsigned)(U * nchunks)), dim3(kWideThreads), 0, stream, a, nchunks, U);
    return hipGetLastError();
}

}  // namespace kf
