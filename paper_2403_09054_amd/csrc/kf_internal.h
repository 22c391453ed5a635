// Host-side declarations shared by the API layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/keyformer.h"

namespace kf {

// ------------------------------------------------------------------ decode
struct DecodeArgs {
    void* K;
    void* V;
    float* score;
    int32_t* pos;
    int32_t* len;
    const void* q;
    const void* k_new;
    const void* v_new;
    float* out;
    const uint64_t* seeds;
    const float* slopes;
    float* ws_part;    // [U][S][G][D+4] partial outputs and softmax statistics of each split and query head
    float* ws_e;       // [U][G][cap]    un-normalised score increments of each token
    int32_t* ws_err;   // [1]         skipped-unit counter
    int32_t* ws_m;     // [U]         tokens this launch scored in each unit (0: skipped); written when split or shared
    int32_t B, H, cap, layer0;
    int32_t G;         // query heads per cached head (q and out hold H*G heads)
    int32_t S;         // splits of a unit's token range
    int32_t chunk;     // tokens per split
    int32_t q_pos;
    int32_t noise;
    int32_t new_pos;   // position bias from slot indices instead of original positions
    int32_t shared;    // one score for all layers: leave the normalised increments in ws_e, do not touch score
    // Step taken from device memory (non-NULL `step`): t = *step, q_pos = n0 + t - 1,
    // tau = tau_init + min(t, T)*dtau; q_pos and inv_tau above are then ignored.
    const int32_t* step;
    int32_t n0, T;
    float tau_init, dtau;
    // Per-sequence query position / temperature (either may be NULL): [B], override the above.
    const int32_t* seq_q_pos;
    const float* seq_tau;
    // Whole step in this launch (single split, slot layout): after the scores are updated the workgroup
    // evicts for its unit and stores the new token straight into the freed slot.  fuse_k = 0: off.
    int32_t fuse_k, fuse_w;
    int32_t* fuse_idx;  // NULL, or [U][k] survivor list as the selection kernel writes it
    int32_t* step_inc;   // NULL, or the device step counter the launch's last workgroup advances (whole-step launch)
    int32_t* ws_ticket;  // [1] workgroups of this launch that are done (zero between launches)
    // Fused step of few, long units: the merge launch (pre_slices workgroups per unit) also leaves, per
    // workgroup, the smallest eviction candidate among the tokens it updated -- what the selection's own
    // candidate scan launch would compute from the finished scores.  pre_slices = 0: off.
    int32_t pre_slices, pre_k, pre_w, pre_layout;
    unsigned long long* pre_min;  // [U][pre_slices] (score key, tie-break) pack, ~0 if the slice has no candidate
    int32_t* pre_slot;            // [U][pre_slices] its slot
    float inv_tau;
    float scale;
};

// Launch shape of the decode kernel for U units of up to m tokens.
struct DecodePlan {
    int32_t S, chunk;
    size_t lds_bytes;
};
DecodePlan plan_decode(int64_t U, int32_t m, int32_t d, int32_t dtype, int32_t G);
hipError_t launch_decode(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                         hipStream_t stream);
// Workgroups per unit of the merge launch that follows a split decode launch.
int32_t decode_merge_slices(int32_t S, int32_t chunk);

// Shared score function: adds up the layers' contributions and gives every layer the same score.
//   inc != NULL (decode): score[l][bh][j] += sum_l' inc[l'][bh][j] for the m[.][bh] tokens just scored
//   inc == NULL (prompt): score[l][bh][j]  = sum_l' score[l'][bh][j] for j < n
struct ShareArgs {
    float* score;
    const float* inc;
    const int32_t* m;   // decode: [L][BH] tokens scored per unit;  prompt: the caches' len
    int32_t* ws_err;
    int32_t L, BH, cap;
    int32_t inc_unit;   // floats between the increments of consecutive units (G*cap)
};
hipError_t launch_share(const ShareArgs& a, hipStream_t stream);

// ------------------------------------------------------------------ select
struct SelectArgs {
    void* K;
    void* V;
    float* score;
    int32_t* pos;
    int32_t* len;
    int32_t* idx;       // [U][k] source slot of every survivor (caller's kept_idx or workspace)
    int32_t cap, k, w;
    int32_t row_bytes;  // d * sizeof(element)
    int32_t idx_is_output;  // idx is the caller's kept_idx (must be complete), not scratch
    int32_t layout;         // kf_layout
    int32_t move;           // 0: only write the survivor index list (rows are gathered elsewhere)
    int32_t* ws_err;        // [1] skipped-unit counter
    int32_t* step_inc;      // NULL, or the device step counter this launch advances by one when it is done
    // Ordered layout, decode shape, rows moved by a second launch of several workgroups per unit
    // ("wide"): the selection launch only finds the evicted slot and saves the chunk-boundary entries.
    int32_t wide;           // 0: the selection workgroup moves the rows itself
    int32_t chunk_rows;     // R: rows a workgroup of the second launch moves
    int32_t nb;             // boundary slots kept per unit: cap / R
    int32_t* ws_evict;      // [U]                  evicted slot, or -1 (nothing for the second launch)
    void* ws_brow;          // [U][nb][2][row_bytes] K and V rows at slots R, 2R, ... saved before anything moves
    float* ws_bscore;       // [U][nb]              their scores
    int32_t* ws_bpos;       // [U][nb]              their positions
    // Long units in the decode shape: a launch ahead of the selection cuts the candidate scan of a unit
    // into `presel` slices, one workgroup each, and leaves every slice's smallest candidate here.
    int32_t presel;             // 0: the selection workgroup scans the candidates itself
    int32_t presel_done;        // the slices' minima are there already (left by the decode merge launch)
    unsigned long long* ws_pmin;  // [U][presel] smallest (score key, tie-break) pack of the slice, ~0 if none
    int32_t* ws_pslot;          // [U][presel] its slot
};
constexpr int32_t kPreselMaxSlices = 16;
// rows per workgroup of the wide shift: 2048 16-byte pieces per tensor, i.e. 32 KB of K and 32 KB of V
inline int32_t wide_chunk_rows(int32_t row_bytes) { return 2048 / (row_bytes >> 4); }
hipError_t launch_select(const SelectArgs& a, int64_t U, hipStream_t stream);
struct GatherArgs {
    const void* src_K;
    const void* src_V;
    const float* src_score;
    const int32_t* src_pos;
    const int32_t* src_len;
    void* dst_K;
    void* dst_V;
    float* dst_score;
    int32_t* dst_pos;
    int32_t* dst_len;
    const int32_t* idx;  // [units][k] survivor slots in the source
    int64_t units;       // units of the source cache
    int64_t dst_unit0;   // first destination unit (dst_layer0 * B * H)
    int32_t src_cap, dst_cap, k, row_bytes;
};
hipError_t launch_gather(const GatherArgs& g, hipStream_t stream);

// Beam fork: row b of the batch takes over the state of row parent[b] (see kf_beam_fork).
struct ForkArgs {
    void* K;
    void* V;
    float* score;
    int32_t* pos;
    int32_t* len;
    const int32_t* parent;  // [B]
    int32_t* ws_err;
    int32_t L, B, H, cap, row_bytes;
};
hipError_t launch_fork(const ForkArgs& f, hipStream_t stream);
// decode merge + select + compact of every unit in one launch (after the split kernel of a fused step)
hipError_t launch_step_tail(const DecodeArgs& d, const SelectArgs& a, int64_t U, int32_t hd, hipStream_t stream);
// the row-shifting launch of the two-launch eviction (after a selection launch that ran with a.wide set)
hipError_t launch_shift(const SelectArgs& a, int64_t U, hipStream_t stream);
// the split kernel alone (no merge launch): first half of a fused step
hipError_t launch_decode_split(const DecodeArgs& a, int64_t U, int32_t d, int32_t dtype, size_t lds_bytes,
                               hipStream_t stream);

// ------------------------------------------------------------------ prefill
struct PrefillArgs {
    const void* Q;
    const void* K;
    float* score;
    int32_t* pos;
    int32_t* len;
    const uint64_t* seeds;
    const float* slopes;
    const int32_t* seq_n;  // [B] per-sequence prompt length, or null: every sequence has n rows
    int32_t* ws_err;       // device error counter
    float* ws_c;        // [U][n_pad] per-row log2 normaliser            (U = L*B*H query units)
    uint32_t* ws_r;     // [U][n_pad] per-row noise key
    float* ws_f;        // [U][n_pad] per-query-head column sums (G > 1 only)
    int32_t B, H, cap, layer0, n, n_pad;  // H counts QUERY heads; the caches hold H/G heads
    int32_t G;          // query heads per cached head
    int32_t noise;
    float inv_tau;
    float scale;
};
hipError_t launch_prefill(const PrefillArgs& a, int64_t U, int32_t d, int32_t dtype, hipStream_t stream);

constexpr int32_t kPrefillRowPad = 128;  // n is padded to this for the row-statistics arrays

}  // namespace kf
