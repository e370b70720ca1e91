// Shared declarations of the gfx950 kernels behind the AudioKV C ABI.
// Device code only needs hip_runtime; nothing here depends on torch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "audiokv.h"

namespace audiokv {

// Geometry handed to kernels by value.
struct Geom {
    int n_items;
    int H_q;
    int H_kv;
    int G;          // H_q / H_kv
    int D;          // head_dim
    int W;          // window
    int pool_kernel;
    int pool_mode;
    int causal;
    int layout;     // AUDIOKV_LAYOUT_*
    float c_log2;   // softmax scale * log2(e): logits are handled in base-2 units
    int cutoff_mode;   // AUDIOKV_CUTOFF_*
    int taper_bins;    // cosine roll-off bins after k*
    // explicit K/V strides in elements (all zero: the packed layout named by `layout`)
    int64_t s_item, s_head, s_tok;
};

// Elements between consecutive tokens of one head.
__device__ __forceinline__ int64_t kv_tok_stride(const Geom& g) {
    if (g.s_tok) return g.s_tok;
    return g.layout == AUDIOKV_LAYOUT_HEAD_MAJOR ? (int64_t)g.D : (int64_t)g.H_kv * g.D;
}

// Where head (item, h), token j starts inside the K/V buffers (in elements). item_tok0 = cu_seqlens[item].
__device__ __forceinline__ int64_t kv_row_offset(const Geom& g, int item, int64_t item_tok0, int L, int h, int j) {
    if (g.s_tok) return (int64_t)item * g.s_item + (int64_t)h * g.s_head + (int64_t)j * g.s_tok;
    const int64_t base = item_tok0 * g.H_kv * g.D;
    if (g.layout == AUDIOKV_LAYOUT_HEAD_MAJOR)
        return base + ((int64_t)h * L + j) * g.D;
    return base + ((int64_t)j * g.H_kv + h) * g.D;
}

// ---- launchers (defined in the .hip files, called from api.hip) ------------

// Arguments of launch_allocate, for callers that let the allocation ride along with another small launch.
struct AllocateJob {
    const float* weights; int n_segments, heads_per_segment, weight_group; const int32_t* cu_seqlens;
    double ratio, floor_frac; int32_t* budgets; int32_t* cu_budgets;
};
// Merge of the per-range row statistics of sweep 1 (stats: [head][nsplit][rows_pad][2]) into one constant per row
// (cst: [head][rows_pad], max + log2(sum); +inf for rows >= R). With `job`, the same launch also runs the budget
// allocation in extra workgroups: neither depends on the other, and each launch costs more than either's work.
hipError_t launch_score_merge(const Geom& g, const float* stats, int nsplit, int rows_pad, float* cst,
                              const AllocateJob* job, hipStream_t s);

// Number of key-range splits per head used by the score kernels; a pure
// function of the batch so that the workspace query and the launch agree.
int score_num_splits(int H_kv, int n_items, const int32_t* seqlens_host, int rows, int D);
// Padded row count (multiple of the MFMA row tiling) for G*W window rows; 0 if unsupported.
int score_padded_rows(int rows, int D);

// between_sweeps: optional event recorded on `s` after the first sweep (timing aid), or nullptr.
// lse: optional fp32 [items][H_q][W] natural-log softmax denominators of the window rows; given, sweep 1 is skipped.
// ride_along: optional allocation to run in the launch that merges the row statistics (ignored with lse: the caller
// must check score_merge_runs(lse) and launch the allocation itself when there is no merge).
hipError_t launch_score(const Geom& g, const void* q_win, const void* k, const int32_t* cu_seqlens,
                        const int32_t* seqlens_host, float* stats_ws, float* raw_out, hipStream_t s,
                        hipEvent_t between_sweeps = nullptr, const float* lse = nullptr,
                        float* raw_second = nullptr, size_t raw_elems = 0, const AllocateJob* ride_along = nullptr);
// More than 448 window rows (d <= 128): sweep 2 runs as two launches and needs a second buffer of the size of the
// scores (raw_second, raw_elems floats).
bool score_needs_second_raw(int rows, int D);
hipError_t launch_pool(const Geom& g, const float* raw, const int32_t* cu_seqlens, int max_L,
                       float* pooled, hipStream_t s);

hipError_t launch_allocate(const Geom& g, const float* weights, int n_segments, int heads_per_segment,
                           int weight_group, const int32_t* cu_seqlens, double ratio, double floor_frac,
                           int32_t* budgets, int32_t* cu_budgets, hipStream_t s);

// pool_on_load: input holds un-pooled scores and the pooling of Geom is applied while loading.
bool smooth_supported(int L);
// Global-memory scratch of the smoothing: what the transforms of lengths that are not powers of two need
// (_required: 0 when every length is a power of two), plus, for calls with few heads, room to spread a
// power-of-two head over several workgroups (_bytes: the sum; what the workspace query reserves).
size_t smooth_workspace_bytes(const int32_t* seqlens_host, int n_items, int H_kv);
size_t smooth_workspace_required(const int32_t* seqlens_host, int n_items, int H_kv);
// kstar_out (may be null): the cutoff bin of every head; cutoffs_only stops after writing it. workspace_bytes: what
// `workspace` holds (at least _required; with less than _bytes every power-of-two head runs in one workgroup).
hipError_t launch_smooth(const Geom& g, const float* in, bool pool_on_load, const int32_t* cu_seqlens,
                         const int32_t* seqlens_host, int n_items, double cutoff_frac, double alpha,
                         float* out, void* workspace, size_t workspace_bytes, int32_t* kstar_out, bool cutoffs_only,
                         hipStream_t s, bool filters_ready = false);
// Lengths that are not powers of two convolve with filters that depend on the lengths and the cutoff only:
// launch_smooth_filters prepares them in the workspace (launch_smooth does it itself unless told they are ready).
hipError_t launch_smooth_filters(const Geom& g, const int32_t* cu_seqlens, const int32_t* seqlens_host, int n_items,
                                 double cutoff_frac, void* workspace, hipStream_t s);

// single-query attention over the packed cache
bool decode_supported(int G);
size_t decode_workspace_bytes(const Geom& g, long long total_rows);
hipError_t launch_decode(const Geom& g, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* cu_budgets, long long total_rows, float* out, void* workspace, hipStream_t s);

bool select_supported(int L);
hipError_t launch_select(const Geom& g, const float* scores, const int32_t* budgets, const int32_t* cu_budgets,
                         const int32_t* cu_seqlens, int max_L, int32_t* indices, hipStream_t s);

hipError_t launch_compact(const Geom& g, const void* k, const void* v, const int32_t* indices,
                          const int32_t* cu_budgets, const int32_t* cu_seqlens, int64_t total_rows,
                          void* k_out, void* v_out, hipStream_t s);

}  // namespace audiokv
