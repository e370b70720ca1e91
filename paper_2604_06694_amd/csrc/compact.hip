// Stage 5: gather the retained K/V rows into the packed cache.
// Pure data movement: every row is d*2 bytes (128-512 B), moved as 16-byte
// vectors so that a row is read and written by 8-32 adjacent lanes.
#include "common.h"

namespace audiokv {

namespace {

constexpr int kThreads = 256;
constexpr int kRowsInFlight = 8;   // independent rows per thread: loads issued before stores

// Largest g with cu_b[g] <= p (cu_b is a non-decreasing exclusive scan, cu_b[n] = total).
__device__ __forceinline__ int head_of_row(const int32_t* __restrict__ cu_b, int n_heads, int p) {
    int lo = 0, hi = n_heads;           // invariant: cu_b[lo] <= p < cu_b[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu_b[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes; the nontemporal builtins need a native vector

template <int VEC_PER_ROW>   // 16-byte vectors per row = D * 2 / 16
__global__ __launch_bounds__(kThreads) void compact_kernel(
    Geom g, const u32x4* __restrict__ k, const u32x4* __restrict__ v,
    const int32_t* __restrict__ indices, const int32_t* __restrict__ cu_b,
    const int32_t* __restrict__ cu_seq, int n_heads, int64_t total_rows,
    u32x4* __restrict__ k_out, u32x4* __restrict__ v_out)
{
    constexpr int ROWS_PER_PASS = kThreads / VEC_PER_ROW;
    const int sub = threadIdx.x / VEC_PER_ROW;     // row within a pass
    const int vec = threadIdx.x % VEC_PER_ROW;     // 16-byte piece of the row
    const int64_t row0 = (int64_t)blockIdx.x * (ROWS_PER_PASS * kRowsInFlight);

    // The block's rows are consecutive output rows: find the head of the first one once (uniform, so the
    // search runs on scalar loads), then every row only walks forward from there.
    const int head0 = head_of_row(cu_b, n_heads, (int)row0);

    // Nothing below branches around a load: rows past the end are clamped to the last row and simply not
    // stored, so all gathers of the block are in flight together.
    int64_t src[kRowsInFlight];
#pragma unroll
    for (int r = 0; r < kRowsInFlight; ++r) {
        const int p = (int)min(row0 + r * ROWS_PER_PASS + sub, total_rows - 1);
        int gh = head0;
        while (gh + 1 < n_heads && cu_b[gh + 1] <= p) ++gh;
        const int item = gh / g.H_kv, h = gh - item * g.H_kv;
        const int tok0 = cu_seq[item];
        const int L = cu_seq[item + 1] - tok0;
        // an index outside the item is a caller error; clamp so that it can never fault
        const int j = min(max(indices[p], 0), L - 1);
        src[r] = kv_row_offset(g, item, tok0, L, h, j) / 8 + vec;   // in u32x4 units (8 bf16; strides are multiples of 8)
    }
    u32x4 kk[kRowsInFlight], vv[kRowsInFlight];
#pragma unroll
    for (int r = 0; r < kRowsInFlight; ++r) {
        kk[r] = __builtin_nontemporal_load(k + src[r]);
        vv[r] = __builtin_nontemporal_load(v + src[r]);
    }
#pragma unroll
    for (int r = 0; r < kRowsInFlight; ++r) {
        const int64_t p = row0 + r * ROWS_PER_PASS + sub;
        if (p < total_rows) {
            __builtin_nontemporal_store(kk[r], k_out + p * VEC_PER_ROW + vec);
            __builtin_nontemporal_store(vv[r], v_out + p * VEC_PER_ROW + vec);
        }
    }
}

}  // namespace

hipError_t launch_compact(const Geom& g, const void* k, const void* v, const int32_t* indices,
                          const int32_t* cu_budgets, const int32_t* cu_seqlens, int64_t total_rows,
                          void* k_out, void* v_out, hipStream_t s)
{
    if (total_rows <= 0) return hipSuccess;
    const int n_heads = g.n_items * g.H_kv;
    const int vec_per_row = g.D / 8;
    const int rows_per_block = (kThreads / vec_per_row) * kRowsInFlight;
    const unsigned blocks = (unsigned)((total_rows + rows_per_block - 1) / rows_per_block);
#define AUDIOKV_LAUNCH_COMPACT(V)                                                                   \
    hipLaunchKernelGGL((compact_kernel<V>), dim3(blocks), dim3(kThreads), 0, s, g,                  \
                       (const u32x4*)k, (const u32x4*)v, indices, cu_budgets, cu_seqlens, n_heads, \
                       total_rows, (u32x4*)k_out, (u32x4*)v_out)
    switch (vec_per_row) {
        case 8:  AUDIOKV_LAUNCH_COMPACT(8);  break;
        case 16: AUDIOKV_LAUNCH_COMPACT(16); break;
        case 32: AUDIOKV_LAUNCH_COMPACT(32); break;
        default: return hipErrorInvalidValue;
    }
#undef AUDIOKV_LAUNCH_COMPACT
    return hipGetLastError();
}

}  // namespace audiokv
