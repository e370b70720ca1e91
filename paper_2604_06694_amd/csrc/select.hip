// Stage 4: per-head top-k with a forced window tail (paper Sec. 1, Solution 2:
// Top-K selection on the importance scores; window w of Sec. 3.1 Eq. 1).
//
// One workgroup per head. Scores become order-preserving 32-bit keys held in
// registers (a contiguous run of tokens per thread, staged through padded LDS
// so that both the global read and the per-thread read are conflict-free).
// The value of the k-th largest key is found bit by bit (32 counting passes,
// no atomics); tokens above it are kept, tokens equal to it are kept in index
// order until the budget is full, and kept indices are written in ascending
// order through a block-wide exclusive scan (gathered in LDS, stored coalesced).
// Integer-only: bit-exact.
#include "common.h"

namespace audiokv {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// float -> uint32 whose unsigned order is the float order; -0.0 and +0.0 map to one key
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Block-wide sum; every thread gets the result. `slots` has 2 * kSelWaves ints, `parity` alternates per call.
__device__ __forceinline__ int block_count(int v, int* slots, int parity) {
    v = wave_sum(v);
    int* s = slots + parity * kSelWaves;
    if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) t += s[w];
    return t;
}

// Block-wide exclusive scan of two counters at once; returns this thread's offsets, totals through pointers.
__device__ __forceinline__ void block_exscan2(int a, int b, int* slots /* 2*kSelWaves */, int& ea, int& eb) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ia = a, ib = b;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int ta = __shfl_up(ia, o, 64), tb = __shfl_up(ib, o, 64);
        if (lane >= o) { ia += ta; ib += tb; }
    }
    if (lane == 63) { slots[wave] = ia; slots[kSelWaves + wave] = ib; }
    __syncthreads();
    int pa = 0, pb = 0;
    for (int w = 0; w < wave; ++w) { pa += slots[w]; pb += slots[kSelWaves + w]; }
    ea = pa + ia - a;
    eb = pb + ib - b;
}

template <int EPT>   // tokens per thread; the head must have at most EPT * kSelThreads candidates
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    Geom g, const float* __restrict__ scores, const int32_t* __restrict__ budgets,
    const int32_t* __restrict__ cu_b, const int32_t* __restrict__ cu_seq, int32_t* __restrict__ indices)
{
    extern __shared__ float stage[];                 // EPT*kSelThreads floats + 1 pad per 32
    __shared__ int slots[4 * kSelWaves];
    const int head = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const float* s = scores + (size_t)tok0 * g.H_kv + (size_t)h * L;
    const int tid = threadIdx.x;

    const int W = min(g.W, L);
    const int n_cand = L - W;
    // never write past this head's slice of the output, whatever the caller's budgets say
    const int room = cu_b[head + 1] - cu_b[head];
    const int b = min(min(max(budgets[head], W), L), room);
    const int want = max(b - W, 0);                  // how many candidates to keep
    int32_t* out = indices + cu_b[head];

    // the forced window tail: highest indices, so they close the ascending list
    for (int w = tid; w < W; w += kSelThreads)
        if (want + w < room) out[want + w] = n_cand + w;
    if (want <= 0) return;
    if (n_cand > EPT * kSelThreads) return;          // launcher never allows this

    // global (coalesced) -> padded LDS -> registers (thread t owns tokens [t*EPT, t*EPT+EPT))
    for (int j = tid; j < n_cand; j += kSelThreads) stage[j + (j >> 5)] = s[j];
    __syncthreads();
    uint32_t key[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int j = tid * EPT + e;
        key[e] = j < n_cand ? order_key(stage[j + (j >> 5)]) : 0u;   // 0 is below every real key
    }

    // k-th largest key: the largest T with #(key >= T) >= want
    uint32_t T = 0;
    int parity = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        // wave-wide count on the scalar unit: one compare per key, its lane mask counted with a population count
        int c = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e) c += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] >= trial));
        int* sl = slots + parity * kSelWaves;
        if ((tid & 63) == 0) sl[tid >> 6] = c;
        __syncthreads();
        int t = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) t += sl[w];
        if (t >= want) T = trial;
        parity ^= 1;
    }
    // tokens strictly above T all stay; tokens equal to T stay in index order while room is left
    int c_gt = 0, c_eq = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int j = tid * EPT + e;
        const bool live = j < n_cand;
        c_gt += (live && key[e] > T) ? 1 : 0;
        c_eq += (live && key[e] == T) ? 1 : 0;
    }
    int gt_before, eq_before;
    block_exscan2(c_gt, c_eq, slots + 2 * kSelWaves, gt_before, eq_before);
    const int total_gt = block_count(c_gt, slots, parity);
    const int need_eq = want - total_gt;             // >= 1 by construction of T

    // Kept indices are gathered in LDS at their output slots (the staging buffer is free: the keys live in
    // registers) and then written out in one coalesced sweep; written straight from here, every store of a wave
    // would touch 64 different cache lines.
    int32_t* lds_out = reinterpret_cast<int32_t*>(stage);
    __syncthreads();                                 // all reads of the staged scores are long done; be explicit
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int j = tid * EPT + e;
        if (j >= n_cand) break;
        if (key[e] > T) {
            lds_out[gt_before + min(eq_before, need_eq)] = j;
            ++gt_before;
        } else if (key[e] == T) {
            if (eq_before < need_eq) lds_out[gt_before + eq_before] = j;
            ++eq_before;
        }
    }
    __syncthreads();
    for (int t = tid; t < want; t += kSelThreads) out[t] = lds_out[t];
}

}  // namespace

bool select_supported(int L) { return L >= 1 && L <= 32 * kSelThreads; }

hipError_t launch_select(const Geom& g, const float* scores, const int32_t* budgets, const int32_t* cu_budgets,
                         const int32_t* cu_seqlens, int max_L, int32_t* indices, hipStream_t s)
{
    const int n_heads = g.n_items * g.H_kv;
    const int ept_needed = (max_L + kSelThreads - 1) / kSelThreads;
#define AUDIOKV_LAUNCH_SELECT(E)                                                                        \
    do {                                                                                                \
        const size_t n = (size_t)(E) * kSelThreads;                                                     \
        const size_t smem = (n + n / 32 + 1) * sizeof(float);                                           \
        static bool attr_set = false;                                                                   \
        if (!attr_set && smem > 48 * 1024) {                                                            \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<E>),         \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);  \
            if (e != hipSuccess) return e;                                                              \
            attr_set = true;                                                                            \
        }                                                                                               \
        hipLaunchKernelGGL((select_kernel<E>), dim3(n_heads), dim3(kSelThreads), smem, s, g, scores,    \
                           budgets, cu_budgets, cu_seqlens, indices);                                   \
    } while (0)
    if (ept_needed <= 4) AUDIOKV_LAUNCH_SELECT(4);
    else if (ept_needed <= 16) AUDIOKV_LAUNCH_SELECT(16);
    else if (ept_needed <= 32) AUDIOKV_LAUNCH_SELECT(32);
    else return hipErrorInvalidValue;   // longer heads would need more than the 160 KiB of LDS staging
#undef AUDIOKV_LAUNCH_SELECT
    return hipGetLastError();
}

}  // namespace audiokv
