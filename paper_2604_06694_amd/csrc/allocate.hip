// Stage 2: head-wise budget allocation (paper Sec. 3.1 Eq. 1, Sec. 3.2 Eq. 12).
//
// One workgroup per budget pool ("segment"). All real arithmetic is float64
// with contraction off and with the order of operations of the plain
// definition (sum of weights accumulated in head order, share = (T*S)/sum),
// so the integers produced are reproducible bit for bit on any IEEE machine.
// Head-parallel steps (shares, floors, remainder ranks) are order-free.
//
// The merge of the score sweeps' per-range row statistics lives here too: it is
// as small as the allocation, neither depends on the other, and inside one
// call on one stream a launch costs more than either's work, so the
// allocation can ride along in extra workgroups of the merge launch.
#include "common.h"

#pragma clang fp contract(off)

namespace audiokv {

namespace {

constexpr int kThreads = 256;

struct AllocShared {
    long long leftover;
    long long isum;
    double tot;
    double T;
    int n_free;
    int granted;
};

// Sum of one integer per thread over the block (order does not matter for integers): lanes by shuffles, the four
// waves through `scratch` (at least kThreads / 64 entries). Two barriers: the second frees `scratch` for the next use.
__device__ long long block_sum_ll(long long v, long long* scratch) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    long long r = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) r += scratch[w];
    __syncthreads();
    return r;
}

__device__ __forceinline__ int n_keep_dev(double ratio, int L) {
    return (int)floor(__dadd_rn(__dmul_rn(ratio, (double)L), 0.5));
}

// the whole allocation of pool `seg` by one workgroup of kThreads threads; smem_raw: alloc_smem_bytes(n) bytes
__device__ __forceinline__ void allocate_pool(
    unsigned char* smem_raw, const int seg,
    const float* __restrict__ weights, int n_segments, int n, int weight_group, int window,
    const int32_t* __restrict__ cu_seq, double ratio, double beta,
    int32_t* __restrict__ budgets, int32_t* __restrict__ cu_budgets)
{
    // layout: S[n] x[n] frac[n] (double) | e[n] (int) | flag[n] (int) | red[kThreads] (ll) | AllocShared
    double* S = reinterpret_cast<double*>(smem_raw);
    double* x = S + n;
    double* frac = x + n;
    long long* red = reinterpret_cast<long long*>(frac + n);
    AllocShared* sh = reinterpret_cast<AllocShared*>(red + kThreads);
    int* e = reinterpret_cast<int*>(sh + 1);
    int* flag = e + n;      // bit 0: capped, bit 1: eligible in the current hand-out round

    const int tid = threadIdx.x;
    const int L = cu_seq[seg + 1] - cu_seq[seg];
    const int nk = n_keep_dev(ratio, L);
    const int r = (int)floor(__dmul_rn(beta, (double)(nk - window)));
    const int f = window + r;                       // w + r of Eq. 1
    const long long Bs = (long long)n * (nk - f);   // budget shared out by weight
    const int cap = L - f;                          // no head keeps more than L tokens

    // criticality per KV head (query-head weights summed inside each group, in index order)
    for (int h = tid; h < n; h += kThreads) {
        const float* w = weights + ((size_t)seg * n + h) * weight_group;
        double acc = 0.0;
        for (int q = 0; q < weight_group; ++q) acc = __dadd_rn(acc, (double)w[q]);
        S[h] = acc;
        x[h] = 0.0;
        flag[h] = 0;
    }
    __syncthreads();

    // proportional shares with the cap: heads over the cap are fixed at it and
    // the rest of the budget is shared again among the others
    for (;;) {
        // In-order float64 sum of the free heads' weights. The order is fixed (head 0, 1, 2, ...), so the adds form
        // one serial chain, kept as short as it can be: all threads first stage the addends (a capped head adds
        // +0.0, which leaves the sum as it is bit for bit; `frac` is free until the floors are taken) and count
        // the capped heads, then one thread adds them up, fetching sixteen at a time.
        long long my_cap = 0;
        for (int h = tid; h < n; h += kThreads) {
            const bool capped = (flag[h] & 1) != 0;
            frac[h] = capped ? 0.0 : S[h];
            my_cap += capped ? 1 : 0;
        }
        const int ncap = (int)block_sum_ll(my_cap, red);    // (its barriers also publish the addends)
        if (tid == 0) {
            constexpr int kBatch = 16;
            double tot = 0.0;
            for (int base = 0; base < n; base += kBatch) {
                double av[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) av[u] = frac[min(base + u, n - 1)];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) tot = __dadd_rn(tot, base + u < n ? av[u] : 0.0);
            }
            sh->tot = tot;
            sh->n_free = n - ncap;
            sh->T = (double)(Bs - (long long)ncap * cap);
        }
        __syncthreads();
        const double tot = sh->tot, T = sh->T;
        const int nfree = sh->n_free;
        int over = 0;
        for (int h = tid; h < n; h += kThreads) {
            if (!(flag[h] & 1)) {
                const double xh = tot > 0.0 ? __ddiv_rn(__dmul_rn(T, S[h]), tot) : __ddiv_rn(T, (double)nfree);
                x[h] = xh;
                if (xh > (double)cap) over = 1;
            }
        }
        const int any_over = __syncthreads_or(over);
        if (!any_over) break;
        for (int h = tid; h < n; h += kThreads) {
            if (!(flag[h] & 1) && x[h] > (double)cap) { flag[h] |= 1; x[h] = (double)cap; }
        }
        __syncthreads();
    }

    // floors and fractional parts
    long long my_sum = 0;
    for (int h = tid; h < n; h += kThreads) {
        if (flag[h] & 1) { e[h] = cap; frac[h] = 0.0; }
        else {
            const double fl = floor(x[h]);
            e[h] = (int)fl;
            frac[h] = __dsub_rn(x[h], fl);
        }
        my_sum += e[h];
    }
    const long long e_sum = block_sum_ll(my_sum, red);
    if (tid == 0) sh->leftover = Bs - e_sum;
    __syncthreads();

    // largest remainder: spare units go to the largest fractional parts, ties to
    // the lower head; (negative leftover, possible only through rounding of the
    // shares, takes units back from the smallest fractional parts, higher head first)
    for (;;) {
        const long long left = sh->leftover;
        if (left == 0) break;
        const bool give = left > 0;
        const long long want = give ? left : -left;
        // eligible heads compete with their fractional parts; the others get a value that is never ahead of anyone
        // (`x` is free once the floors are taken)
        for (int h = tid; h < n; h += kThreads) {
            const bool el = !(flag[h] & 1) && (give ? e[h] < cap : e[h] > 0);
            flag[h] = (flag[h] & 1) | (el ? 2 : 0);
            x[h] = el ? frac[h] : (give ? -1.0 : 2.0);
        }
        if (tid == 0) sh->granted = 0;
        __syncthreads();
        int my_granted = 0;
        for (int h = tid; h < n; h += kThreads) {
            if (!(flag[h] & 2)) continue;
            const double fh = frac[h];
            long long rank = 0;
            // (the other heads' values sixteen at a time: one LDS latency per batch instead of one per head)
            constexpr int kBatch = 16;
            for (int base = 0; base < n; base += kBatch) {
                double fo[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) fo[u] = x[min(base + u, n - 1)];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int o = base + u;
                    const bool ahead = give ? (fo[u] > fh || (fo[u] == fh && o < h))
                                            : (fo[u] < fh || (fo[u] == fh && o > h));
                    rank += (o < n && ahead) ? 1 : 0;
                }
            }
            if (rank < want) { e[h] += give ? 1 : -1; ++my_granted; }
        }
        if (my_granted) atomicAdd(&sh->granted, my_granted);
        __syncthreads();
        if (tid == 0) {
            const int gr = sh->granted;
            // no eligible head left: cannot happen for valid input (n_keep <= L); stop rather than spin
            sh->leftover = gr == 0 ? 0 : (give ? left - gr : left + gr);
        }
        __syncthreads();
    }

    // budgets and their exclusive scan; the scan base is the total of the pools before this one
    long long base = 0;
    for (int s2 = 0; s2 < seg; ++s2)
        base += (long long)n * n_keep_dev(ratio, cu_seq[s2 + 1] - cu_seq[s2]);
    const int per = (n + kThreads - 1) / kThreads;
    const int h0 = min(tid * per, n), h1 = min(h0 + per, n);
    long long chunk = 0;
    for (int h = h0; h < h1; ++h) chunk += f + e[h];
    // exclusive scan of the 256 chunk totals (integers: any order): lanes by shuffles, waves through `red`;
    // the total goes to the last segment's end marker
    long long incl = chunk;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long t = __shfl_up(incl, off, 64);
        if ((tid & 63) >= off) incl += t;
    }
    if ((tid & 63) == 63) red[tid >> 6] = incl;
    __syncthreads();
    long long before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        if (w < (tid >> 6)) before += red[w];
        total += red[w];
    }
    if (tid == 0 && seg == n_segments - 1) cu_budgets[(size_t)n_segments * n] = (int32_t)(base + total);
    long long run = base + before + incl - chunk;
    for (int h = h0; h < h1; ++h) {
        const int b = f + e[h];
        budgets[(size_t)seg * n + h] = b;
        cu_budgets[(size_t)seg * n + h] = (int32_t)run;
        run += b;
    }
}

__global__ __launch_bounds__(kThreads) void allocate_kernel(
    const float* __restrict__ weights, int n_segments, int n, int weight_group, int window,
    const int32_t* __restrict__ cu_seq, double ratio, double beta,
    int32_t* __restrict__ budgets, int32_t* __restrict__ cu_budgets)
{
    extern __shared__ unsigned char smem_raw[];
    allocate_pool(smem_raw, blockIdx.x, weights, n_segments, n, weight_group, window, cu_seq, ratio, beta, budgets, cu_budgets);
}

// Row r of head `head`: the per-range softmax statistics (reference in base-2 units, sum of exp2) of sweep 1 merged
// into max + log2(sum). The statistics are fetched sixteen ranges at a time, so that the loads overlap instead of
// forming a chain of memory latencies as long as the number of ranges, and merged as they come (one pass: a running
// reference and a sum rescaled when the reference rises). The multiply-adds are written out as fused ones: the
// result does not depend on how this file is compiled.
__device__ __forceinline__ void merge_row(const float* __restrict__ stats, int nsplit, int rows_pad, int R,
                                          int head, int r, float* __restrict__ cst)
{
    if (r >= rows_pad) return;
    float out = INFINITY;
    if (r < R) {
        const float2* hs = reinterpret_cast<const float2*>(stats) + (size_t)head * nsplit * rows_pad + r;
        float M = -INFINITY, Z = 0.f;
        for (int s0 = 0; s0 < nsplit; s0 += 16) {
            float2 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = hs[(size_t)min(s0 + u, nsplit - 1) * rows_pad];
            float Mb = M;
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (s0 + u < nsplit && v[u].y > 0.f) Mb = fmaxf(Mb, v[u].x);
            if (Mb == -INFINITY) continue;                  // nothing seen in these ranges either
            Z *= __builtin_amdgcn_exp2f(M - Mb);            // exp2(-inf) = 0 while Z is still 0
            M = Mb;
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (s0 + u < nsplit && v[u].y > 0.f) Z = __builtin_fmaf(v[u].y, __builtin_amdgcn_exp2f(v[u].x - M), Z);
        }
        out = M + __log2f(Z);
    }
    cst[(size_t)head * rows_pad + r] = out;
}

// Workgroups [0, alloc_blocks) allocate one pool each (alloc_blocks = 0: none), the others merge kThreads rows each.
__global__ __launch_bounds__(kThreads) void merge_allocate_kernel(
    const float* __restrict__ stats, int nsplit, int rows_pad, int R, float* __restrict__ cst, int alloc_blocks,
    const float* __restrict__ weights, int n_segments, int n, int weight_group, int window,
    const int32_t* __restrict__ cu_seq, double ratio, double beta,
    int32_t* __restrict__ budgets, int32_t* __restrict__ cu_budgets)
{
    extern __shared__ unsigned char smem_raw[];
    if ((int)blockIdx.x < alloc_blocks) {          // uniform over the workgroup
        allocate_pool(smem_raw, blockIdx.x, weights, n_segments, n, weight_group, window, cu_seq, ratio, beta, budgets, cu_budgets);
        return;
    }
    const int mb = blockIdx.x - alloc_blocks;
    const int blocks_per_head = (rows_pad + kThreads - 1) / kThreads;
    const int head = mb / blocks_per_head;
    merge_row(stats, nsplit, rows_pad, R, head, (mb - head * blocks_per_head) * kThreads + threadIdx.x, cst);
}

size_t alloc_smem_bytes(int n) {
    return (size_t)n * (3 * sizeof(double) + 2 * sizeof(int)) + kThreads * sizeof(long long) + sizeof(AllocShared) + 16;
}

}  // namespace

hipError_t launch_score_merge(const Geom& g, const float* stats, int nsplit, int rows_pad, float* cst,
                              const AllocateJob* job, hipStream_t s)
{
    const int n_heads = g.n_items * g.H_kv;
    const unsigned merge_blocks = (unsigned)(n_heads * ((rows_pad + kThreads - 1) / kThreads));
    size_t smem = 0;
    int alloc_blocks = 0;
    AllocateJob j{};
    if (job) {
        j = *job;
        smem = alloc_smem_bytes(j.heads_per_segment);
        if (smem > 64 * 1024) return hipErrorInvalidValue;
        alloc_blocks = j.n_segments;
    }
    hipLaunchKernelGGL(merge_allocate_kernel, dim3(merge_blocks + (unsigned)alloc_blocks), dim3(kThreads), smem, s, stats,
                       nsplit, rows_pad, g.G * g.W, cst, alloc_blocks, j.weights, j.n_segments, j.heads_per_segment,
                       j.weight_group, g.W, j.cu_seqlens, j.ratio, j.floor_frac, j.budgets, j.cu_budgets);
    return hipGetLastError();
}

hipError_t launch_allocate(const Geom& g, const float* weights, int n_segments, int heads_per_segment,
                           int weight_group, const int32_t* cu_seqlens, double ratio, double floor_frac,
                           int32_t* budgets, int32_t* cu_budgets, hipStream_t s)
{
    const int n = heads_per_segment;
    const size_t smem = alloc_smem_bytes(n);
    if (smem > 64 * 1024) return hipErrorInvalidValue;   // caller limits heads_per_segment
    hipLaunchKernelGGL(allocate_kernel, dim3(n_segments), dim3(kThreads), smem, s, weights, n_segments, n,
                       weight_group, g.W, cu_seqlens, ratio, floor_frac, budgets, cu_budgets);
    return hipGetLastError();
}

}  // namespace audiokv
