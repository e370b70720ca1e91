// Stage 2: head-wise budget allocation (paper Sec. 3.1 Eq. 1, Sec. 3.2 Eq. 12).
//
// One workgroup per budget pool ("segment"). All real arithmetic is float64
// with contraction off and with the order of operations of the plain
// definition (sum of weights accumulated in head order, share = (T*S)/sum),
// so the integers produced are reproducible bit for bit on any IEEE machine.
// Head-parallel steps (shares, floors, remainder ranks) are order-free.
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

// Sum of an int array over the block (order does not matter for integers).
__device__ long long block_sum_ll(long long v, long long* scratch /* [kThreads] */) {
    scratch[threadIdx.x] = v;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) scratch[threadIdx.x] += scratch[threadIdx.x + s];
        __syncthreads();
    }
    const long long r = scratch[0];
    __syncthreads();
    return r;
}

__device__ __forceinline__ int n_keep_dev(double ratio, int L) {
    return (int)floor(__dadd_rn(__dmul_rn(ratio, (double)L), 0.5));
}

__global__ __launch_bounds__(kThreads) void allocate_kernel(
    const float* __restrict__ weights, int n_segments, int n, int weight_group, int window,
    const int32_t* __restrict__ cu_seq, double ratio, double beta,
    int32_t* __restrict__ budgets, int32_t* __restrict__ cu_budgets)
{
    extern __shared__ unsigned char smem_raw[];
    // layout: S[n] x[n] frac[n] (double) | e[n] (int) | flag[n] (int) | red[kThreads] (ll) | AllocShared
    double* S = reinterpret_cast<double*>(smem_raw);
    double* x = S + n;
    double* frac = x + n;
    long long* red = reinterpret_cast<long long*>(frac + n);
    AllocShared* sh = reinterpret_cast<AllocShared*>(red + kThreads);
    int* e = reinterpret_cast<int*>(sh + 1);
    int* flag = e + n;      // bit 0: capped, bit 1: eligible in the current hand-out round

    const int seg = blockIdx.x;
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
    red[tid] = chunk;
    __syncthreads();
    // exclusive scan of the 256 chunk totals (integers: any order), total to the last segment's end marker
    const long long mine = chunk;
    for (int off = 1; off < kThreads; off <<= 1) {
        const long long add = tid >= off ? red[tid - off] : 0;
        __syncthreads();
        red[tid] += add;
        __syncthreads();
    }
    if (tid == kThreads - 1 && seg == n_segments - 1) cu_budgets[(size_t)n_segments * n] = (int32_t)(base + red[tid]);
    const long long excl = red[tid] - mine;
    __syncthreads();
    red[tid] = excl;
    __syncthreads();
    long long run = base + red[tid];
    for (int h = h0; h < h1; ++h) {
        const int b = f + e[h];
        budgets[(size_t)seg * n + h] = b;
        cu_budgets[(size_t)seg * n + h] = (int32_t)run;
        run += b;
    }
}

}  // namespace

hipError_t launch_allocate(const Geom& g, const float* weights, int n_segments, int heads_per_segment,
                           int weight_group, const int32_t* cu_seqlens, double ratio, double floor_frac,
                           int32_t* budgets, int32_t* cu_budgets, hipStream_t s)
{
    const int n = heads_per_segment;
    const size_t smem = (size_t)n * (3 * sizeof(double) + 2 * sizeof(int)) + kThreads * sizeof(long long) +
                        sizeof(AllocShared) + 16;
    if (smem > 64 * 1024) return hipErrorInvalidValue;   // caller limits heads_per_segment
    hipLaunchKernelGGL(allocate_kernel, dim3(n_segments), dim3(kThreads), smem, s, weights, n_segments, n,
                       weight_group, g.W, cu_seqlens, ratio, floor_frac, budgets, cu_budgets);
    return hipGetLastError();
}

}  // namespace audiokv
