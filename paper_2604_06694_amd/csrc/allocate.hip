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
        if (tid < 64) {
            // In-order float64 sum of the free heads' weights. The order is fixed (head 0, 1, 2, ...), so the adds
            // are serial, but the operands are staged 64 at a time in the lanes of one wave and read back with
            // readlane, instead of one LDS round trip per head from a single thread.
            int ncap = 0, nfree = 0;
            double tot = 0.0;
            for (int base = 0; base < n; base += 64) {
                const int h = base + tid;
                const double sv = h < n ? S[h] : 0.0;
                const int fv = h < n ? flag[h] : 0;
                const int cnt = min(64, n - base);
                for (int j = 0; j < cnt; ++j) {
                    const int lo = __builtin_amdgcn_readlane(__double2loint(sv), j);
                    const int hi = __builtin_amdgcn_readlane(__double2hiint(sv), j);
                    const int fj = __builtin_amdgcn_readlane(fv, j);
                    if (fj & 1) ++ncap;
                    else { tot = __dadd_rn(tot, __hiloint2double(hi, lo)); ++nfree; }
                }
            }
            if (tid == 0) {
                sh->tot = tot;
                sh->n_free = nfree;
                sh->T = (double)(Bs - (long long)ncap * cap);
            }
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
        for (int h = tid; h < n; h += kThreads) {
            const bool el = !(flag[h] & 1) && (give ? e[h] < cap : e[h] > 0);
            flag[h] = (flag[h] & 1) | (el ? 2 : 0);
        }
        if (tid == 0) sh->granted = 0;
        __syncthreads();
        int my_granted = 0;
        for (int h = tid; h < n; h += kThreads) {
            if (!(flag[h] & 2)) continue;
            const double fh = frac[h];
            long long rank = 0;
            for (int o = 0; o < n; ++o) {
                if (!(flag[o] & 2)) continue;
                const double fo = frac[o];
                const bool ahead = give ? (fo > fh || (fo == fh && o < h))
                                        : (fo < fh || (fo == fh && o > h));
                rank += ahead ? 1 : 0;
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
