// Stage 1 tail (local pooling) and stage 3 (Spectral Score Smoothing, paper
// Sec. 3.3 Eqs. 13, 17-20).
//
// SSS for a power-of-two L runs entirely inside one workgroup's LDS: the real
// sequence is viewed as L/2 complex numbers, transformed by an in-place
// decimation-in-frequency FFT (natural order in, bit-reversed out),
// turned into the real spectrum pair by pair, masked above k*, turned back,
// and inverted by a decimation-in-time FFT (bit-reversed in, natural out), so
// no reordering pass is needed. Four radix-2 stages at a time run in registers
// (16 points per thread), so the data crosses LDS, and the workgroup meets at
// a barrier, once per four stages. Twiddles come from two small tables filled
// from float64 sincospi: w^e = hi[e >> 7] * lo[e & 127]; the part of a twiddle
// that depends on the position inside the 16-point group is a constant 16th
// root of unity.
//
// Any other length (the transform length must be exactly L: zero-padding would be a different circular
// filter) goes through Bluestein's chirp-z identity: a length-L DFT is a convolution with a chirp, done with
// power-of-two FFTs in a per-head global-memory workspace. Only the K = k* + T + 1 lowest bins are ever needed
// (everything above is masked), so the convolutions have L + K - 1 significant points and the transform size is
// M >= L + K - 1 rather than 2L - 1: half the size for most lengths at the usual cutoffs. Stages whose span
// exceeds the LDS (M > 16384) run on global memory, the rest on 16384-point chunks inside LDS.
#include <atomic>
#include <type_traits>
#include <algorithm>
#include "common.h"

namespace audiokv {

namespace {

// ----------------------------- pooling --------------------------------------

// Pooled value at position j of one head's sequence x[0..L) (global or LDS).
__device__ __forceinline__ float pooled_at(const float* x, int L, int j, int kernel, int mode) {
    const int half = kernel >> 1;
    if (mode == AUDIOKV_POOL_AVG) {
        float acc = 0.f;
        for (int t = -half; t <= half; ++t) {
            const int p = j + t;
            acc += (p >= 0 && p < L) ? x[p] : 0.f;       // zero padding
        }
        return acc * (1.0f / (float)kernel);              // divisor is always the kernel size (one rounded reciprocal)
    }
    float acc = -INFINITY;
    for (int t = -half; t <= half; ++t) {
        const int p = j + t;
        if (p >= 0 && p < L) acc = fmaxf(acc, x[p]);
    }
    return acc;
}

// Pooled values at positions j0 and j0 + 1 of a sequence held in LDS, kernel size K known at compile time. Same
// taps, padding, order of operations and reciprocal as pooled_at, so both give the same bits.
template <int K>
__device__ __forceinline__ void pooled_pair_lds(const float* x, int L, int j0, int mode, float& o0, float& o1) {
    const float fill = mode == AUDIOKV_POOL_AVG ? 0.f : -INFINITY;
    float w[K + 1];
    if (j0 - K / 2 >= 0 && j0 + 1 + K / 2 < L) {     // every tap inside the sequence: all but the edge threads
#pragma unroll
        for (int u = 0; u <= K; ++u) w[u] = x[j0 - K / 2 + u];
    } else {
#pragma unroll
        for (int u = 0; u <= K; ++u) {
            const int p = j0 - K / 2 + u;
            const float v = x[min(max(p, 0), L - 1)];
            w[u] = (p >= 0 && p < L) ? v : fill;
        }
    }
    if (mode == AUDIOKV_POOL_AVG) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int u = 0; u < K; ++u) { a0 += w[u]; a1 += w[u + 1]; }
        o0 = a0 * (1.0f / (float)K);
        o1 = a1 * (1.0f / (float)K);
    } else {
        float a0 = -INFINITY, a1 = -INFINITY;
#pragma unroll
        for (int u = 0; u < K; ++u) { a0 = fmaxf(a0, w[u]); a1 = fmaxf(a1, w[u + 1]); }
        o0 = a0;
        o1 = a1;
    }
}

// Pooled values at positions j0 and j0 + 1 of x[0..L) (global memory or LDS): the common kernel sizes take all their
// taps at once (independent loads), any other size goes tap by tap. Same bits either way.
__device__ __forceinline__ void pooled_pair(const float* x, int L, int j0, int kernel, int mode, float& o0, float& o1) {
    switch (kernel) {
        case 3:  pooled_pair_lds<3>(x, L, j0, mode, o0, o1); break;
        case 5:  pooled_pair_lds<5>(x, L, j0, mode, o0, o1); break;
        case 7:  pooled_pair_lds<7>(x, L, j0, mode, o0, o1); break;
        case 9:  pooled_pair_lds<9>(x, L, j0, mode, o0, o1); break;
        default:
            o0 = pooled_at(x, L, j0, kernel, mode);
            o1 = pooled_at(x, L, j0 + 1, kernel, mode);
    }
}

__global__ __launch_bounds__(256) void pool_kernel(Geom g, const float* __restrict__ raw,
                                                   const int32_t* __restrict__ cu_seq,
                                                   float* __restrict__ pooled)
{
    const int head = blockIdx.y;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const size_t off = (size_t)tok0 * g.H_kv + (size_t)h * L;
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < L; j += gridDim.x * blockDim.x)
        pooled[off + j] = pooled_at(raw + off, L, j, g.pool_kernel, g.pool_mode);
}

// ------------------------ LDS-resident real FFT ------------------------------

constexpr int kFftThreads = 1024;
constexpr int kMaxPow2L = 32768;          // 128 KiB of fp32 in LDS
constexpr int kTwLo = 128;

__host__ __device__ inline bool pow2_length(int L) { return L >= 4 && L <= kMaxPow2L && (L & (L - 1)) == 0; }

struct cf { float re, im; };
__device__ __forceinline__ cf cmul(cf a, cf b) { return {a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re}; }
__device__ __forceinline__ cf cadd(cf a, cf b) { return {a.re + b.re, a.im + b.im}; }
__device__ __forceinline__ cf csub(cf a, cf b) { return {a.re - b.re, a.im - b.im}; }
__device__ __forceinline__ cf cconj(cf a) { return {a.re, -a.im}; }

// exp(-2*pi*i*e/L) for 0 <= e <= L/2
__device__ __forceinline__ cf twiddle(const cf* lo, const cf* hi, int e) {
    return cmul(hi[e >> 7], lo[e & (kTwLo - 1)]);
}

// LDS slot of complex element i. One spare slot per 16 elements: a thread's 16-point group at stride 1 or 4 would
// otherwise sit in a single bank.
__device__ __forceinline__ int pad(int i) { return i + (i >> 4); }
__host__ __device__ constexpr size_t padded_len(size_t n) { return n + (n >> 4) + 1; }

// w * exp(-2*pi*i*k/16) for k = 0..7; k is a compile-time constant once the callers' loops are unrolled
__device__ __forceinline__ cf mul_root16(cf w, int k) {
    constexpr float C1 = 0.92387953251128674f, S1 = 0.38268343236508977f, H = 0.70710678118654752f;
    switch (k) {
        case 0:  return w;
        case 1:  return cmul(w, {C1, -S1});
        case 2:  return cmul(w, {H, -H});
        case 3:  return cmul(w, {S1, -C1});
        case 4:  return {w.im, -w.re};
        case 5:  return cmul(w, {-S1, -C1});
        case 6:  return cmul(w, {-H, -H});
        default: return cmul(w, {-C1, -S1});
    }
}

// R decimation-in-frequency stages (half-sizes 2^s down to 2^(s-R+1)) of an in-place FFT on n complex points in
// LDS. The twiddle of stage s' at offset j inside its half is root^(j << (tw_shift - s')), root = exp(-2*pi*i/2^(tw_shift+1)).
// A thread owns the 2^R points that differ in index bits [s-R+1, s]. Ends with a barrier.
template <int R>
__device__ __forceinline__ void dif_pass(cf* z, int n, int s, int tw_shift, const cf* lo, const cf* hi) {
    const int sb = s - R + 1;
    for (int gi = threadIdx.x; gi < (n >> R); gi += blockDim.x) {
        const int j0 = gi & ((1 << sb) - 1);
        const int base = ((gi >> sb) << (sb + R)) | j0;
        cf v[1 << R];
#pragma unroll
        for (int q = 0; q < (1 << R); ++q) v[q] = z[pad(base + (q << sb))];
        const int e0 = j0 << (tw_shift - s);
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int bit = R - 1 - t;
            const cf wt = twiddle(lo, hi, e0 << t);      // the part of the exponent that comes from j0
#pragma unroll
            for (int q = 0; q < (1 << R); ++q) {
                if (q & (1 << bit)) continue;
                const int qlow = q & ((1 << bit) - 1);   // the part that comes from the position in the group
                const cf tw = mul_root16(wt, (qlow << t) << (4 - R));
                const cf a = v[q], c = v[q | (1 << bit)];
                v[q] = cadd(a, c);
                v[q | (1 << bit)] = cmul(csub(a, c), tw);
            }
        }
#pragma unroll
        for (int q = 0; q < (1 << R); ++q) z[pad(base + (q << sb))] = v[q];
    }
    __syncthreads();
}

// R decimation-in-time stages (half-sizes 2^s0 up to 2^(s0+R-1)) with conjugate twiddles: the mirror image.
template <int R>
__device__ __forceinline__ void dit_pass(cf* z, int n, int s0, int tw_shift, const cf* lo, const cf* hi) {
    for (int gi = threadIdx.x; gi < (n >> R); gi += blockDim.x) {
        const int j0 = gi & ((1 << s0) - 1);
        const int base = ((gi >> s0) << (s0 + R)) | j0;
        cf v[1 << R];
#pragma unroll
        for (int q = 0; q < (1 << R); ++q) v[q] = z[pad(base + (q << s0))];
        const int e0 = j0 << (tw_shift - s0 - R + 1);
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const cf wt = twiddle(lo, hi, e0 << (R - 1 - t));
#pragma unroll
            for (int q = 0; q < (1 << R); ++q) {
                if (q & (1 << t)) continue;
                const int qlow = q & ((1 << t) - 1);
                const cf tw = cconj(mul_root16(wt, qlow << (3 - t)));
                const cf a = v[q], c = cmul(v[q | (1 << t)], tw);
                v[q] = cadd(a, c);
                v[q | (1 << t)] = csub(a, c);
            }
        }
#pragma unroll
        for (int q = 0; q < (1 << R); ++q) z[pad(base + (q << s0))] = v[q];
    }
    __syncthreads();
}

// all log2(n) stages on LDS-resident data: forward = natural order in, bit-reversed out; inverse = the reverse,
// unnormalised
__device__ __forceinline__ void fft_lds(cf* z, int logn, int tw_shift, bool inverse, const cf* lo, const cf* hi) {
    const int n = 1 << logn;
    if (!inverse) {
        for (int s = logn - 1; s >= 0;) {
            const int R = s + 1 < 4 ? s + 1 : 4;
            if (R == 4) dif_pass<4>(z, n, s, tw_shift, lo, hi);
            else if (R == 3) dif_pass<3>(z, n, s, tw_shift, lo, hi);
            else if (R == 2) dif_pass<2>(z, n, s, tw_shift, lo, hi);
            else dif_pass<1>(z, n, s, tw_shift, lo, hi);
            s -= R;
        }
    } else {
        for (int s0 = 0; s0 < logn;) {
            const int R = logn - s0 < 4 ? logn - s0 : 4;
            if (R == 4) dit_pass<4>(z, n, s0, tw_shift, lo, hi);
            else if (R == 3) dit_pass<3>(z, n, s0, tw_shift, lo, hi);
            else if (R == 2) dit_pass<2>(z, n, s0, tw_shift, lo, hi);
            else dit_pass<1>(z, n, s0, tw_shift, lo, hi);
            s0 += R;
        }
    }
}

// Frequency mask (Eqs. 17-18): 1 up to k*, a half-cosine roll-off over the next T bins, 0 beyond.
__device__ __forceinline__ float mask_weight(int k, int kstar, int T) {
    if (k <= kstar) return 1.f;
    if (k > kstar + T) return 0.f;
    return 0.5f * (1.f + cospif((float)(k - kstar) / (float)(T + 1)));
}

// Masks for which the filter needs no transform at all, and for which a transform would only add rounding noise to
// what is exactly a plateau or exactly the input (the selection that follows breaks ties by index, so the noise
// would decide instead): 2 = every bin is kept with weight 1 (Eq. 19 returns s itself), 1 = only the DC bin
// survives (Eq. 19 returns the mean of s at every position), 0 = anything else.
__host__ __device__ inline int degenerate_mask(int L, int kstar, int T) {
    if (kstar >= (L >> 1)) return 2;
    if (kstar + T == 0) return 1;
    return 0;
}

// The result for a degenerate mask, by all kFftThreads threads of the workgroup; `part` holds kFftThreads doubles.
// The mean is one value (float64 sum in a fixed order, rounded once), written to every position. In place is fine:
// all reads of the mean case come before a barrier, and the copy case reads position n only to write position n.
__device__ __forceinline__ void write_degenerate(int kind, const Geom& g, const float* src, float* dst, int L,
                                                 int pool_on_load, float alpha, double* part) {
    const int tid = threadIdx.x;
    auto s_at = [&](int n) { return pool_on_load ? pooled_at(src, L, n, g.pool_kernel, g.pool_mode) : src[n]; };
    if (kind == 2) {
        for (int n = tid; n < L; n += kFftThreads) dst[n] = s_at(n);
        return;
    }
    double mine = 0.0;
    for (int n = tid; n < L; n += kFftThreads) mine += (double)s_at(n);
    part[tid] = mine;
    __syncthreads();
    for (int off = kFftThreads >> 1; off > 0; off >>= 1) {
        if (tid < off) part[tid] += part[tid + off];
        __syncthreads();
    }
    const float mean = (float)(part[0] / (double)L);
    if (alpha == 1.f && !pool_on_load) {
        for (int n = tid; n < L; n += kFftThreads) dst[n] = mean;
    } else {
        // with pooling on load src and dst are different arrays; without it s_at(n) is src[n], read before written
        for (int n = tid; n < L; n += kFftThreads) {
            const float s0 = s_at(n);
            dst[n] = alpha == 1.f ? mean : (1.f - alpha) * s0 + alpha * mean;
        }
    }
}

// LDS scratch of the energy search: kFftThreads partial sums and the result
struct EnergyScratch {
    double part[kFftThreads];
    int cross;
    int kstar;
};

// Adaptive cutoff (Eqs. 14-16): the smallest k >= first with sum_{first<=i<=k} e(i) >= rho * sum_{first<=i<n_bins} e(i).
// Bin energies are fp32, all sums float64: every thread adds a contiguous run of bins, the runs' totals are
// scanned, and the thread whose run crosses the target walks it again. Uniform result; ends synchronised.
template <class EnergyFn>
__device__ __forceinline__ int energy_cutoff(EnergyFn&& energy, int n_bins, int first, double rho, EnergyScratch* sc) {
    const int tid = threadIdx.x;
    const int per = (n_bins + kFftThreads - 1) / kFftThreads;
    const int k0 = max(min(tid * per, n_bins), first), k1 = max(min(tid * per + per, n_bins), k0);
    double mine = 0.0;
    for (int k = k0; k < k1; ++k) mine += (double)energy(k);
    sc->part[tid] = mine;
    if (tid == 0) { sc->cross = kFftThreads; sc->kstar = min(first, n_bins - 1); }
    __syncthreads();
    for (int off = 1; off < kFftThreads; off <<= 1) {          // inclusive scan
        const double add = tid >= off ? sc->part[tid - off] : 0.0;
        __syncthreads();
        sc->part[tid] += add;
        __syncthreads();
    }
    const double target = rho * sc->part[kFftThreads - 1];
    const double incl = sc->part[tid];
    if (target > 0.0 && k1 > k0 && incl >= target) atomicMin(&sc->cross, tid);
    __syncthreads();
    if (tid == sc->cross) {
        double acc = incl - mine;
        int ks = k1 - 1;                                       // rounding between the two summation orders
        for (int k = k0; k < k1; ++k) {
            acc += (double)energy(k);
            if (acc >= target) { ks = k; break; }
        }
        sc->kstar = ks;
    }
    __syncthreads();
    return sc->kstar;
}

__device__ __forceinline__ bool dec_owns(const Geom& g, int L, double cutoff_frac);   // heads of the several-workgroups path

__global__ __launch_bounds__(kFftThreads) void smooth_pow2_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq,
    double cutoff_frac, float alpha,
    float* __restrict__ out, int32_t* __restrict__ kstar_out, int cutoffs_only, int skip_dec)
{
    extern __shared__ float smem[];
    const int head = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const size_t off = (size_t)tok0 * g.H_kv + (size_t)h * L;
    const float* src = in + off;
    float* dst = out + off;
    const int tid = threadIdx.x;

    if (alpha == 0.f) {
        // alpha = 0: the mix returns s itself, whatever the length
        for (int j = tid; j < L; j += kFftThreads)
            dst[j] = pool_on_load ? pooled_at(src, L, j, g.pool_kernel, g.pool_mode) : src[j];
        return;
    }
    if (!pow2_length(L)) return;                      // the chirp-z kernel owns this head
    if (skip_dec && dec_owns(g, L, cutoff_frac)) return;   // spread over several workgroups by the dec_* kernels
    const int T = g.taper_bins;
    if (g.cutoff_mode == AUDIOKV_CUTOFF_FRACTION && cutoffs_only) {
        if (tid == 0) kstar_out[head] = (int)floor(cutoff_frac * (double)(L >> 1));
        return;
    }

    if (g.cutoff_mode == AUDIOKV_CUTOFF_FRACTION &&
        degenerate_mask(L, (int)floor(cutoff_frac * (double)(L >> 1)), T) == 2) {
        // every bin kept: the filter is the identity (the DC-only mask needs nothing special here: with a single
        // non-zero bin the inverse butterflies only add exact zeros, and every output is the same value)
        write_degenerate(2, g, src, dst, L, pool_on_load, alpha, reinterpret_cast<double*>(smem));
        return;
    }

    const int N = L >> 1;                         // complex length
    const int logN = 31 - __clz(N);
    cf* z = reinterpret_cast<cf*>(smem);          // N complex = L floats, padded
    cf* lo = z + padded_len(N);                   // kTwLo entries: w^j
    cf* hi = lo + kTwLo;                          // (L/2)/128 + 1 entries: w^(128 j)
    const int n_hi = (N >> 7) + 1;

    if (pool_on_load) {
        // one coalesced read of the raw scores into LDS, pooling from there (every tap from global memory would
        // cost kernel-size times the loads), pooled values parked in registers while the buffer changes layout
        float* rawf = smem;
        for (int j = tid; j < L; j += 8 * kFftThreads) {         // eight loads in flight per thread
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = src[min(j + u * kFftThreads, L - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (j + u * kFftThreads < L) rawf[j + u * kFftThreads] = t[u];
        }
        __syncthreads();
        constexpr int kPer = (kMaxPow2L / 2) / kFftThreads;      // complex points per thread at the longest L
        cf keep[kPer];
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            const int i = tid + e * kFftThreads;
            if (i < N) {
                pooled_pair(rawf, L, 2 * i, g.pool_kernel, g.pool_mode, keep[e].re, keep[e].im);
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            const int i = tid + e * kFftThreads;
            if (i < N) z[pad(i)] = keep[e];
        }
    } else {
        for (int i = tid; i < N; i += kFftThreads) z[pad(i)] = {src[2 * i], src[2 * i + 1]};
    }
    for (int t = tid; t < kTwLo + n_hi; t += kFftThreads) {
        const long long e = t < kTwLo ? t : (long long)(t - kTwLo) * kTwLo;
        double sn, cs;
        sincospi(2.0 * (double)e / (double)L, &sn, &cs);
        const cf w = {(float)cs, (float)(-sn)};
        if (t < kTwLo) lo[t] = w; else hi[t - kTwLo] = w;
    }
    __syncthreads();

    // forward transform of the half-length complex sequence; stage twiddles w_N^(j N/(2m)) = w_L^(j << (logN - s))
    fft_lds(z, logN, logN, false, lo, hi);

    const int shift = 32 - logN;
    // bin k of the real spectrum from the half-length transform: X_k = E_k + w^k O_k with E, O the transforms of
    // the even and odd samples, both read off Z[k] and conj(Z[N-k]) (stored bit-reversed)
    int kstar = (int)floor(cutoff_frac * (double)N);            // N = floor(L/2) = n_bins - 1
    if (g.cutoff_mode != AUDIOKV_CUTOFF_FRACTION) {
        auto bin_energy = [&](int k) -> float {
            if (k == 0 || k == N) {
                const cf z0 = z[0];
                const float x = k == 0 ? z0.re + z0.im : z0.re - z0.im;
                return x * x;
            }
            const cf A = z[pad((int)(__brev((unsigned)k) >> shift))];
            const cf B = cconj(z[pad((int)(__brev((unsigned)(N - k)) >> shift))]);
            const cf E = {0.5f * (A.re + B.re), 0.5f * (A.im + B.im)};
            const cf Dm = csub(A, B);
            const cf O = {0.5f * Dm.im, -0.5f * Dm.re};
            const cf X = cadd(E, cmul(twiddle(lo, hi, k), O));
            return X.re * X.re + X.im * X.im;
        };
        EnergyScratch* sc = reinterpret_cast<EnergyScratch*>(hi + n_hi + 1);
        kstar = energy_cutoff(bin_energy, N + 1, g.cutoff_mode == AUDIOKV_CUTOFF_ENERGY_NO_DC ? 1 : 0, cutoff_frac, sc);
    }
    if (kstar_out && tid == 0) kstar_out[head] = kstar;
    if (cutoffs_only) return;
    if (g.cutoff_mode != AUDIOKV_CUTOFF_FRACTION && degenerate_mask(L, kstar, T) == 2) {
        __syncthreads();                                        // everyone is done with the spectrum in LDS
        write_degenerate(2, g, src, dst, L, pool_on_load, alpha, reinterpret_cast<double*>(smem));
        return;
    }

    // low-pass mask (Eq. 17-18) and back to the half-length form, pair (k, N-k) at a time. The transform sits in
    // bit-reversed order, so the loop runs over storage slots, not bins: slot p holds bin brev(p), consecutive
    // lanes touch consecutive slots (bins in natural order would put a whole wave on one LDS bank), and the
    // partner slot brev(N - k) runs backwards through consecutive slots as well. Bins 1..N/2-1 are exactly the
    // even slots (their top bit is clear); slot 0 is bin 0 (with the Nyquist bin folded into it), slot 1 is bin N/2.
    const int ktop = kstar + T;                                 // last bin with a non-zero weight
    for (int q = tid; q < (N >> 1) + 1; q += kFftThreads) {
        if (q == 0) {
            const cf z0 = z[0];
            const float X0 = z0.re + z0.im;                     // DC bin, always kept (0 <= k*)
            const float XN = (z0.re - z0.im) * mask_weight(N, kstar, T);   // Nyquist bin
            z[0] = {0.5f * (X0 + XN), 0.5f * (X0 - XN)};
            continue;
        }
        const int slot = q == (N >> 1) ? 1 : 2 * q;             // the extra trip takes the self-paired bin N/2
        const int k = (int)(__brev((unsigned)slot) >> shift);
        const int pa = pad(slot);
        const int pb = pad((int)(__brev((unsigned)(N - k)) >> shift));
        if (k > ktop && N - k > ktop) {                         // both bins masked
            z[pa] = {0.f, 0.f};
            z[pb] = {0.f, 0.f};
            continue;
        }
        const cf A = z[pa];
        const cf B = cconj(z[pb]);
        const cf E = {0.5f * (A.re + B.re), 0.5f * (A.im + B.im)};
        const cf Dm = csub(A, B);
        const cf O = {0.5f * Dm.im, -0.5f * Dm.re};             // -i (A - B) / 2
        const cf Wk = twiddle(lo, hi, k);
        const cf WO = cmul(Wk, O);
        cf Xk = cadd(E, WO);                                    // bin k
        cf Xn = cconj(csub(E, WO));                             // bin N - k
        const float wk = mask_weight(k, kstar, T), wn = mask_weight(N - k, kstar, T);
        Xk = {Xk.re * wk, Xk.im * wk};
        Xn = {Xn.re * wn, Xn.im * wn};
        const cf Xnc = cconj(Xn);
        const cf E2 = {0.5f * (Xk.re + Xnc.re), 0.5f * (Xk.im + Xnc.im)};
        const cf H2 = {0.5f * (Xk.re - Xnc.re), 0.5f * (Xk.im - Xnc.im)};
        const cf O2 = cmul(H2, cconj(Wk));
        // Z'[k] = E' + i O' ; Z'[N-k] = conj(E') + i conj(O')
        z[pa] = {E2.re - O2.im, E2.im + O2.re};
        if (pb != pa) z[pb] = {E2.re + O2.im, -E2.im + O2.re};
    }
    __syncthreads();

    fft_lds(z, logN, logN, true, lo, hi);

    // residual mix (Eq. 20); 1/N completes the inverse transform
    const float inv = 1.0f / (float)N;
    for (int i = tid; i < N; i += kFftThreads) {
        const cf st = z[pad(i)];
        float o0 = st.re * inv, o1 = st.im * inv;
        if (alpha != 1.f) {
            const float a0 = pool_on_load ? pooled_at(src, L, 2 * i, g.pool_kernel, g.pool_mode) : src[2 * i];
            const float a1 = pool_on_load ? pooled_at(src, L, 2 * i + 1, g.pool_kernel, g.pool_mode) : src[2 * i + 1];
            o0 = (1.f - alpha) * a0 + alpha * o0;
            o1 = (1.f - alpha) * a1 + alpha * o1;
        }
        dst[2 * i] = o0;
        dst[2 * i + 1] = o1;
    }
}

// twiddle tables for the root exp(-2*pi*i/M): lo[t] = root^t (t < 128), hi[t] = root^(128 t), from float64 angles
__device__ __forceinline__ void fill_tables(cf* lo, cf* hi, int n_hi, int M) {
    for (int t = threadIdx.x; t < kTwLo + n_hi; t += blockDim.x) {
        const long long e = t < kTwLo ? t : (long long)(t - kTwLo) * kTwLo;
        double sn, cs;
        sincospi(2.0 * (double)e / (double)M, &sn, &cs);
        const cf w = {(float)cs, (float)(-sn)};
        if (t < kTwLo) lo[t] = w; else hi[t - kTwLo] = w;
    }
}

// ------------------------ power-of-two lengths, few heads: one head on several workgroups ------------------------
// A call with few heads (one layer of a prefill: four) leaves all but a handful of CUs idle while each head's
// transform runs in one workgroup. For those calls a head of L = 2^p >= 16384 samples is cut into D = 16 interleaved
// sub-sequences x_{16 m + r} of M = L / 16 samples, the first stage of a decimation-in-time FFT taken out of the
// workgroup:
//   dec_forward   per pair (r, r + 1): one complex M-point FFT in LDS gives the spectra G_r, G_{r+1} of the two
//                 real sub-sequences (bins 0..M/2)                                          8 workgroups per head
//   dec_combine   per bin j of the sub-spectra: F_{j + t M} = DFT16_r(w_L^{j r} G_r[j]) are the 16 bins of the
//                 full spectrum in j's residue class; mask them (Eqs. 17-18); H_{r'}[j] =
//                 w_L^{-j r'} IDFT16_t(F~_{j + t M})[r'] are the sub-spectra of the filtered sequence
//   dec_inverse   per pair: one complex M-point inverse FFT returns s~_{16 m + r}, s~_{16 m + r + 1}; residual mix
// Same arithmetic as the single-workgroup kernel up to the order of the butterflies (fp32, twiddles from float64 or
// from exactly representable angles). Fixed-fraction cutoff only: an energy-adaptive cutoff needs the whole spectrum
// in one place first.
constexpr int kDecLog = 4, kDec = 1 << kDecLog;      // D
constexpr int kDecThreads = 1024;    // the strided (and, inside evict, pooled) loads want many waves in flight
constexpr int kDecMinL = 16384;   // below this one workgroup per head is as fast (measured: 8192 19 us alone, 21 us spread; 16384 33 and 21)
constexpr int kDecMaxHeads = 64;                     // beyond this the heads fill the chip by themselves

__host__ __device__ inline bool dec_length(int L) { return pow2_length(L) && L >= kDecMinL; }
// complex values per head in the workspace: G and H, 16 sub-spectra of M/2 + 1 bins each
__host__ __device__ inline size_t dec_head_elems(int L) { return 2 * (size_t)kDec * ((L >> (kDecLog + 1)) + 1); }

struct DecWs {
    cf* base;
    size_t per_head;        // of the longest head of the batch
    __device__ cf* g_of(int head, int r, int M) const { return base + (size_t)head * per_head + (size_t)r * ((M >> 1) + 1); }
    __device__ cf* h_of(int head, int r, int M) const { return base + (size_t)head * per_head + (size_t)(kDec + r) * ((M >> 1) + 1); }
};

// which heads this path owns: identical test in all three kernels and in the single-workgroup kernel's skip
__device__ __forceinline__ bool dec_owns(const Geom& g, int L, double cutoff_frac) {
    return dec_length(L) && degenerate_mask(L, (int)floor(cutoff_frac * (double)(L >> 1)), g.taper_bins) != 2;
}

__global__ __launch_bounds__(kDecThreads) void dec_forward_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq, double cutoff_frac, DecWs ws)
{
    extern __shared__ float smem[];
    const int head = blockIdx.y, pr = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    if (!dec_owns(g, L, cutoff_frac)) return;
    const int M = L >> kDecLog, logM = 31 - __clz(M);
    const float* src = in + (size_t)tok0 * g.H_kv + (size_t)h * L;
    cf* z = reinterpret_cast<cf*>(smem);
    cf* lo = z + padded_len(M);
    cf* hi = lo + kTwLo;
    const int tid = threadIdx.x;
    fill_tables(lo, hi, (M >> 8) + 1, M);
    const int r0 = 2 * pr;
    for (int m = tid; m < M; m += kDecThreads) {
        const int n = (m << kDecLog) + r0;
        cf v;
        if (pool_on_load) pooled_pair(src, L, n, g.pool_kernel, g.pool_mode, v.re, v.im);
        else { const float2 t = *reinterpret_cast<const float2*>(src + n); v.re = t.x; v.im = t.y; }
        z[pad(m)] = v;
    }
    __syncthreads();
    fft_lds(z, logM, logM - 1, false, lo, hi);        // bin k sits in slot brev(k)
    const int shift = 32 - logM;
    cf* G0 = ws.g_of(head, r0, M);
    cf* G1 = ws.g_of(head, r0 + 1, M);
    for (int j = tid; j <= (M >> 1); j += kDecThreads) {
        const cf A = z[pad((int)(__brev((unsigned)j) >> shift))];
        const cf B = cconj(z[pad((int)(__brev((unsigned)((M - j) & (M - 1))) >> shift))]);
        G0[j] = {0.5f * (A.re + B.re), 0.5f * (A.im + B.im)};       // transform of the real parts
        G1[j] = {0.5f * (A.im - B.im), -0.5f * (A.re - B.re)};      // -i (A - B) / 2: of the imaginary parts
    }
}

// in-register 16-point DFT (forward: exp(-2 pi i / 16)); v[t] in, X[t] out
__device__ __forceinline__ void dft16(cf (&v)[16]) {
#pragma unroll
    for (int half = 8; half >= 1; half >>= 1) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            if (q & half) continue;
            const cf a = v[q], c = v[q | half];
            v[q] = cadd(a, c);
            v[q | half] = mul_root16(csub(a, c), (q & (half - 1)) * (8 / half));
        }
    }
    // results are in bit-reversed order: swap in place
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int rq = ((q & 1) << 3) | ((q & 2) << 1) | ((q & 4) >> 1) | ((q & 8) >> 3);
        if (rq > q) { const cf t = v[q]; v[q] = v[rq]; v[rq] = t; }
    }
}

constexpr int kDecCombineThreads = 64;   // one bin per thread, many small workgroups

__global__ __launch_bounds__(kDecCombineThreads) void dec_combine_kernel(
    Geom g, const int32_t* __restrict__ cu_seq, double cutoff_frac, DecWs ws)
{
    const int head = blockIdx.y;
    const int item = head / g.H_kv;
    const int L = cu_seq[item + 1] - cu_seq[item];
    if (!dec_owns(g, L, cutoff_frac)) return;
    const int M = L >> kDecLog;
    const int j = blockIdx.x * kDecCombineThreads + threadIdx.x;
    if (j > (M >> 1)) return;
    const int kstar = (int)floor(cutoff_frac * (double)(L >> 1));
    const int T = g.taper_bins;
    // twiddles w_L^{j r}: the angle 2 j r / L is exact in fp32 (j r < 2^15)
    cf tw[kDec];
#pragma unroll
    for (int r = 0; r < kDec; ++r) {
        float sn, cs;
        sincospif(2.0f * (float)(j * r) / (float)L, &sn, &cs);
        tw[r] = {cs, -sn};
    }
    cf v[kDec];
#pragma unroll
    for (int r = 0; r < kDec; ++r) v[r] = cmul(tw[r], ws.g_of(head, r, M)[j]);
    dft16(v);                                          // v[t] = F_{j + t M}
#pragma unroll
    for (int t = 0; t < kDec; ++t) {
        const int k = j + t * M;
        const float wgt = mask_weight(k <= (L >> 1) ? k : L - k, kstar, T);
        // conjugated for the inverse transform below: IDFT(x) = conj(DFT(conj(x)))
        v[t] = {v[t].re * wgt, -v[t].im * wgt};
    }
    dft16(v);
#pragma unroll
    for (int r = 0; r < kDec; ++r) ws.h_of(head, r, M)[j] = cmul(cconj(tw[r]), cconj(v[r]));
}

__global__ __launch_bounds__(kDecThreads) void dec_inverse_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq, double cutoff_frac, float alpha,
    float* __restrict__ out, DecWs ws)
{
    extern __shared__ float smem[];
    const int head = blockIdx.y, pr = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    if (!dec_owns(g, L, cutoff_frac)) return;
    const int M = L >> kDecLog, logM = 31 - __clz(M);
    const size_t off = (size_t)tok0 * g.H_kv + (size_t)h * L;
    const float* src = in + off;
    float* dst = out + off;
    cf* z = reinterpret_cast<cf*>(smem);
    cf* lo = z + padded_len(M);
    cf* hi = lo + kTwLo;
    const int tid = threadIdx.x;
    fill_tables(lo, hi, (M >> 8) + 1, M);
    const int r0 = 2 * pr, shift = 32 - logM;
    const cf* H0 = ws.h_of(head, r0, M);
    const cf* H1 = ws.h_of(head, r0 + 1, M);
    // Z[j] = H0[j] + i H1[j] over all M bins; both sub-sequences are real, so bins above M/2 are conjugates
    for (int j = tid; j < M; j += kDecThreads) {
        const bool up = j > (M >> 1);
        const int jj = up ? M - j : j;
        cf a = H0[jj], b = H1[jj];
        if (up) { a = cconj(a); b = cconj(b); }
        z[pad((int)(__brev((unsigned)j) >> shift))] = {a.re - b.im, a.im + b.re};
    }
    __syncthreads();
    fft_lds(z, logM, logM - 1, true, lo, hi);          // natural order out, unnormalised
    const float inv = 1.0f / (float)L;
    for (int m = tid; m < M; m += kDecThreads) {
        const int n = (m << kDecLog) + r0;
        const cf st = z[pad(m)];
        float o0 = st.re * inv, o1 = st.im * inv;
        if (alpha != 1.f) {
            float a0, a1;
            if (pool_on_load) pooled_pair(src, L, n, g.pool_kernel, g.pool_mode, a0, a1);
            else { a0 = src[n]; a1 = src[n + 1]; }
            o0 = (1.f - alpha) * a0 + alpha * o0;
            o1 = (1.f - alpha) * a1 + alpha * o1;
        }
        *reinterpret_cast<float2*>(dst + n) = make_float2(o0, o1);
    }
}

// ------------------------ arbitrary length: Bluestein over global memory -----------------------

constexpr int kChunkLog = 14;                     // 16384 complex = 128 KiB: the part of an FFT that fits in LDS
constexpr int kWideMinLog = 12;                   // transforms of 4096 points and more are spread over four workgroups,
constexpr int kWideMaxLog = 18;                   // in chunks of at most 16384 points: four up to 65536, then 8 or 16
constexpr int kMaxBluesteinLog = 18;              // M <= 262144: any L <= 131072 at any cutoff
__host__ __device__ inline bool wide_size(int logM) { return logM >= kWideMinLog && logM <= kWideMaxLog; }

// log2 of the transform size for L samples and K wanted bins: the smallest power of two >= L + K - 1
__host__ __device__ inline int bluestein_log(int L, int K) {
    int lg = 1;
    while ((1 << lg) < L + K - 1) ++lg;
    return lg;
}
__host__ __device__ inline int bluestein_log_max(int L) { return bluestein_log(L, (L >> 1) + 1); }

// bins 0 .. K-1 that the filter can leave non-zero (all of them when the cutoff is found from the spectrum)
__host__ __device__ inline int wanted_bins(int L, double cutoff_frac, int cutoff_mode, int taper_bins) {
    const int half = L >> 1;
    if (cutoff_mode != AUDIOKV_CUTOFF_FRACTION) return half + 1;
    const long long ktop = (long long)floor(cutoff_frac * (double)half) + taper_bins;
    return (int)(ktop < half ? ktop : half) + 1;
}

// exp(-i*pi*n^2/L): the chirp, from an exactly reduced angle in float64
__device__ __forceinline__ cf chirp(int n, int L) {
    const long long r = ((long long)n * n) % (2LL * L);
    double sn, cs;
    sincospi((double)r / (double)L, &sn, &cs);
    return {(float)cs, (float)(-sn)};
}

// exp(-2*pi*i*e/M) for 0 <= e < M/2 from the two tables of root M
__device__ __forceinline__ cf tw_m(const cf* lo, const cf* hi, int e) { return cmul(hi[e >> 7], lo[e & (kTwLo - 1)]); }

// The transforms of size M = 2^logM on global memory are decimation in frequency forwards (natural order in,
// bit-reversed out) and decimation in time backwards (bit-reversed in, natural out, conjugate twiddles,
// unnormalised). The stages whose span fits a chunk of C = min(M, 16384) points run in LDS on one chunk at a time;
// the one or two wider stages ("top" stages) run on global memory, fused into a single radix-4 pass when there are
// two. `z` is the padded LDS chunk; lo/hi are the twiddle tables of root M.

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ cf mul_neg_i(cf a) { return {a.im, -a.re}; }
__device__ __forceinline__ cf mul_pos_i(cf a) { return {-a.im, a.re}; }

// two consecutive complex values as one 16-byte access (i even: the arrays are 16-byte aligned)
__device__ __forceinline__ void ld2(const cf* x, int i, cf& a, cf& b) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(x + i);
    a = {v[0], v[1]};
    b = {v[2], v[3]};
}
__device__ __forceinline__ void st2(cf* x, int i, cf a, cf b) {
    const f32x4 v = {a.re, a.im, b.re, b.im};
    *reinterpret_cast<f32x4*>(x + i) = v;
}

__device__ __noinline__ void top_stages(cf* __restrict__ x, int logM, bool inverse, const cf* lo, const cf* hi) {
    const int tid = threadIdx.x;
    const int M = 1 << logM;
    const int extra = logM - (logM < kChunkLog ? logM : kChunkLog);
    if (extra == 1) {
        // one stage of half-size M/2: pairs (i, i + M/2), twiddle root^i
        const int m = M >> 1;
        for (int i = 2 * tid; i < m; i += 2 * kFftThreads) {
            cf a[2], c[2];
            ld2(x, i, a[0], a[1]);
            ld2(x, i + m, c[0], c[1]);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const cf w = tw_m(lo, hi, i + u);
                if (!inverse) { const cf d = csub(a[u], c[u]); a[u] = cadd(a[u], c[u]); c[u] = cmul(d, w); }
                else { const cf cw = cmul(c[u], cconj(w)); c[u] = csub(a[u], cw); a[u] = cadd(a[u], cw); }
            }
            st2(x, i, a[0], a[1]);
            st2(x, i + m, c[0], c[1]);
        }
        __syncthreads();
    } else if (extra == 2) {
        // half-sizes M/2 and M/4 in one pass over the quadruples (i, i + M/4, i + M/2, i + 3M/4)
        const int q = M >> 2;
        for (int i = 2 * tid; i < q; i += 2 * kFftThreads) {
            cf v[4][2];
#pragma unroll
            for (int r = 0; r < 4; ++r) ld2(x, i + r * q, v[r][0], v[r][1]);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const cf w1 = tw_m(lo, hi, i + u);            // stage M/2 at offset i (offset i + M/4: times -i)
                const cf w2 = tw_m(lo, hi, 2 * (i + u));      // stage M/4 at offset i
                cf a0 = v[0][u], a1 = v[1][u], a2 = v[2][u], a3 = v[3][u];
                if (!inverse) {
                    const cf b0 = cadd(a0, a2), b2 = cmul(csub(a0, a2), w1);
                    const cf b1 = cadd(a1, a3), b3 = mul_neg_i(cmul(csub(a1, a3), w1));
                    a0 = cadd(b0, b1); a1 = cmul(csub(b0, b1), w2);
                    a2 = cadd(b2, b3); a3 = cmul(csub(b2, b3), w2);
                } else {
                    const cf w1c = cconj(w1), w2c = cconj(w2);
                    const cf t1 = cmul(a1, w2c), t3 = cmul(a3, w2c);
                    const cf b0 = cadd(a0, t1), b1 = csub(a0, t1), b2 = cadd(a2, t3), b3 = csub(a2, t3);
                    const cf u2 = cmul(b2, w1c), u3 = mul_pos_i(cmul(b3, w1c));
                    a0 = cadd(b0, u2); a2 = csub(b0, u2);
                    a1 = cadd(b1, u3); a3 = csub(b1, u3);
                }
                v[0][u] = a0; v[1][u] = a1; v[2][u] = a2; v[3][u] = a3;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) st2(x, i + r * q, v[r][0], v[r][1]);
        }
        __syncthreads();
    } else if (extra > 2) {
        // very long heads (M > 65536): one plain radix-2 pass over global memory per top stage, half-sizes M/2,
        // M/4, ... forwards and the reverse order backwards. Stage `sh` has half-size m = M >> (sh + 1): pair p sits
        // in block p / m at offset p % m, and its twiddle is root_M^(offset * 2^sh).
        for (int st = 0; st < extra; ++st) {
            const int sh = inverse ? extra - 1 - st : st;
            const int logm = logM - 1 - sh;
            const int m = 1 << logm;
            for (int p = 2 * tid; p < (M >> 1); p += 2 * kFftThreads) {     // m is even: p and p + 1 share a block
                const int off = p & (m - 1);
                const int i = ((p >> logm) << (logm + 1)) + off;
                cf a[2], c[2];
                ld2(x, i, a[0], a[1]);
                ld2(x, i + m, c[0], c[1]);
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const cf w = tw_m(lo, hi, (off + u) << sh);
                    if (!inverse) { const cf d = csub(a[u], c[u]); a[u] = cadd(a[u], c[u]); c[u] = cmul(d, w); }
                    else { const cf cw = cmul(c[u], cconj(w)); c[u] = csub(a[u], cw); a[u] = cadd(a[u], cw); }
                }
                st2(x, i, a[0], a[1]);
                st2(x, i + m, c[0], c[1]);
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ void chunk_load(cf* z, const cf* __restrict__ x, int C) {
    for (int i = 2 * threadIdx.x; i < C; i += 2 * kFftThreads) {
        cf a, b;
        ld2(x, i, a, b);
        z[pad(i)] = a;
        z[pad(i + 1)] = b;
    }
    __syncthreads();
}
__device__ __forceinline__ void chunk_store(cf* __restrict__ x, const cf* z, int C) {
    for (int i = 2 * threadIdx.x; i < C; i += 2 * kFftThreads) st2(x, i, z[pad(i)], z[pad(i + 1)]);
    __syncthreads();
}

// forward transform only (the filter's spectrum)
__device__ __noinline__ void fft_forward(cf* __restrict__ x, int logM, cf* z, const cf* lo, const cf* hi) {
    const int M = 1 << logM;
    const int logC = logM < kChunkLog ? logM : kChunkLog;
    const int C = 1 << logC;
    top_stages(x, logM, false, lo, hi);
    for (int base = 0; base < M; base += C) {
        chunk_load(z, x + base, C);
        // stage s of the whole transform, restricted to a chunk, is stage s of a C-point transform with the
        // twiddles of root M
        fft_lds(z, logC, logM - 1, false, lo, hi);
        chunk_store(x + base, z, C);
    }
}

// x <- IFFT(FFT(x) * bhat), unnormalised: circular convolution with the filter whose spectrum is bhat (same
// bit-reversed order). The product and both sets of chunk-local stages happen while a chunk sits in LDS.
__device__ __noinline__ void convolve(cf* __restrict__ x, const cf* __restrict__ bhat, int logM, cf* z,
                                      const cf* lo, const cf* hi) {
    const int M = 1 << logM;
    const int logC = logM < kChunkLog ? logM : kChunkLog;
    const int C = 1 << logC;
    top_stages(x, logM, false, lo, hi);
    for (int base = 0; base < M; base += C) {
        chunk_load(z, x + base, C);
        fft_lds(z, logC, logM - 1, false, lo, hi);
        for (int i = 2 * threadIdx.x; i < C; i += 2 * kFftThreads) {
            cf b0, b1;
            ld2(bhat + base, i, b0, b1);
            z[pad(i)] = cmul(z[pad(i)], b0);
            z[pad(i + 1)] = cmul(z[pad(i + 1)], b1);
        }
        __syncthreads();
        fft_lds(z, logC, logM - 1, true, lo, hi);
        chunk_store(x + base, z, C);
    }
    top_stages(x, logM, true, lo, hi);
}

// workspace of the chirp-z path, in complex elements: per head one array of M; per item the spectra of the two
// filters (M each) and the chirp itself (L <= M entries in a slot of M, which keeps every array 16-byte aligned)
struct BluesteinWs {
    cf* base;
    size_t M;          // stride unit: the largest transform of the batch
    int n_heads;
    __device__ cf* a_of(int head) const { return base + (size_t)head * M; }
    __device__ cf* bhat_of(int item, int which) const { return base + (size_t)n_heads * M + ((size_t)item * 3 + which) * M; }
    __device__ cf* chirp_of(int item) const { return bhat_of(item, 2); }
};

// the first item with the same length computes (and owns) the filter spectrum and the chirp table
__device__ __forceinline__ int owner_item(const int32_t* __restrict__ cu_seq, int item, int L) {
    for (int i = 0; i < item; ++i)
        if (cu_seq[i + 1] - cu_seq[i] == L) return i;
    return item;
}


// once per distinct length: the chirp table and the spectra of the two convolution filters.
//   forward transform (L samples in, K bins out): conj(chirp(m)) for m in (-L, K), wrapped around M;
//   inverse transform (K bins in, L samples out): conj(chirp(m)) for m in (-K, L), which is the first one read
//   backwards, so its spectrum is the first spectrum at the negated frequency.
__global__ __launch_bounds__(kFftThreads) void bluestein_prepare_kernel(const int32_t* __restrict__ cu_seq, BluesteinWs ws,
                                                                         double cutoff_frac, int cutoff_mode, int taper_bins,
                                                                         int skip_wide)
{
    extern __shared__ float smem[];
    const int item = blockIdx.x;
    const int L = cu_seq[item + 1] - cu_seq[item];
    if (pow2_length(L) || owner_item(cu_seq, item, L) != item) return;
    const int tid = threadIdx.x;
    const int K = wanted_bins(L, cutoff_frac, cutoff_mode, taper_bins);
    const int logM = bluestein_log(L, K);
    if (skip_wide && wide_size(logM)) return;         // prepared by the multi-workgroup kernels
    const int M = 1 << logM;
    const int C = M < (1 << kChunkLog) ? M : (1 << kChunkLog);
    cf* z = reinterpret_cast<cf*>(smem);
    cf* lo = z + padded_len(C);
    cf* hi = lo + kTwLo;
    fill_tables(lo, hi, (M >> 8) + 1, M);
    cf* B1 = ws.bhat_of(item, 0);
    cf* B2 = ws.bhat_of(item, 1);
    cf* ch = ws.chirp_of(item);
    for (int n = tid; n < L; n += kFftThreads) ch[n] = chirp(n, L);
    __syncthreads();
    for (int n = tid; n < M; n += kFftThreads) {
        cf b = {0.f, 0.f};
        if (n < K) b = cconj(ch[n]);
        else if (n > M - L) b = cconj(ch[M - n]);
        B1[n] = b;
    }
    __syncthreads();
    fft_forward(B1, logM, z, lo, hi);
    // both spectra sit in bit-reversed order: slot p holds frequency brev(p)
    const int shift = 32 - logM;
    for (int p = tid; p < M; p += kFftThreads) {
        const unsigned f = __brev((unsigned)p) >> shift;
        const unsigned nf = (M - f) & (M - 1);
        B2[p] = B1[__brev(nf) >> shift];
    }
}

__global__ __launch_bounds__(kFftThreads) void smooth_bluestein_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq,
    double cutoff_frac, float alpha, float* __restrict__ out, BluesteinWs ws,
    int32_t* __restrict__ kstar_out, int cutoffs_only, int skip_wide)
{
    extern __shared__ float smem[];
    const int head = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    if (alpha == 0.f || pow2_length(L)) return;       // the LDS kernel owns this head
    const int T = g.taper_bins;
    // a fixed cutoff that leaves only the mean, or everything: no transform (this kernel owns such heads whatever
    // the transform size would have been)
    const int fixed_kind = g.cutoff_mode == AUDIOKV_CUTOFF_FRACTION
                               ? degenerate_mask(L, (int)floor(cutoff_frac * (double)(L >> 1)), T) : 0;
    // all but the small transforms are spread over several workgroups by the kernels below
    if (skip_wide && fixed_kind == 0 &&
        wide_size(bluestein_log(L, wanted_bins(L, cutoff_frac, g.cutoff_mode, g.taper_bins)))) return;
    const size_t off = (size_t)tok0 * g.H_kv + (size_t)h * L;
    const float* src = in + off;
    float* dst = out + off;
    const int tid = threadIdx.x;
    if (g.cutoff_mode == AUDIOKV_CUTOFF_FRACTION && cutoffs_only) {
        if (tid == 0) kstar_out[head] = (int)floor(cutoff_frac * (double)(L >> 1));
        return;
    }
    if (fixed_kind != 0) {
        write_degenerate(fixed_kind, g, src, dst, L, pool_on_load, alpha, reinterpret_cast<double*>(smem));
        return;
    }
    const int K = wanted_bins(L, cutoff_frac, g.cutoff_mode, T);
    const int logM = bluestein_log(L, K);
    const int M = 1 << logM;
    const int C = M < (1 << kChunkLog) ? M : (1 << kChunkLog);
    cf* z = reinterpret_cast<cf*>(smem);
    cf* lo = z + padded_len(C);
    cf* hi = lo + kTwLo;
    const int n_hi = (M >> 8) + 1;                    // exponents below M/2
    const int owner = owner_item(cu_seq, item, L);
    cf* A = ws.a_of(head);
    const cf* ch = ws.chirp_of(owner);               // exp(-i*pi*n^2/L), n < L

    fill_tables(lo, hi, n_hi, M);
    // the chirped input, zero beyond L
    for (int n = tid; n < M; n += kFftThreads) {
        cf a = {0.f, 0.f};
        if (n < L) {
            const cf w = ch[n];
            const float sv = pool_on_load ? pooled_at(src, L, n, g.pool_kernel, g.pool_mode) : src[n];
            a = {sv * w.re, sv * w.im};
        }
        A[n] = a;
    }
    __syncthreads();
    convolve(A, ws.bhat_of(owner, 0), logM, z, lo, hi);

    // F_k = chirp(k) * A[k] / M for k < K. Low-pass mask (Eq. 17-18), then the inverse real transform from the
    // one-sided bins: s~_n = (1/L) Re sum_{k<K} g_k F~_k e^{+2 pi i k n / L}, g_k = 1 for k = 0 and for the Nyquist
    // bin of an even L, else 2. That sum is the conjugate of a forward chirp-z transform of conj(g F~), K points
    // in and L points out, so conj(g F~) * chirp goes into the same machinery with the second filter.
    int kstar = (int)floor(cutoff_frac * (double)(L >> 1));
    const float inv_m = 1.0f / (float)M;
    if (g.cutoff_mode != AUDIOKV_CUTOFF_FRACTION) {
        // |F_k| = |A[k]| / M: the chirp has unit modulus
        auto bin_energy = [&](int k) -> float {
            const cf a = A[k];
            const float re = a.re * inv_m, im = a.im * inv_m;
            return re * re + im * im;
        };
        EnergyScratch* sc = reinterpret_cast<EnergyScratch*>(hi + n_hi + 1);
        kstar = energy_cutoff(bin_energy, (L >> 1) + 1, g.cutoff_mode == AUDIOKV_CUTOFF_ENERGY_NO_DC ? 1 : 0, cutoff_frac, sc);
    }
    if (kstar_out && tid == 0) kstar_out[head] = kstar;
    if (cutoffs_only) return;
    if (g.cutoff_mode != AUDIOKV_CUTOFF_FRACTION && degenerate_mask(L, kstar, T) != 0) {
        // the energy rule left only the mean (usual when the DC bin is counted: it holds most of the energy of a
        // non-negative sequence) or everything
        __syncthreads();
        write_degenerate(degenerate_mask(L, kstar, T), g, src, dst, L, pool_on_load, alpha, reinterpret_cast<double*>(smem));
        return;
    }
    for (int k = tid; k < M; k += kFftThreads) {
        cf v = {0.f, 0.f};
        if (k < K) {
            const float wgt = mask_weight(k, kstar, T) * ((k == 0 || 2 * k == L) ? 1.f : 2.f);
            if (wgt > 0.f) {
                const cf w = ch[k];
                cf F = cmul(w, A[k]);
                F = {F.re * inv_m * wgt, F.im * inv_m * wgt};
                v = cmul(cconj(F), w);
            }
        }
        A[k] = v;
    }
    __syncthreads();
    convolve(A, ws.bhat_of(owner, 1), logM, z, lo, hi);

    // s~_n = Re(chirp(n) * A[n]) / (M * L); residual mix (Eq. 20)
    const float scale = inv_m / (float)L;
    for (int n = tid; n < L; n += kFftThreads) {
        const cf y = cmul(ch[n], A[n]);
        const float st = y.re * scale;
        if (alpha == 1.f) dst[n] = st;
        else {
            const float s0 = pool_on_load ? pooled_at(src, L, n, g.pool_kernel, g.pool_mode) : src[n];
            dst[n] = (1.f - alpha) * s0 + alpha * st;
        }
    }
}

// ---- transforms of 4096 points and more, spread over several workgroups (fixed-fraction cutoff) -------------------
// The same convolutions as above, cut at the points where every element of the array has to be complete:
//   wide_first   chirped input formed on the fly, forward top stage(s)            (one thread per butterfly)
//   wide_chunk   per chunk of M / 4 points: forward LDS stages, x filter, inverse LDS stages
//   wide_middle  inverse top stage(s) -> bins; mask; input of the inverse transform; forward top stage(s)
//   wide_chunk   again, with the second filter
//   wide_last    inverse top stage(s) -> samples; residual mix; store
// Few heads (one layer of a prefill) then use 8-64 workgroups per head instead of one.

constexpr int kWideThreads = 256;

struct WideHead {                      // what every kernel of the sequence derives for its head
    int L, K, logM, M, extra, R, q, owner;
    size_t off;
};

__device__ __forceinline__ bool wide_head(const Geom& g, const int32_t* __restrict__ cu_seq, int head, double cutoff_frac,
                                          WideHead& w) {
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    w.L = cu_seq[item + 1] - tok0;
    if (pow2_length(w.L)) return false;
    // (the multi-workgroup sequence runs with a fixed cutoff only) masks that need no transform: single-workgroup kernel
    if (degenerate_mask(w.L, (int)floor(cutoff_frac * (double)(w.L >> 1)), g.taper_bins) != 0) return false;
    w.K = wanted_bins(w.L, cutoff_frac, g.cutoff_mode, g.taper_bins);
    w.logM = bluestein_log(w.L, w.K);
    if (!wide_size(w.logM)) return false;              // small or very large: the single-workgroup kernel owns it
    w.M = 1 << w.logM;
    // two top stages and four chunks of M / 4 points up to M = 65536; beyond, as many top stages as it takes for
    // a chunk to fit the LDS (8 or 16 chunks of 16384 points)
    w.extra = w.logM - kChunkLog > 2 ? w.logM - kChunkLog : 2;
    w.R = 1 << w.extra;
    w.q = w.M >> w.extra;
    w.owner = owner_item(cu_seq, item, w.L);
    w.off = (size_t)tok0 * g.H_kv + (size_t)h * w.L;
    return true;
}

// exp(-2*pi*i*e/M), e < M/2, straight from the fp32 library (e/M is exact)
__device__ __forceinline__ cf root_m(int e, int M) {
    float sn, cs;
    sincospif(2.0f * (float)e / (float)M, &sn, &cs);
    return {cs, -sn};
}

constexpr int kWideMaxR = 16;          // chunks per transform at most (M = 262144)

// one radix-2 stage on the register values v[r] = x[i + r*q], partners HS chunks apart; `st` counts the stages from
// the top (half-size M >> (st + 1)), so the twiddle is root_M^(offset in the half * 2^st)
template <int HS>
__device__ __forceinline__ void top_stage(cf* v, int R, int q, int i, int M, int st, bool inverse) {
#pragma unroll
    for (int r = 0; r < kWideMaxR; ++r) {
        if ((r & HS) != 0 || r + HS >= kWideMaxR) continue;      // compile-time after unrolling
        if (r + HS < R) {
            const cf w = root_m(((r & (HS - 1)) * q + i) << st, M);
            if (!inverse) { const cf d = csub(v[r], v[r + HS]); v[r] = cadd(v[r], v[r + HS]); v[r + HS] = cmul(d, w); }
            else { const cf cw = cmul(v[r + HS], cconj(w)); v[r + HS] = csub(v[r], cw); v[r] = cadd(v[r], cw); }
        }
    }
}

// the top stage(s) on the R values v[r] = x[i + r*q] held in registers (see top_stages for the index algebra)
template <int MAXR>
__device__ __forceinline__ void top_butterfly(cf* v, int i, int M, int extra, bool inverse) {
    if (MAXR > 4 && extra > 2) {
        // 8 or 16 chunks: three or four plain radix-2 stages, largest half-size first forwards, last backwards
        const int R = 1 << extra, q = M >> extra;
        if (!inverse) {
            if (extra == 4) top_stage<8>(v, R, q, i, M, 0, false);
            top_stage<4>(v, R, q, i, M, extra - 3, false);
            top_stage<2>(v, R, q, i, M, extra - 2, false);
            top_stage<1>(v, R, q, i, M, extra - 1, false);
        } else {
            top_stage<1>(v, R, q, i, M, extra - 1, true);
            top_stage<2>(v, R, q, i, M, extra - 2, true);
            top_stage<4>(v, R, q, i, M, extra - 3, true);
            if (extra == 4) top_stage<8>(v, R, q, i, M, 0, true);
        }
        return;
    }
    if (extra == 1) {
        const cf w = root_m(i, M);
        if (!inverse) { const cf d = csub(v[0], v[1]); v[0] = cadd(v[0], v[1]); v[1] = cmul(d, w); }
        else { const cf cw = cmul(v[1], cconj(w)); v[1] = csub(v[0], cw); v[0] = cadd(v[0], cw); }
        return;
    }
    const cf w1 = root_m(i, M), w2 = root_m(2 * i, M);
    cf a0 = v[0], a1 = v[1], a2 = v[2], a3 = v[3];
    if (!inverse) {
        const cf b0 = cadd(a0, a2), b2 = cmul(csub(a0, a2), w1);
        const cf b1 = cadd(a1, a3), b3 = mul_neg_i(cmul(csub(a1, a3), w1));
        a0 = cadd(b0, b1); a1 = cmul(csub(b0, b1), w2);
        a2 = cadd(b2, b3); a3 = cmul(csub(b2, b3), w2);
    } else {
        const cf w1c = cconj(w1), w2c = cconj(w2);
        const cf t1 = cmul(a1, w2c), t3 = cmul(a3, w2c);
        const cf b0 = cadd(a0, t1), b1 = csub(a0, t1), b2 = cadd(a2, t3), b3 = csub(a2, t3);
        const cf u2 = cmul(b2, w1c), u3 = mul_pos_i(cmul(b3, w1c));
        a0 = cadd(b0, u2); a2 = csub(b0, u2);
        a1 = cadd(b1, u3); a3 = csub(b1, u3);
    }
    v[0] = a0; v[1] = a1; v[2] = a2; v[3] = a3;
}

// preparation of the filters of a wide transform, spread the same way: chirp table; wrapped filter + forward top
// stage(s); chunk-local stages (wide_chunk_kernel, which_filter = -1); second filter by the frequency-negating gather.
// Grids run over the first head of every item; only items that own their length work.
__device__ __forceinline__ bool wide_owner(const Geom& g, const int32_t* __restrict__ cu_seq, int item, double cutoff_frac,
                                           WideHead& w) {
    return wide_head(g, cu_seq, item * g.H_kv, cutoff_frac, w) && w.owner == item;
}

__global__ __launch_bounds__(kWideThreads) void wide_prep_chirp_kernel(Geom g, const int32_t* __restrict__ cu_seq,
                                                                       double cutoff_frac, BluesteinWs ws)
{
    WideHead w;
    const int item = blockIdx.y;
    if (!wide_owner(g, cu_seq, item, cutoff_frac, w)) return;
    cf* ch = ws.chirp_of(item);
    for (int n = blockIdx.x * kWideThreads + threadIdx.x; n < w.L; n += gridDim.x * kWideThreads) ch[n] = chirp(n, w.L);
}

template <int MAXR>
__global__ __launch_bounds__(kWideThreads) void wide_prep_first_kernel(Geom g, const int32_t* __restrict__ cu_seq,
                                                                       double cutoff_frac, BluesteinWs ws)
{
    WideHead w;
    const int item = blockIdx.y;
    if (!wide_owner(g, cu_seq, item, cutoff_frac, w)) return;
    if (w.R > MAXR) return;                             // (the launcher picks the instantiation that holds every head)
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    if (i >= w.q) return;
    const cf* ch = ws.chirp_of(item);
    cf* B1 = ws.bhat_of(item, 0);
    cf v[MAXR];
#pragma unroll
    for (int r = 0; r < MAXR; ++r) {
        const int n = i + r * w.q;
        cf b = {0.f, 0.f};
        if (r < w.R) {
            if (n < w.K) b = cconj(ch[n]);
            else if (n > w.M - w.L) b = cconj(ch[w.M - n]);
        }
        v[r] = b;
    }
    top_butterfly<MAXR>(v, i, w.M, w.extra, false);
#pragma unroll
    for (int r = 0; r < MAXR; ++r)
        if (r < w.R) B1[i + r * w.q] = v[r];
}

__global__ __launch_bounds__(kWideThreads) void wide_prep_second_kernel(Geom g, const int32_t* __restrict__ cu_seq,
                                                                        double cutoff_frac, BluesteinWs ws)
{
    WideHead w;
    const int item = blockIdx.y;
    if (!wide_owner(g, cu_seq, item, cutoff_frac, w)) return;
    const cf* B1 = ws.bhat_of(item, 0);
    cf* B2 = ws.bhat_of(item, 1);
    const int shift = 32 - w.logM;
    for (int p = blockIdx.x * kWideThreads + threadIdx.x; p < w.M; p += gridDim.x * kWideThreads) {
        const unsigned f = __brev((unsigned)p) >> shift;
        const unsigned nf = (w.M - f) & (w.M - 1);
        B2[p] = B1[__brev(nf) >> shift];
    }
}

template <int MAXR>
__global__ __launch_bounds__(kWideThreads) void wide_first_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq, double cutoff_frac,
    BluesteinWs ws)
{
    WideHead w;
    const int head = blockIdx.y;
    if (!wide_head(g, cu_seq, head, cutoff_frac, w)) return;
    if (w.R > MAXR) return;                             // (the launcher picks the instantiation that holds every head)
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    if (i >= w.q) return;
    const float* src = in + w.off;
    const cf* ch = ws.chirp_of(w.owner);
    cf* A = ws.a_of(head);
    cf v[MAXR];
#pragma unroll
    for (int r = 0; r < MAXR; ++r) {          // (guards, not breaks: the loop must unroll for v to stay in registers)
        const int n = i + r * w.q;
        cf a = {0.f, 0.f};
        if (r < w.R && n < w.L) {
            const cf c = ch[n];
            const float sv = pool_on_load ? pooled_at(src, w.L, n, g.pool_kernel, g.pool_mode) : src[n];
            a = {sv * c.re, sv * c.im};
        }
        v[r] = a;
    }
    top_butterfly<MAXR>(v, i, w.M, w.extra, false);
#pragma unroll
    for (int r = 0; r < MAXR; ++r)
        if (r < w.R) A[i + r * w.q] = v[r];
}

__global__ __launch_bounds__(kFftThreads) void wide_chunk_kernel(
    Geom g, const int32_t* __restrict__ cu_seq, double cutoff_frac, BluesteinWs ws, int which_filter)
{
    extern __shared__ float smem[];
    WideHead w;
    const int head = blockIdx.y;
    if (!wide_head(g, cu_seq, head, cutoff_frac, w)) return;
    const int chunk = blockIdx.x;
    if (chunk >= w.R) return;
    const int logC = w.logM - w.extra;
    const int C = 1 << logC;
    cf* z = reinterpret_cast<cf*>(smem);
    cf* lo = z + padded_len(C);
    cf* hi = lo + kTwLo;
    fill_tables(lo, hi, (w.M >> 8) + 1, w.M);
    if (which_filter < 0) {
        // preparation: chunk-local forward stages of the first filter itself (one head per item does it)
        const int item = head / g.H_kv;
        if (head != item * g.H_kv || w.owner != item) return;
        cf* b = ws.bhat_of(item, 0) + (size_t)chunk * C;
        chunk_load(z, b, C);
        fft_lds(z, logC, w.logM - 1, false, lo, hi);
        chunk_store(b, z, C);
        return;
    }
    cf* x = ws.a_of(head) + (size_t)chunk * C;
    const cf* bhat = ws.bhat_of(w.owner, which_filter) + (size_t)chunk * C;
    chunk_load(z, x, C);                                // ends with a barrier: the tables are complete too
    fft_lds(z, logC, w.logM - 1, false, lo, hi);
    for (int i = 2 * threadIdx.x; i < C; i += 2 * kFftThreads) {
        cf b0, b1;
        ld2(bhat, i, b0, b1);
        z[pad(i)] = cmul(z[pad(i)], b0);
        z[pad(i + 1)] = cmul(z[pad(i + 1)], b1);
    }
    __syncthreads();
    fft_lds(z, logC, w.logM - 1, true, lo, hi);
    chunk_store(x, z, C);
}

template <int MAXR>
__global__ __launch_bounds__(kWideThreads) void wide_middle_kernel(
    Geom g, const int32_t* __restrict__ cu_seq, double cutoff_frac, BluesteinWs ws, int32_t* __restrict__ kstar_out)
{
    WideHead w;
    const int head = blockIdx.y;
    if (!wide_head(g, cu_seq, head, cutoff_frac, w)) return;
    if (w.R > MAXR) return;                             // (the launcher picks the instantiation that holds every head)
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    const int kstar = (int)floor(cutoff_frac * (double)(w.L >> 1));
    if (kstar_out && i == 0) kstar_out[head] = kstar;
    if (i >= w.q) return;
    const cf* ch = ws.chirp_of(w.owner);
    cf* A = ws.a_of(head);
    const float inv_m = 1.0f / (float)w.M;
    const int T = g.taper_bins;
    cf v[MAXR];
#pragma unroll
    for (int r = 0; r < MAXR; ++r) v[r] = r < w.R ? A[i + r * w.q] : cf{0.f, 0.f};
    top_butterfly<MAXR>(v, i, w.M, w.extra, true);            // v[r] is now the convolution at position k = i + r*q
#pragma unroll
    for (int r = 0; r < MAXR; ++r) {
        const int k = i + r * w.q;
        cf o = {0.f, 0.f};
        if (r < w.R && k < w.K) {
            const float wgt = mask_weight(k, kstar, T) * ((k == 0 || 2 * k == w.L) ? 1.f : 2.f);
            if (wgt > 0.f) {
                const cf c = ch[k];
                cf F = cmul(c, v[r]);
                F = {F.re * inv_m * wgt, F.im * inv_m * wgt};
                o = cmul(cconj(F), c);
            }
        }
        v[r] = o;
    }
    top_butterfly<MAXR>(v, i, w.M, w.extra, false);
#pragma unroll
    for (int r = 0; r < MAXR; ++r)
        if (r < w.R) A[i + r * w.q] = v[r];
}

template <int MAXR>
__global__ __launch_bounds__(kWideThreads) void wide_last_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq, double cutoff_frac,
    float alpha, float* __restrict__ out, BluesteinWs ws)
{
    WideHead w;
    const int head = blockIdx.y;
    if (!wide_head(g, cu_seq, head, cutoff_frac, w)) return;
    if (w.R > MAXR) return;                             // (the launcher picks the instantiation that holds every head)
    const int i = blockIdx.x * kWideThreads + threadIdx.x;
    if (i >= w.q) return;
    const float* src = in + w.off;
    float* dst = out + w.off;
    const cf* ch = ws.chirp_of(w.owner);
    const cf* A = ws.a_of(head);
    const float scale = 1.0f / (float)w.M / (float)w.L;
    cf v[MAXR];
#pragma unroll
    for (int r = 0; r < MAXR; ++r) v[r] = r < w.R ? A[i + r * w.q] : cf{0.f, 0.f};
    top_butterfly<MAXR>(v, i, w.M, w.extra, true);
#pragma unroll
    for (int r = 0; r < MAXR; ++r) {
        const int n = i + r * w.q;
        if (r < w.R && n < w.L) {
            const cf y = cmul(ch[n], v[r]);
            const float st = y.re * scale;
            if (alpha == 1.f) dst[n] = st;
            else {
                const float s0 = pool_on_load ? pooled_at(src, w.L, n, g.pool_kernel, g.pool_mode) : src[n];
                dst[n] = (1.f - alpha) * s0 + alpha * st;
            }
        }
    }
}

}  // namespace

hipError_t launch_pool(const Geom& g, const float* raw, const int32_t* cu_seqlens, int max_L,
                       float* pooled, hipStream_t s)
{
    const int n_heads = g.n_items * g.H_kv;
    const int bx = max(1, min(64, (max_L + 255) / 256));
    hipLaunchKernelGGL(pool_kernel, dim3(bx, n_heads), dim3(256), 0, s, g, raw, cu_seqlens, pooled);
    return hipGetLastError();
}

bool smooth_supported(int L) { return pow2_length(L) || (L >= 1 && L <= 131072 && bluestein_log_max(L) <= kMaxBluesteinLog); }

namespace {
// scratch of the chirp-z transforms (lengths that are not powers of two), sized for the largest transform any cutoff
// can ask for (all bins wanted): per head the working array (M), per item the two filter spectra and the chirp table
size_t bluestein_bytes(const int32_t* seqlens_host, int n_items, int H_kv) {
    int max_log = 0;
    for (int i = 0; i < n_items; ++i)
        if (!pow2_length(seqlens_host[i])) max_log = max(max_log, bluestein_log_max(seqlens_host[i]));
    if (max_log == 0) return 0;
    const size_t M = (size_t)1 << max_log;
    return ((size_t)n_items * H_kv * M + (size_t)n_items * 3 * M) * sizeof(cf);
}
// sub-spectra of the several-workgroups path for power-of-two lengths (calls with few heads only)
int dec_max_length(const int32_t* seqlens_host, int n_items, int H_kv) {
    if ((long long)n_items * H_kv > kDecMaxHeads) return 0;
    int mx = 0;
    for (int i = 0; i < n_items; ++i)
        if (dec_length(seqlens_host[i])) mx = max(mx, seqlens_host[i]);
    return mx;
}
size_t dec_bytes(const int32_t* seqlens_host, int n_items, int H_kv) {
    const int mx = dec_max_length(seqlens_host, n_items, H_kv);
    return mx ? (size_t)n_items * H_kv * dec_head_elems(mx) * sizeof(cf) : 0;
}
}  // namespace

// The two regions follow each other in the workspace (chirp-z first). Only the first is indispensable: without room
// for the second, power-of-two heads simply stay on one workgroup each.
size_t smooth_workspace_bytes(const int32_t* seqlens_host, int n_items, int H_kv) {
    return bluestein_bytes(seqlens_host, n_items, H_kv) + dec_bytes(seqlens_host, n_items, H_kv);
}
size_t smooth_workspace_required(const int32_t* seqlens_host, int n_items, int H_kv) {
    return bluestein_bytes(seqlens_host, n_items, H_kv);
}

namespace {
struct SmoothPlan { int max_pow2 = 0, max_log = 0; bool any_wide = false; };

SmoothPlan plan_smooth(const Geom& g, const int32_t* seqlens_host, int n_items, double cutoff_frac) {
    SmoothPlan p;
    for (int i = 0; i < n_items; ++i) {
        if (pow2_length(seqlens_host[i])) p.max_pow2 = max(p.max_pow2, seqlens_host[i]);
        else {
            const int lg = bluestein_log(seqlens_host[i], wanted_bins(seqlens_host[i], cutoff_frac, g.cutoff_mode, g.taper_bins));
            p.max_log = max(p.max_log, lg);
            p.any_wide = p.any_wide || wide_size(lg);
        }
    }
    return p;
}

hipError_t smooth_kernel_attributes() {
    static std::atomic<bool> attr_set{false};
    if (attr_set) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(smooth_pow2_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(smooth_bluestein_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(bluestein_prepare_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(wide_chunk_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) attr_set = true;
    return e;
}

size_t bluestein_smem(const Geom& g, size_t M) {
    const size_t extra = g.cutoff_mode != AUDIOKV_CUTOFF_FRACTION ? sizeof(EnergyScratch) + 2 * sizeof(cf) : 0;
    const size_t C = M < ((size_t)1 << kChunkLog) ? M : ((size_t)1 << kChunkLog);
    return std::max((padded_len(C) + kTwLo + (M >> 8) + 1) * sizeof(cf) + extra, (size_t)kFftThreads * sizeof(double));
}
}  // namespace

hipError_t launch_smooth_filters(const Geom& g, const int32_t* cu_seqlens, const int32_t* seqlens_host, int n_items,
                                 double cutoff_frac, void* workspace, hipStream_t s)
{
    const SmoothPlan pl = plan_smooth(g, seqlens_host, n_items, cutoff_frac);
    if (pl.max_log == 0) return hipSuccess;
    if (!workspace) return hipErrorInvalidValue;
    hipError_t e = smooth_kernel_attributes();
    if (e != hipSuccess) return e;
    const size_t M = (size_t)1 << pl.max_log;
    const BluesteinWs bw{static_cast<cf*>(workspace), M, g.n_items * g.H_kv};
    const bool wide = pl.any_wide;
    hipLaunchKernelGGL(bluestein_prepare_kernel, dim3(g.n_items), dim3(kFftThreads), bluestein_smem(g, M), s, cu_seqlens,
                       bw, cutoff_frac, g.cutoff_mode, g.taper_bins, wide ? 1 : 0);
    if (wide) {
        const int extra_stages = pl.max_log - kChunkLog > 2 ? pl.max_log - kChunkLog : 2;    // of the largest transform
        const unsigned q = (unsigned)(M >> extra_stages);
        const dim3 ew((q + kWideThreads - 1) / kWideThreads, (unsigned)g.n_items);
        hipLaunchKernelGGL(wide_prep_chirp_kernel, ew, dim3(kWideThreads), 0, s, g, cu_seqlens, cutoff_frac, bw);
        if (extra_stages <= 2)
            hipLaunchKernelGGL(wide_prep_first_kernel<4>, ew, dim3(kWideThreads), 0, s, g, cu_seqlens, cutoff_frac, bw);
        else
            hipLaunchKernelGGL(wide_prep_first_kernel<kWideMaxR>, ew, dim3(kWideThreads), 0, s, g, cu_seqlens, cutoff_frac, bw);
        hipLaunchKernelGGL(wide_chunk_kernel, dim3((unsigned)1 << extra_stages, (unsigned)(g.n_items * g.H_kv)),
                           dim3(kFftThreads), bluestein_smem(g, M), s, g, cu_seqlens, cutoff_frac, bw, -1);
        hipLaunchKernelGGL(wide_prep_second_kernel, ew, dim3(kWideThreads), 0, s, g, cu_seqlens, cutoff_frac, bw);
    }
    return hipGetLastError();
}

hipError_t launch_smooth(const Geom& g, const float* in, bool pool_on_load, const int32_t* cu_seqlens,
                         const int32_t* seqlens_host, int n_items, double cutoff_frac, double alpha,
                         float* out, void* workspace, size_t workspace_bytes, int32_t* kstar_out, bool cutoffs_only,
                         hipStream_t s, bool filters_ready)
{
    if (cutoffs_only && !kstar_out) return hipErrorInvalidValue;
    const size_t extra = g.cutoff_mode != AUDIOKV_CUTOFF_FRACTION ? sizeof(EnergyScratch) + 2 * sizeof(cf) : 0;
    const SmoothPlan pl = plan_smooth(g, seqlens_host, n_items, cutoff_frac);
    const int max_pow2 = pl.max_pow2, max_log = pl.max_log;
    const int n_heads = g.n_items * g.H_kv;
    {
        const hipError_t e = smooth_kernel_attributes();
        if (e != hipSuccess) return e;
    }
    // power-of-two heads of a call with few heads go over several workgroups each (fixed cutoff only)
    const int dec_L = (alpha != 0.0 && !cutoffs_only && g.cutoff_mode == AUDIOKV_CUTOFF_FRACTION && workspace &&
                       workspace_bytes >= smooth_workspace_bytes(seqlens_host, n_items, g.H_kv))
                          ? dec_max_length(seqlens_host, n_items, g.H_kv) : 0;
    const DecWs dw{reinterpret_cast<cf*>(static_cast<char*>(workspace) + bluestein_bytes(seqlens_host, n_items, g.H_kv)),
                   dec_L ? dec_head_elems(dec_L) : 0};
    // every head is handled by exactly one path (alpha = 0 copies: the single-workgroup kernel)
    bool all_dec = dec_L > 0;
    for (int i = 0; i < n_items && all_dec; ++i)
        all_dec = dec_length(seqlens_host[i]) &&
                  degenerate_mask(seqlens_host[i], (int)floor(cutoff_frac * (double)(seqlens_host[i] >> 1)), g.taper_bins) != 2;
    if (!all_dec && (max_pow2 > 0 || alpha == 0.0 || max_log == 0)) {
        const int n_hi = (max_pow2 >> 8) + 1;
        // (at least the kFftThreads doubles that the no-transform paths reduce in)
        const size_t smem = std::max((padded_len((size_t)max_pow2 >> 1) + kTwLo + n_hi) * sizeof(cf) + extra,
                                     (size_t)kFftThreads * sizeof(double));
        hipLaunchKernelGGL(smooth_pow2_kernel, dim3(n_heads), dim3(kFftThreads), smem, s, g, in,
                           pool_on_load ? 1 : 0, cu_seqlens, cutoff_frac, (float)alpha, out, kstar_out, cutoffs_only ? 1 : 0,
                           dec_L ? 1 : 0);
    }
    if (dec_L) {
        const int M = dec_L >> kDecLog;
        const size_t smem = (padded_len(M) + kTwLo + (M >> 8) + 1) * sizeof(cf);
        const dim3 pairs(kDec / 2, (unsigned)n_heads);
        hipLaunchKernelGGL(dec_forward_kernel, pairs, dim3(kDecThreads), smem, s, g, in, pool_on_load ? 1 : 0, cu_seqlens,
                           cutoff_frac, dw);
        hipLaunchKernelGGL(dec_combine_kernel,
                           dim3((unsigned)(((M >> 1) + 1 + kDecCombineThreads - 1) / kDecCombineThreads), (unsigned)n_heads),
                           dim3(kDecCombineThreads), 0, s, g, cu_seqlens, cutoff_frac, dw);
        hipLaunchKernelGGL(dec_inverse_kernel, pairs, dim3(kDecThreads), smem, s, g, in, pool_on_load ? 1 : 0, cu_seqlens,
                           cutoff_frac, (float)alpha, out, dw);
    }
    if (max_log > 0 && alpha != 0.0) {
        if (!workspace) return hipErrorInvalidValue;
        if (!filters_ready) {
            const hipError_t e = launch_smooth_filters(g, cu_seqlens, seqlens_host, n_items, cutoff_frac, workspace, s);
            if (e != hipSuccess) return e;
        }
        const size_t M = (size_t)1 << max_log;
        const BluesteinWs bw{static_cast<cf*>(workspace), M, n_heads};
        // transforms wider than one LDS chunk go to the multi-workgroup sequence, unless the cutoff has to be found
        // from the whole spectrum first
        const bool wide = pl.any_wide && g.cutoff_mode == AUDIOKV_CUTOFF_FRACTION && !cutoffs_only;
        hipLaunchKernelGGL(smooth_bluestein_kernel, dim3(n_heads), dim3(kFftThreads), bluestein_smem(g, M), s, g, in,
                           pool_on_load ? 1 : 0, cu_seqlens, cutoff_frac, (float)alpha, out, bw, kstar_out,
                           cutoffs_only ? 1 : 0, wide ? 1 : 0);
        if (wide) {
            const int extra_stages = max_log - kChunkLog > 2 ? max_log - kChunkLog : 2;      // of the largest transform
            const unsigned q = (unsigned)(M >> extra_stages);
            const dim3 ew((q + kWideThreads - 1) / kWideThreads, (unsigned)n_heads);
            const dim3 cw((unsigned)1 << extra_stages, (unsigned)n_heads);
            const size_t csm = bluestein_smem(g, M);
            // instantiated for at most 4 chunks per transform (the usual case: everything in registers is small) and for 16
            auto sequence = [&](auto maxr) {
                constexpr int MAXR = decltype(maxr)::value;
                hipLaunchKernelGGL(wide_first_kernel<MAXR>, ew, dim3(kWideThreads), 0, s, g, in, pool_on_load ? 1 : 0,
                                   cu_seqlens, cutoff_frac, bw);
                hipLaunchKernelGGL(wide_chunk_kernel, cw, dim3(kFftThreads), csm, s, g, cu_seqlens, cutoff_frac, bw, 0);
                hipLaunchKernelGGL(wide_middle_kernel<MAXR>, ew, dim3(kWideThreads), 0, s, g, cu_seqlens, cutoff_frac, bw,
                                   kstar_out);
                hipLaunchKernelGGL(wide_chunk_kernel, cw, dim3(kFftThreads), csm, s, g, cu_seqlens, cutoff_frac, bw, 1);
                hipLaunchKernelGGL(wide_last_kernel<MAXR>, ew, dim3(kWideThreads), 0, s, g, in, pool_on_load ? 1 : 0,
                                   cu_seqlens, cutoff_frac, (float)alpha, out, bw);
            };
            if (extra_stages <= 2) sequence(std::integral_constant<int, 4>{});
            else sequence(std::integral_constant<int, kWideMaxR>{});
        }
    }
    return hipGetLastError();
}

}  // namespace audiokv
