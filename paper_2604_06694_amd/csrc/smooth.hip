// Stage 1 tail (local pooling) and stage 3 (Spectral Score Smoothing, paper
// Sec. 3.3 Eqs. 13, 17-20).
//
// SSS for a power-of-two L runs entirely inside one workgroup's LDS: the real
// sequence is viewed as L/2 complex numbers, transformed by an in-place
// radix-2 decimation-in-frequency FFT (natural order in, bit-reversed out),
// turned into the real spectrum pair by pair, masked above k*, turned back,
// and inverted by a decimation-in-time FFT (bit-reversed in, natural out), so
// no reordering pass is needed. Twiddles come from two small tables filled
// from float64 sincospi: w^e = hi[e >> 7] * lo[e & 127].
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
        return acc / (float)kernel;                       // divisor is always the kernel size
    }
    float acc = -INFINITY;
    for (int t = -half; t <= half; ++t) {
        const int p = j + t;
        if (p >= 0 && p < L) acc = fmaxf(acc, x[p]);
    }
    return acc;
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

struct cf { float re, im; };
__device__ __forceinline__ cf cmul(cf a, cf b) { return {a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re}; }
__device__ __forceinline__ cf cadd(cf a, cf b) { return {a.re + b.re, a.im + b.im}; }
__device__ __forceinline__ cf csub(cf a, cf b) { return {a.re - b.re, a.im - b.im}; }
__device__ __forceinline__ cf cconj(cf a) { return {a.re, -a.im}; }

// exp(-2*pi*i*e/L) for 0 <= e <= L/2
__device__ __forceinline__ cf twiddle(const cf* lo, const cf* hi, int e) {
    return cmul(hi[e >> 7], lo[e & (kTwLo - 1)]);
}

__global__ __launch_bounds__(kFftThreads) void smooth_pow2_kernel(
    Geom g, const float* __restrict__ in, int pool_on_load, const int32_t* __restrict__ cu_seq,
    double cutoff_frac, float alpha,
    float* __restrict__ out)
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

    if (alpha == 0.f || L < 4 || (L & (L - 1)) != 0) {
        // alpha = 0: the mix returns s itself. (Other lengths never reach this kernel.)
        for (int j = tid; j < L; j += kFftThreads)
            dst[j] = pool_on_load ? pooled_at(src, L, j, g.pool_kernel, g.pool_mode) : src[j];
        return;
    }

    const int N = L >> 1;                         // complex length
    const int logN = 31 - __clz(N);
    float* x = smem;                              // L floats = N complex
    cf* z = reinterpret_cast<cf*>(smem);
    cf* lo = reinterpret_cast<cf*>(smem + L);     // kTwLo entries: w^j
    cf* hi = lo + kTwLo;                          // (L/2)/128 + 1 entries: w^(128 j)
    const int n_hi = (N >> 7) + 1;

    for (int j = tid; j < L; j += kFftThreads)
        x[j] = pool_on_load ? pooled_at(src, L, j, g.pool_kernel, g.pool_mode) : src[j];
    for (int t = tid; t < kTwLo + n_hi; t += kFftThreads) {
        const long long e = t < kTwLo ? t : (long long)(t - kTwLo) * kTwLo;
        double sn, cs;
        sincospi(2.0 * (double)e / (double)L, &sn, &cs);
        const cf w = {(float)cs, (float)(-sn)};
        if (t < kTwLo) lo[t] = w; else hi[t - kTwLo] = w;
    }
    __syncthreads();

    // forward: decimation in frequency, half-size m = N/2 ... 1
    for (int s = logN - 1; s >= 0; --s) {
        const int m = 1 << s;
        for (int b = tid; b < (N >> 1); b += kFftThreads) {
            const int j = b & (m - 1);
            const int i = ((b >> s) << (s + 1)) | j;
            const cf a = z[i], c = z[i + m];
            z[i] = cadd(a, c);
            // w_N^(j * N/(2m)) = w_L^(2 * j * N/(2m)) = w_L^(j << (logN - s))
            z[i + m] = cmul(csub(a, c), twiddle(lo, hi, j << (logN - s)));
        }
        __syncthreads();
    }

    // spectrum of the real sequence, low-pass mask (Eq. 17-18), and back, pair (k, N-k) at a time
    const int kstar = (int)floor(cutoff_frac * (double)N);     // N = floor(L/2) = n_bins - 1
    const int shift = 32 - logN;
    for (int k = tid; k <= (N >> 1); k += kFftThreads) {
        if (k == 0) {
            const cf z0 = z[0];
            const float X0 = z0.re + z0.im;                     // DC bin, always kept (0 <= k*)
            const float XN = (N <= kstar) ? (z0.re - z0.im) : 0.f;   // Nyquist bin
            z[0] = {0.5f * (X0 + XN), 0.5f * (X0 - XN)};
            continue;
        }
        const int pa = logN ? (int)(__brev((unsigned)k) >> shift) : 0;
        const int pb = logN ? (int)(__brev((unsigned)(N - k)) >> shift) : 0;
        const cf A = z[pa];
        const cf B = cconj(z[pb]);
        const cf E = {0.5f * (A.re + B.re), 0.5f * (A.im + B.im)};
        const cf Dm = csub(A, B);
        const cf O = {0.5f * Dm.im, -0.5f * Dm.re};             // -i (A - B) / 2
        const cf Wk = twiddle(lo, hi, k);
        const cf WO = cmul(Wk, O);
        cf Xk = cadd(E, WO);                                    // bin k
        cf Xn = cconj(csub(E, WO));                             // bin N - k
        if (k > kstar) Xk = {0.f, 0.f};
        if (N - k > kstar) Xn = {0.f, 0.f};
        const cf Xnc = cconj(Xn);
        const cf E2 = {0.5f * (Xk.re + Xnc.re), 0.5f * (Xk.im + Xnc.im)};
        const cf H2 = {0.5f * (Xk.re - Xnc.re), 0.5f * (Xk.im - Xnc.im)};
        const cf O2 = cmul(H2, cconj(Wk));
        // Z'[k] = E' + i O' ; Z'[N-k] = conj(E') + i conj(O')
        z[pa] = {E2.re - O2.im, E2.im + O2.re};
        if (pb != pa) z[pb] = {E2.re + O2.im, -E2.im + O2.re};
    }
    __syncthreads();

    // inverse: decimation in time, half-size m = 1 ... N/2, conjugate twiddles
    for (int s = 0; s < logN; ++s) {
        const int m = 1 << s;
        for (int b = tid; b < (N >> 1); b += kFftThreads) {
            const int j = b & (m - 1);
            const int i = ((b >> s) << (s + 1)) | j;
            const cf a = z[i];
            const cf c = cmul(z[i + m], cconj(twiddle(lo, hi, j << (logN - s))));
            z[i] = cadd(a, c);
            z[i + m] = csub(a, c);
        }
        __syncthreads();
    }

    // residual mix (Eq. 20); 1/N completes the inverse transform
    const float inv = 1.0f / (float)N;
    for (int j = tid; j < L; j += kFftThreads) {
        const float st = x[j] * inv;
        if (alpha == 1.f) dst[j] = st;
        else {
            const float s0 = pool_on_load ? pooled_at(src, L, j, g.pool_kernel, g.pool_mode) : src[j];
            dst[j] = (1.f - alpha) * s0 + alpha * st;
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

bool smooth_supported(int L) { return L >= 4 && L <= kMaxPow2L && (L & (L - 1)) == 0; }

hipError_t launch_smooth(const Geom& g, const float* in, bool pool_on_load, const int32_t* cu_seqlens,
                         const int32_t* seqlens_host, int n_items, double cutoff_frac, double alpha,
                         float* out, hipStream_t s)
{
    int max_L = 0;
    for (int i = 0; i < n_items; ++i) max_L = max(max_L, seqlens_host[i]);
    const int n_hi = (max_L >> 8) + 1;
    const size_t smem = (size_t)max_L * sizeof(float) + (size_t)(kTwLo + n_hi) * sizeof(cf);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(smooth_pow2_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(smooth_pow2_kernel, dim3(g.n_items * g.H_kv), dim3(kFftThreads), smem, s, g, in,
                       pool_on_load ? 1 : 0, cu_seqlens, cutoff_frac, (float)alpha, out);
    return hipGetLastError();
}

}  // namespace audiokv
