// After the eviction path: one decoding step on the compacted cache (paper Sec. 1 / Sec. 4.6: decoding runs on
// the retained tokens only). Every query head attends to the b_h packed rows of its KV head.
//
// Pure streaming: each K and V row is read once, so the bound is HBM. A workgroup takes one chunk of kChunk
// consecutive rows of one KV head (rows of a head are contiguous in the packed cache) and all G query heads of
// its group:
//   1. logits  Q (G x d, padded to 8 or 16 rows, stationary) times the chunk's K rows on the matrix cores
//              (16 keys per MFMA group, 16-byte loads straight from HBM into the B operand), into LDS;
//   2. softmax statistics of the chunk per query head (one wave per query head), weights back into LDS;
//   3. weights times V on the vector ALUs: a thread owns 8 channels of every (256 / (d/8))-th row, so a wave's
//      load covers whole consecutive rows; fp32 accumulators, reduced over the threads of a channel at the end.
// Chunks of a head are combined by a second small kernel (max / sum rescaling in base 2). No atomics.
// Budgets differ from head to head, so a first tiny kernel numbers the chunks of all heads consecutively; the
// grid then holds (almost) no empty workgroups, whatever the spread of the budgets.
#include "common.h"

namespace audiokv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
// rows per workgroup: as many as the weights' LDS buffer allows (8 or 16 padded query heads per KV head)
__host__ __device__ constexpr int chunk_rows(int GP) { return GP <= 8 ? 1024 : 512; }

__device__ __forceinline__ float bf16_lo(unsigned int w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return __uint_as_float(w & 0xffff0000u); }

// workspace: per (head, chunk): G * D accumulators, then G * 2 statistics (max in base-2 units, sum)
__host__ __device__ inline size_t part_stride(int G, int D) { return (size_t)G * (D + 2); }

// rows of head g that are used: its budget, cut so that nothing past total_rows is ever read
__device__ __forceinline__ int head_rows(const int32_t* __restrict__ cu_b, int g, long long total_rows) {
    const long long b0 = cu_b[g], b1 = cu_b[g + 1];
    const long long hi = b1 < total_rows ? b1 : total_rows;
    return hi > b0 ? (int)(hi - b0) : 0;
}

// first[g] = number of chunks of the heads before g (exclusive scan of ceil(rows / kChunk)); first[n_heads] = total
// table[c] = (head, first cache row, number of rows) of chunk c, so that a workgroup finds its work with one load
__global__ __launch_bounds__(1024) void decode_chunks_kernel(const int32_t* __restrict__ cu_b, int n_heads,
                                                             long long total_rows, int kChunk,
                                                             int32_t* __restrict__ first,
                                                             int4* __restrict__ table, int table_len)
{
    __shared__ int sc[1024];
    __shared__ int carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n_heads; base += 1024) {
        const int g = base + tid;
        const int mine = g < n_heads ? (head_rows(cu_b, g, total_rows) + kChunk - 1) / kChunk : 0;
        sc[tid] = mine;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            const int add = tid >= off ? sc[tid - off] : 0;
            __syncthreads();
            sc[tid] += add;
            __syncthreads();
        }
        if (g < n_heads) {
            const int f = carry + sc[tid] - mine;
            first[g] = f;
            const int rows = head_rows(cu_b, g, total_rows), b0 = cu_b[g];
            for (int c = 0; c < mine && f + c < table_len; ++c)
                table[f + c] = make_int4(g, b0 + c * kChunk, min(kChunk, rows - c * kChunk), c);
        }
        __syncthreads();
        if (tid == 1023) carry += sc[1023];
        __syncthreads();
    }
    if (tid == 0) first[n_heads] = carry;
}

template <int D, int GP>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(
    Geom g, const __bf16* __restrict__ q, const __bf16* __restrict__ kc, const __bf16* __restrict__ vc,
    const int32_t* __restrict__ first, const int4* __restrict__ table, int n_heads, float* __restrict__ part)
{
    constexpr int VPR = D / 8;                 // 16-byte pieces (lanes) per row
    constexpr int KQ = kThreads / VPR;         // rows in flight per pass of phase 3
    constexpr int KK = D / 32;                 // MFMA k-steps
    constexpr int kChunk = chunk_rows(GP);
    __shared__ __attribute__((aligned(16))) float lg[kChunk * GP];      // logits, then weights: [row][query head]
    __shared__ float st_m[GP], st_l[GP];
    __shared__ __attribute__((aligned(16))) float red[GP * D];          // accumulators summed over the waves, in wave order

    const int cid = blockIdx.x;
    if (cid >= first[n_heads]) return;         // uniform: the grid is sized from an upper bound
    const int4 job = table[cid];
    const int head = job.x, rows = job.z;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = g.G;
    const __bf16* krow0 = kc + (size_t)job.y * D;
    const __bf16* vrow0 = vc + (size_t)job.y * D;

    // ---- phase 1: logits in base-2 units ----
    {
        const int qr = lane & 15, kgrp = lane >> 4;             // A operand: query row qr, channels 8*kgrp + 32*kk
        bf16x8 qa[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            if (qr < G)
                z = *reinterpret_cast<const bf16x8*>(q + ((size_t)item * g.H_q + (size_t)h * G + qr) * D + kgrp * 8 + kk * 32);
            qa[kk] = z;
        }
        const int groups = (rows + 15) >> 4;                    // 16 keys per MFMA group
        for (int gi = wave; gi < groups; gi += 8) {             // two groups per trip: loads of both in flight
            const int gj = gi + 4;
            const int ka = min(gi * 16 + qr, rows - 1);         // B operand: key = lane & 15 (clamped, masked below)
            const int kb = min(gj * 16 + qr, rows - 1);
            bf16x8 fa[KK], fb[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                fa[kk] = *reinterpret_cast<const bf16x8*>(krow0 + (size_t)ka * D + kgrp * 8 + kk * 32);
                fb[kk] = *reinterpret_cast<const bf16x8*>(krow0 + (size_t)kb * D + kgrp * 8 + kk * 32);
            }
            f32x4 ca = {0.f, 0.f, 0.f, 0.f}, cb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                ca = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[kk], fa[kk], ca, 0, 0, 0);
                cb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[kk], fb[kk], cb, 0, 0, 0);
            }
            // result: lane holds key (lane & 15), query rows 4 * (lane >> 4) + i
            if (kgrp * 4 < GP) {
                const int keya = gi * 16 + qr, keyb = gj * 16 + qr;
                f32x4 oa, ob;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    oa[i] = keya < rows ? ca[i] * g.c_log2 : -INFINITY;
                    ob[i] = keyb < rows ? cb[i] * g.c_log2 : -INFINITY;
                }
                *reinterpret_cast<f32x4*>(&lg[keya * GP + kgrp * 4]) = oa;
                if (gj < groups) *reinterpret_cast<f32x4*>(&lg[keyb * GP + kgrp * 4]) = ob;
            }
        }
    }
    // the first V rows of phase 3 are requested now: their latency passes under the softmax statistics
    const int c8 = tid % VPR, kq = tid / VPR;
    constexpr int UN = 8;                                       // rows in flight per thread
    u32x4 vv[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
        const int rc = min(kq + u * KQ, rows - 1);
        vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vrow0 + (size_t)rc * D) + c8);
    }
    __syncthreads();

    // ---- phase 2: per query head, max and sum over the chunk; logits become weights ----
    const int rows16 = ((rows + 15) >> 4) << 4;                 // rows that phase 1 wrote (the tail holds -inf)
    for (int qh = wave; qh < GP; qh += 4) {
        if (qh < G) {
            float m = -INFINITY;
            for (int r = lane; r < rows16; r += 64) m = fmaxf(m, lg[r * GP + qh]);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
            float l = 0.f;
            for (int r = lane; r < rows16; r += 64) {
                const float p = __builtin_amdgcn_exp2f(lg[r * GP + qh] - m);
                lg[r * GP + qh] = p;
                l += p;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o, 64);
            if (lane == 0) { st_m[qh] = m; st_l[qh] = l; }
        } else {
            for (int r = lane; r < rows16; r += 64) lg[r * GP + qh] = 0.f;
        }
    }
    __syncthreads();

    // ---- phase 3: weights times V ----
    float acc[GP][8];
#pragma unroll
    for (int qh = 0; qh < GP; ++qh)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[qh][i] = 0.f;
    for (int r = kq; r < rows16; r += KQ * UN) {
        int rr[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            rr[u] = r + u * KQ;
            if (r != kq) {                                      // (the first batch is already on its way)
                const int rc = min(rr[u], rows - 1);            // clamped rows carry weight 0 (or are skipped below)
                vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vrow0 + (size_t)rc * D) + c8);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            if (rr[u] >= rows16) continue;                      // past the rows that hold weights
            float p[GP];
#pragma unroll
            for (int q4 = 0; q4 < GP / 4; ++q4) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(&lg[rr[u] * GP + q4 * 4]);
                p[q4 * 4 + 0] = t[0]; p[q4 * 4 + 1] = t[1]; p[q4 * 4 + 2] = t[2]; p[q4 * 4 + 3] = t[3];
            }
            float v[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[2 * i] = bf16_lo(vv[u][i]); v[2 * i + 1] = bf16_hi(vv[u][i]); }
#pragma unroll
            for (int qh = 0; qh < GP; ++qh)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[qh][i] = fmaf(p[qh], v[i], acc[qh][i]);
        }
    }
    // threads of one wave that share c8 (fixed order: xor tree), then the four waves through LDS, in wave order
#pragma unroll
    for (int o = VPR; o < 64; o <<= 1)
#pragma unroll
        for (int qh = 0; qh < GP; ++qh)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[qh][i] += __shfl_xor(acc[qh][i], o, 64);
    for (int w = 0; w < 4; ++w) {
        if (wave == w && lane < VPR) {
#pragma unroll
            for (int qh = 0; qh < GP; ++qh)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float* slot = &red[qh * D + c8 * 8 + i];
                    *slot = w == 0 ? acc[qh][i] : *slot + acc[qh][i];
                }
        }
        __syncthreads();
    }
    float* out = part + (size_t)cid * part_stride(G, D);
    for (int e = tid; e < G * D; e += kThreads) out[e] = red[e];
    if (tid < G) {
        out[(size_t)G * D + 2 * tid] = st_m[tid];
        out[(size_t)G * D + 2 * tid + 1] = st_l[tid];
    }
}

// one workgroup per (KV head, query head of its group): combine the chunks
__global__ __launch_bounds__(256) void decode_merge_kernel(
    Geom g, const int32_t* __restrict__ first, int grid_chunks, const float* __restrict__ part, float* __restrict__ out)
{
    const int head = blockIdx.x / g.G, qh = blockIdx.x - head * g.G;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int c0 = min(first[head], grid_chunks), c1 = min(first[head + 1], grid_chunks);
    const size_t stride = part_stride(g.G, g.D);
    const float* st0 = part + (size_t)g.G * g.D + 2 * qh;       // statistics of chunk c at st0 + c * stride
    const int nc = c1 - c0;
    float* o = out + ((size_t)item * g.H_q + (size_t)h * g.G + qh) * g.D;
    constexpr int kFast = 256;                                  // chunks whose statistics fit the LDS arrays
    __shared__ float wgt[kFast], sm[kFast], sl[kFast];
    if (nc <= kFast) {
        // chunk weights 2^(m_c - M) / sum: all statistics are fetched at once (one chunk per thread), not in a chain
        if ((int)threadIdx.x < nc) {
            sm[threadIdx.x] = st0[(c0 + threadIdx.x) * stride];
            sl[threadIdx.x] = st0[(c0 + threadIdx.x) * stride + 1];
        }
        __syncthreads();
        float M = -INFINITY;
        for (int c = 0; c < nc; ++c) M = fmaxf(M, sm[c]);
        float den = 0.f;
        for (int c = 0; c < nc; ++c) den += sl[c] * __builtin_amdgcn_exp2f(sm[c] - M);
        if ((int)threadIdx.x < nc) wgt[threadIdx.x] = __builtin_amdgcn_exp2f(sm[threadIdx.x] - M) / den;
        __syncthreads();
        for (int ch = threadIdx.x; ch < g.D; ch += blockDim.x) {
            const float* col = part + (size_t)c0 * stride + (size_t)qh * g.D + ch;
            float num = 0.f;
            int c = 0;
            for (; c + 4 <= nc; c += 4) {                       // four loads in flight; the order of the adds is fixed
                const float a0 = col[(size_t)c * stride], a1 = col[(size_t)(c + 1) * stride];
                const float a2 = col[(size_t)(c + 2) * stride], a3 = col[(size_t)(c + 3) * stride];
                num += a0 * wgt[c];
                num += a1 * wgt[c + 1];
                num += a2 * wgt[c + 2];
                num += a3 * wgt[c + 3];
            }
            for (; c < nc; ++c) num += col[(size_t)c * stride] * wgt[c];
            o[ch] = nc > 0 ? num : 0.f;
        }
        return;
    }
    // a head with more than 256 chunks (beyond a quarter of a million rows): the same sums straight from memory
    float M = -INFINITY;
    for (int c = c0; c < c1; ++c) M = fmaxf(M, st0[c * stride]);
    float den = 0.f;
    for (int c = c0; c < c1; ++c) den += st0[c * stride + 1] * __builtin_amdgcn_exp2f(st0[c * stride] - M);
    for (int ch = threadIdx.x; ch < g.D; ch += blockDim.x) {
        float num = 0.f;
        for (int c = c0; c < c1; ++c)
            num += part[c * stride + (size_t)qh * g.D + ch] * (__builtin_amdgcn_exp2f(st0[c * stride] - M) / den);
        o[ch] = num;
    }
}

}  // namespace

bool decode_supported(int G) { return G >= 1 && G <= 16; }

// upper bound on the number of chunks: every head wastes less than one
static size_t chunk_bound(const Geom& g, long long total_rows) {
    return (size_t)(total_rows / chunk_rows(g.G)) + (size_t)g.n_items * g.H_kv;
}
static size_t first_bytes(const Geom& g) { return (((size_t)g.n_items * g.H_kv + 1) * sizeof(int32_t) + 255) & ~(size_t)255; }
static size_t table_bytes(size_t bound) { return (bound * sizeof(int4) + 255) & ~(size_t)255; }

size_t decode_workspace_bytes(const Geom& g, long long total_rows) {
    const size_t bound = chunk_bound(g, total_rows);
    return first_bytes(g) + table_bytes(bound) + bound * part_stride(g.G, g.D) * sizeof(float);
}

hipError_t launch_decode(const Geom& g, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* cu_budgets, long long total_rows, float* out, void* workspace, hipStream_t s)
{
    const int n_heads = g.n_items * g.H_kv;
    const size_t bound = chunk_bound(g, total_rows);
    if (total_rows < 0 || bound > (size_t)INT32_MAX || !decode_supported(g.G)) return hipErrorInvalidValue;
    int32_t* first = static_cast<int32_t*>(workspace);
    int4* table = reinterpret_cast<int4*>(static_cast<char*>(workspace) + first_bytes(g));
    float* part = reinterpret_cast<float*>(static_cast<char*>(workspace) + first_bytes(g) + table_bytes(bound));
    hipLaunchKernelGGL(decode_chunks_kernel, dim3(1), dim3(1024), 0, s, cu_budgets, n_heads, total_rows,
                       chunk_rows(g.G), first, table, (int)bound);
    const dim3 grid((unsigned)bound);
#define AUDIOKV_LAUNCH_DECODE(DD, GG)                                                                           \
    hipLaunchKernelGGL((decode_partial_kernel<DD, GG>), grid, dim3(kThreads), 0, s, g, (const __bf16*)q,       \
                       (const __bf16*)k_cache, (const __bf16*)v_cache, (const int32_t*)first,                  \
                       (const int4*)table, n_heads, part)
    const bool wide = g.G > 8;
    switch (g.D) {
        case 64:  if (wide) AUDIOKV_LAUNCH_DECODE(64, 16);  else AUDIOKV_LAUNCH_DECODE(64, 8);  break;
        case 128: if (wide) AUDIOKV_LAUNCH_DECODE(128, 16); else AUDIOKV_LAUNCH_DECODE(128, 8); break;
        case 256: if (wide) AUDIOKV_LAUNCH_DECODE(256, 16); else AUDIOKV_LAUNCH_DECODE(256, 8); break;
        default: return hipErrorInvalidValue;
    }
#undef AUDIOKV_LAUNCH_DECODE
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)(n_heads * g.G)), dim3(256), 0, s, g,
                       (const int32_t*)first, (int)bound, (const float*)part, out);
    return hipGetLastError();
}

}  // namespace audiokv
