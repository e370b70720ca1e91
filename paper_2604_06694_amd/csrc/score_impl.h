// Stage 1: observation-window importance (paper Sec. 3.3: the per-head
// importance sequence s; the last W queries attend to all L keys).
//
//   raw[h, j] = sum over rows r = (query head of the group, window row) of
//               softmax_j(scale * <q_r, k_j>)
//
// The contraction (G*W rows) x (L keys) x d is dense, so it runs on bf16 MFMA
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate). A softmax row needs its max and
// its sum over ALL keys before any column sum can be formed, so the work is
// two sweeps over K with the same tiling:
//   sweep 1: logits tile -> running (max, sum of exp) per row, per key range
//   sweep 2: logits tile -> exp2(z - max - log2 sum) summed over rows, per key
// Keeping logits instead would cost G*W*4 bytes per token and head against the
// d*2 bytes of the key itself, so recomputing is the cheaper choice.
//
// Tiling. A workgroup (4 waves) owns one KV head and a range of key tiles. The
// window queries are the stationary MFMA operand: each wave keeps NB blocks of
// 16 rows in registers for the whole kernel (WR waves split the rows, the
// other 4/WR split the keys of a tile). K tiles are read from HBM once per
// sweep with 16-byte coalesced loads, staged in LDS, and each wave pulls the
// 16-key x 32-channel fragments it needs. Sweep 1 uses C = K Q^T (a lane owns
// one query row, so max/sum stay in the lane); sweep 2 uses C = Q K^T (a lane
// owns one key, so the column sum stays in the lane). Both orientations use
// the same register fragments: only the operand order of the MFMA differs.
//
// Everything is in base-2 units: z2 = <q,k> * scale * log2(e).
#pragma once

#include "common.h"

namespace audiokv {
namespace score_detail {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;

template <int D, int NB, int WR>
struct Tile {
    static constexpr int WK = 4 / WR;                 // waves splitting the keys of a tile
    static constexpr int KB = (D == 256) ? 2 : 4;     // 16-key blocks per wave per tile
    static constexpr int KW = 16 * KB;                // keys per wave per tile
    static constexpr int TK = KW * WK;                // keys per workgroup tile
    static constexpr int KK = D / 32;                 // MFMA k-steps per logit
    static constexpr int ROWS = NB * 16 * WR;         // padded window rows per head
    static constexpr int ROW_BYTES = D * 2 + 16;      // LDS row pitch (16 B pad: conflict-free fragment reads)
    static constexpr int CHUNKS = TK * D / 8;         // 16-byte pieces per tile
    static constexpr int CH = CHUNKS / kThreads;      // pieces per thread
    static_assert(CHUNKS % kThreads == 0, "tile must split evenly over the workgroup");
    static constexpr int LDS_K = TK * ROW_BYTES;
    static constexpr int LDS_BYTES = LDS_K + ROWS * 8 + WR * TK * 4;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m, l) <- merge of two partial softmax statistics in raw-logit units (c > 0 converts to base 2)
__device__ __forceinline__ void merge_stats(float& m, float& l, float m2, float l2, float c) {
    const float M = fmaxf(m, m2);
    const float Ms = (M == -INFINITY) ? 0.f : M;
    l = l * fast_exp2((m - Ms) * c) + l2 * fast_exp2((m2 - Ms) * c);
    m = M;
}

template <int D, int NB, int WR, bool SWEEP2>
__global__ __launch_bounds__(kThreads) void score_kernel(
    Geom g, const __bf16* __restrict__ q_win, const __bf16* __restrict__ k,
    const int32_t* __restrict__ cu_seq, int nsplit,
    float* __restrict__ stats,      // [head][split][ROWS][2] : (max in base-2 units, sum of exp2)
    float* __restrict__ raw)        // sweep 2 output, packed like scores
{
    using T = Tile<D, NB, WR>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char* lds_k = lds;
    float* lds_rows = reinterpret_cast<float*>(lds + T::LDS_K);            // ROWS * 2 floats
    float* lds_cols = lds_rows + T::ROWS * 2;                              // WR * TK floats

    const int head = blockIdx.x / nsplit;
    const int split = blockIdx.x - head * nsplit;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const int R = g.G * g.W;                          // real window rows of this head
    const float c = g.c_log2;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave % WR, wk = wave / WR;
    const int l16 = lane & 15, lg = lane >> 4;
    const int row0 = wr * NB * 16;

    const int n_tiles = (L + T::TK - 1) / T::TK;
    const int tps = (n_tiles + nsplit - 1) / nsplit;
    const int t_begin = split * tps;
    const int t_end = min(n_tiles, t_begin + tps);
    float* my_stats = stats + ((size_t)head * nsplit + split) * T::ROWS * 2;

    if (t_begin >= t_end) {                           // uniform over the workgroup
        if (!SWEEP2)
            for (int r = tid; r < T::ROWS; r += kThreads) { my_stats[2 * r] = -INFINITY; my_stats[2 * r + 1] = 0.f; }
        return;
    }

    // ---- stationary operand: this wave's window queries, as MFMA fragments --------------------
    // fragment (rb, kk): lane holds row rb*16 + l16, channels kk*32 + lg*8 .. +8
    bf16x8 qf[NB][T::KK];
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
        const int r = row0 + rb * 16 + l16;
        const bool live = r < R;
        const int qh = live ? r / g.W : 0, wrow = live ? r - qh * g.W : 0;
        const __bf16* src = q_win + (((size_t)item * g.H_q + (size_t)h * g.G + qh) * g.W + wrow) * D + lg * 8;
#pragma unroll
        for (int kk = 0; kk < T::KK; ++kk) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (live) v = *reinterpret_cast<const bf16x8*>(src + kk * 32);
            qf[rb][kk] = v;
        }
    }

    // ---- sweep 2 needs each row's final max + log2(sum): merge the per-range partials -----------
    if (SWEEP2) {
        const float* hs = stats + (size_t)head * nsplit * T::ROWS * 2;
        for (int r = tid; r < T::ROWS; r += kThreads) {
            float cst = INFINITY;                     // padded rows: exp2(z - inf) = 0, they add nothing
            if (r < R) {
                float M = -INFINITY;
                for (int s = 0; s < nsplit; ++s) M = fmaxf(M, hs[((size_t)s * T::ROWS + r) * 2]);
                float Z = 0.f;
                for (int s = 0; s < nsplit; ++s) {
                    const float ms = hs[((size_t)s * T::ROWS + r) * 2], ls = hs[((size_t)s * T::ROWS + r) * 2 + 1];
                    if (ls > 0.f) Z += ls * fast_exp2(ms - M);
                }
                cst = M + __log2f(Z);
            }
            lds_rows[r] = cst;
        }
    }

    // sweep 1 state: running max (raw logit units) and sum for row rb*16 + l16, over this lane's keys
    float run_m[NB], run_l[NB];
    int last_vis[NB];                                  // last key index the lane's row may see (sweep 1)
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
        run_m[rb] = -INFINITY;
        run_l[rb] = 0.f;
        const int r = row0 + rb * 16 + l16;
        last_vis[rb] = (r < R) ? (g.causal ? (L - g.W + (r % g.W)) : (L - 1)) : -1;
    }

    // ---- K tile staging: global -> registers (next tile) -> LDS -> MFMA fragments ----------------
    uint4 stage[T::CH];
    auto load_tile = [&](int t) {
        const int j0 = t * T::TK;
#pragma unroll
        for (int it = 0; it < T::CH; ++it) {
            const int cidx = tid + it * kThreads;
            const int key = cidx / (D / 8), part = cidx - key * (D / 8);
            const int j = j0 + key;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (j < L) v = *reinterpret_cast<const uint4*>(k + kv_row_offset(g, tok0, L, h, j) + part * 8);
            stage[it] = v;
        }
    };
    load_tile(t_begin);

    for (int t = t_begin; t < t_end; ++t) {
        const int j0 = t * T::TK;
#pragma unroll
        for (int it = 0; it < T::CH; ++it) {
            const int cidx = tid + it * kThreads;
            const int key = cidx / (D / 8), part = cidx - key * (D / 8);
            *reinterpret_cast<uint4*>(lds_k + key * T::ROW_BYTES + part * 16) = stage[it];
        }
        __syncthreads();

        bf16x8 kf[T::KB][T::KK];                       // fragment: key kb*16 + l16, channels kk*32 + lg*8 .. +8
#pragma unroll
        for (int kb = 0; kb < T::KB; ++kb)
#pragma unroll
            for (int kk = 0; kk < T::KK; ++kk)
                kf[kb][kk] = *reinterpret_cast<const bf16x8*>(
                    lds_k + (wk * T::KW + kb * 16 + l16) * T::ROW_BYTES + (kk * 32 + lg * 8) * 2);

        if (t + 1 < t_end) load_tile(t + 1);           // in flight while this tile is computed
        __syncthreads();                               // every wave holds its fragments: the LDS tile is free

        const int jw0 = j0 + wk * T::KW;               // first key of this wave's part of the tile
        // does any (row, key) pair of this tile need the visibility test?
        const bool masked = g.causal ? (j0 + T::TK - 1 > L - g.W) : (j0 + T::TK > L);

        if (!SWEEP2) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) {
                f32x4 acc[T::KB];
#pragma unroll
                for (int kb = 0; kb < T::KB; ++kb) acc[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < T::KK; ++kk)
#pragma unroll
                    for (int kb = 0; kb < T::KB; ++kb)    // C[key][row]: lane = row l16, keys 4*lg + i
                        acc[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][kk], qf[rb][kk], acc[kb], 0, 0, 0);
                if (masked) {
#pragma unroll
                    for (int kb = 0; kb < T::KB; ++kb)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (jw0 + kb * 16 + 4 * lg + i > last_vis[rb]) acc[kb][i] = -INFINITY;
                }
                float mx = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < T::KB; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mx = fmaxf(mx, acc[kb][i]);
                const float m_new = fmaxf(run_m[rb], mx);
                const float ms = (m_new == -INFINITY) ? 0.f : m_new;
                const float msc = ms * c;
                float sum = 0.f;
#pragma unroll
                for (int kb = 0; kb < T::KB; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) sum += fast_exp2(fmaf(acc[kb][i], c, -msc));
                run_l[rb] = run_l[rb] * fast_exp2((run_m[rb] - ms) * c) + sum;
                run_m[rb] = m_new;
            }
        } else {
            float colsum[T::KB];
#pragma unroll
            for (int kb = 0; kb < T::KB; ++kb) colsum[kb] = 0.f;
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) {
                f32x4 acc[T::KB];
#pragma unroll
                for (int kb = 0; kb < T::KB; ++kb) acc[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < T::KK; ++kk)
#pragma unroll
                    for (int kb = 0; kb < T::KB; ++kb)    // C[row][key]: lane = key l16, rows 4*lg + i
                        acc[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[rb][kk], kf[kb][kk], acc[kb], 0, 0, 0);
                const f32x4 cst = *reinterpret_cast<const f32x4*>(lds_rows + row0 + rb * 16 + 4 * lg);
                if (masked) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = row0 + rb * 16 + 4 * lg + i;
                        const int lv = (r < R) ? (g.causal ? (L - g.W + (r % g.W)) : (L - 1)) : -1;
#pragma unroll
                        for (int kb = 0; kb < T::KB; ++kb)
                            if (jw0 + kb * 16 + l16 > lv) acc[kb][i] = -INFINITY;
                    }
                }
#pragma unroll
                for (int kb = 0; kb < T::KB; ++kb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) colsum[kb] += fast_exp2(fmaf(acc[kb][i], c, -cst[i]));
            }
            // rows of the other lane groups, then rows of the other waves (fixed order: deterministic)
#pragma unroll
            for (int kb = 0; kb < T::KB; ++kb) {
                float v = colsum[kb];
                v += __shfl_xor(v, 16, 64);
                v += __shfl_xor(v, 32, 64);
                if (lg == 0) lds_cols[wr * T::TK + wk * T::KW + kb * 16 + l16] = v;
            }
            __syncthreads();
            if (tid < T::TK && j0 + tid < L) {
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < WR; ++w) v += lds_cols[w * T::TK + tid];
                raw[(size_t)tok0 * g.H_kv + (size_t)h * L + j0 + tid] = v;
            }
        }
    }

    if (!SWEEP2) {
        // a row's keys are spread over the 4 lane groups of a wave and over the WK key-splitting waves
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                const float m2 = __shfl_xor(run_m[rb], o, 64), l2 = __shfl_xor(run_l[rb], o, 64);
                merge_stats(run_m[rb], run_l[rb], m2, l2, c);
            }
        }
        if (T::WK == 2) {
            __syncthreads();                            // lds_rows is not in use by anyone in sweep 1
            if (wk == 1 && lg == 0) {
#pragma unroll
                for (int rb = 0; rb < NB; ++rb) {
                    lds_rows[2 * (row0 + rb * 16 + l16)] = run_m[rb];
                    lds_rows[2 * (row0 + rb * 16 + l16) + 1] = run_l[rb];
                }
            }
            __syncthreads();
            if (wk == 0 && lg == 0) {
#pragma unroll
                for (int rb = 0; rb < NB; ++rb)
                    merge_stats(run_m[rb], run_l[rb], lds_rows[2 * (row0 + rb * 16 + l16)],
                                lds_rows[2 * (row0 + rb * 16 + l16) + 1], c);
            }
        }
        if (wk == 0 && lg == 0) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) {
                const int r = row0 + rb * 16 + l16;
                my_stats[2 * r] = (run_m[rb] == -INFINITY) ? -INFINITY : run_m[rb] * c;
                my_stats[2 * r + 1] = run_l[rb];
            }
        }
    }
}

template <int D, int NB, int WR>
hipError_t launch_both_sweeps(const Geom& g, const void* q_win, const void* k, const int32_t* cu_seq,
                              int nsplit, float* stats, float* raw, hipStream_t s, hipEvent_t between)
{
    using T = Tile<D, NB, WR>;
    const int n_heads = g.n_items * g.H_kv;
    const dim3 grid((unsigned)(n_heads * nsplit));
    static bool attr_set = false;
    if (!attr_set && T::LDS_BYTES > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_kernel<D, NB, WR, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_kernel<D, NB, WR, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((score_kernel<D, NB, WR, false>), grid, dim3(kThreads), T::LDS_BYTES, s, g,
                       (const __bf16*)q_win, (const __bf16*)k, cu_seq, nsplit, stats, raw);
    if (between) {
        const hipError_t e = hipEventRecord(between, s);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((score_kernel<D, NB, WR, true>), grid, dim3(kThreads), T::LDS_BYTES, s, g,
                       (const __bf16*)q_win, (const __bf16*)k, cu_seq, nsplit, stats, raw);
    return hipGetLastError();
}

}  // namespace score_detail

// one translation unit per head_dim keeps the build parallel
hipError_t launch_score_d64(const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, float* stats, float* raw, hipStream_t s, hipEvent_t between);
hipError_t launch_score_d128(const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, float* stats, float* raw, hipStream_t s, hipEvent_t between);
hipError_t launch_score_d256(const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, float* stats, float* raw, hipStream_t s, hipEvent_t between);

}  // namespace audiokv
