// Stage 1: observation-window importance (paper Sec. 3.3: the per-head
// importance sequence s; the last W queries attend to all L keys).
//
//   raw[h, j] = sum over rows r = (query head of the group, window row) of
//               softmax_j(scale * <q_r, k_j>)
//
// The contraction (G*W rows) x (L keys) x d is dense, so it runs on bf16 MFMA
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate). A softmax row needs its max and
// its sum over ALL keys before any column sum can be formed, so the work is
// two sweeps over K with the same tiling, and a tiny merge in between:
//   sweep 1: logits tile -> running (max, sum of exp) per row, per key range
//   merge  : per row, max + log2(sum) over the key ranges
//   sweep 2: logits tile -> exp2(z - max - log2 sum) summed over rows, per key
// Keeping logits instead would cost G*W*4 bytes per token and head against the
// d*2 bytes of the key itself, so recomputing is the cheaper choice.
//
// Both sweeps are bound by the vector ALU next to the matrix pipe: each logit
// costs one MFMA-lane-slot plus (fma, exp2, add); measured on gfx950 a plain
// vector op takes 4 issue cycles of a SIMD, an exp2 about 8.5, an MFMA issue
// about 8 (its 32 cycles on the matrix pipe run beside the vector work). The
// 32x32x16 shape is used because one MFMA issue then covers twice as many
// logits as 16x16x32, which leaves more issue slots in which the vector work
// of the previous block hides.
//
// Tiling. A workgroup of WR compute waves plus one loader wave owns one KV head
// and a range of key tiles. The window queries are the stationary MFMA operand:
// compute wave w keeps rows [w*NB*32, (w+1)*NB*32) as register fragments for
// the whole kernel. K tiles (64 keys, or 32 at d = 256) are read from HBM once
// per sweep by the loader wave (16-byte load-to-LDS instructions that go from
// HBM straight into a ring of three or four LDS buffers, two or three tiles
// ahead of the compute waves, one barrier per tile), so the HBM latency is paid
// by a wave that has nothing else to do and no wave holds staging registers.
// Every compute wave pulls all 32-key x 16-channel fragments of the tile.
// Sweep 1 keeps no running maximum: its exponentials are taken against a fixed
// reference (the maximum of the wave's first block) and only a block whose sum
// leaves the safe range is redone against a new reference. Sweep 1 computes
// C = K Q^T (a lane owns one query row, so max/sum stay in the lane); sweep 2
// computes C = Q K^T (a lane owns one key, so the column sum stays in the
// lane). Both orientations use the same register fragments: only the operand
// order of the MFMA differs. Only the last tiles of a head contain keys that
// some window row may not see; they take a separate, masked instantiation of
// the tile body so that the common path carries no compare/select work.
//
// Everything is in base-2 units: z2 = <q,k> * scale * log2(e).
#pragma once

#include <atomic>
#include <type_traits>
#include <utility>

#include "common.h"

#ifndef AUDIOKV_SCORE_KB
#define AUDIOKV_SCORE_KB 2
#endif

namespace audiokv {
namespace score_detail {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int D, int NB, int WR>
struct Tile {
    static constexpr int THREADS = 64 * (WR + 1);      // WR compute waves + 1 loader wave
    static constexpr int KB = (D == 256) ? 1 : AUDIOKV_SCORE_KB;   // 32-key blocks per tile
    static constexpr int TK = 32 * KB;                // keys per tile
    static constexpr int KK = D / 16;                 // MFMA k-steps per logit
    static constexpr int ROWS = NB * 32 * WR;         // padded window rows per head
    // LDS rows are unpadded; the 16-byte chunk c of key row r sits at chunk slot (c + r) mod 8 of its group of eight
    // slots. That is bank for bank what a row pitch of d*2 + 16 bytes gives (slot s starts at bank 4 s mod 32), the
    // layout under which the fragment reads (32 rows, same chunk) measure no bank conflict, while a wave-wide
    // load-to-LDS instruction, which can only fill 1 KiB of consecutive LDS bytes, still deposits whole rows.
    // (The bank-conflict counter still reads about 28 cycles per load-to-LDS instruction, whichever way the slots
    // are permuted: that is how the incoming 1 KiB is written, not the fragment reads.)
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;              // rows per wave-wide load instruction
    static_assert(64 % CPR == 0 && CPR >= 8, "a wave-wide load covers whole rows of at least 8 chunks");
    static constexpr int CHUNKS = TK * D / 8;         // 16-byte pieces per tile
    static constexpr int CH = CHUNKS / 64;            // load instructions per tile
    static_assert(CHUNKS % 64 == 0, "a tile is a whole number of wave-wide 16-byte loads");
    // LDS ring: the loader wave requests tile t + AHEAD while tile t is consumed, straight from HBM into the ring
    // (no staging registers), so AHEAD - 1 whole tiles are in flight across every barrier. Workgroups of one or two
    // compute waves keep a shorter ring: there the number of resident workgroups matters more.
    static constexpr int STAGES = (WR >= 4) ? 4 : 3;
    static constexpr int AHEAD = STAGES - 1;
    static_assert((AHEAD - 1) * CH <= 63, "the outstanding loads must fit the vmcnt field");
    static constexpr int LDS_K = TK * ROW_BYTES;      // one K buffer
    static constexpr int LDS_COLS = WR * TK * 4;      // one column-sum exchange buffer
    static constexpr int LDS_RC = ROWS * 4;           // sweep 2: per-row normalisation constants
    static constexpr int LDS_BYTES = STAGES * LDS_K + 3 * LDS_COLS + LDS_RC;
    static constexpr int FLUSH_WAVE = (WR - 1 < 3) ? WR - 1 : 3;   // the compute wave that stores the column sums
    // chunk slot of chunk c of tile row r, and the chunk that slot s of row r holds
    __host__ __device__ static constexpr int slot_of_chunk(int c, int r) { return (c & ~7) | ((c + r) & 7); }
    __host__ __device__ static constexpr int chunk_in_slot(int s, int r) { return (s & ~7) | ((s - r) & 7); }
};

// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding and for nothing else
// (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int vmcnt_only(int n) { return (n & 15) | (((n >> 4) & 3) << 14) | (7 << 4) | (15 << 8); }

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m, l) <- merge of two partial softmax statistics (m in base-2 units)
__device__ __forceinline__ void merge_stats(float& m, float& l, float m2, float l2) {
    const float M = fmaxf(m, m2);
    const float Ms = (M == -INFINITY) ? 0.f : M;
    l = l * fast_exp2(m - Ms) + l2 * fast_exp2(m2 - Ms);
    m = M;
}

// last key index that window row r may attend to (-1: padded row, sees nothing)
__device__ __forceinline__ int last_visible(const Geom& g, int L, int R, int r) {
    return (r < R) ? (g.causal ? (L - g.W + (r % g.W)) : (L - 1)) : -1;
}

// Row (sweep 2) or key (sweep 1) offset inside a 32x32 MFMA result block of element i (0..15) for lane half g2.
__device__ __forceinline__ constexpr int c_row(int i, int g2) { return (i >> 2) * 8 + g2 * 4 + (i & 3); }

template <int D, int NB, int WR, bool SWEEP2>
__global__ __launch_bounds__(64 * (WR + 1), (NB == 1 && D <= 128) ? 4 : 2) void score_kernel(
    Geom g, const __bf16* __restrict__ q_win, const __bf16* __restrict__ k,
    const int32_t* __restrict__ cu_seq, int nsplit,
    int rows_pad,                     // row pitch of stats / cst (>= ROWS: the two sweeps may tile the rows differently)
    int row_base,                     // first window row of this launch (sweep 2 may cover the rows in two launches)
    float* __restrict__ stats,        // sweep 1 out: [head][split][rows_pad][2] = (max in base-2 units, sum of exp2)
    const float* __restrict__ cst,    // sweep 2 in : [head][rows_pad] = max + log2(sum), +inf for padded rows
    float* __restrict__ raw)          // sweep 2 out, packed like scores
{
    using T = Tile<D, NB, WR>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    float* lds_cols = reinterpret_cast<float*>(lds + T::STAGES * T::LDS_K);
    float* lds_rc = reinterpret_cast<float*>(lds + T::STAGES * T::LDS_K + 3 * T::LDS_COLS);

    // Workgroups go to the 8 XCDs round-robin by index, and each XCD has its own L2. All key-range splits of a head
    // are therefore given indices with the same residue mod 8, so that the head's window queries (and the tile
    // shared by neighbouring splits) are fetched from HBM by one L2 only.
    int head, split;
    {
        const int n_heads = gridDim.x / nsplit;
        const int full = n_heads & ~7;                  // heads that fill whole groups of 8
        const int bid = blockIdx.x;
        if (bid < full * nsplit) {
            const int q = bid >> 3;
            split = q % nsplit;
            head = (q / nsplit) * 8 + (bid & 7);
        } else {
            const int r = bid - full * nsplit;
            head = full + r / nsplit;
            split = r - (r / nsplit) * nsplit;
        }
    }
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const int R = g.G * g.W;                          // real window rows of this head
    const float c = g.c_log2;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g2 = lane >> 5;
    const int row0 = wave * NB * 32;                  // first row of this wave inside the launch's row range
    const int rowg0 = row_base + row0;                // the same as a window row of the head

    const int n_tiles = (L + T::TK - 1) / T::TK;
    const int tps = (n_tiles + nsplit - 1) / nsplit;
    const int t_begin = split * tps;
    const int t_end = min(n_tiles, t_begin + tps);

    const int n_loc = t_end - t_begin;                  // tiles of this workgroup
    if (t_begin >= t_end) {                           // uniform over the workgroup
        if (!SWEEP2) {
            float* my_stats = stats + ((size_t)head * nsplit + split) * rows_pad * 2;
            for (int r = tid; r < T::ROWS; r += T::THREADS) { my_stats[2 * r] = -INFINITY; my_stats[2 * r + 1] = 0.f; }
        }
        return;
    }

    // sweep 2: add the WR waves' partial column sums of the tile starting at j0 (fixed order) and store them
    auto flush_cols = [&](int buf, int j0) {
        // (the lane index passes through an empty asm so that the addresses are formed here, once per tile, instead
        // of living in registers across the whole tile loop)
        int lane_here = lane;
#if defined(__HIP_DEVICE_COMPILE__)
        asm volatile("" : "+v"(lane_here));
#endif
#pragma unroll
        for (int cc = 0; cc < T::TK; cc += 64) {
            const int col = cc + lane_here;
            if (col < T::TK && j0 + col < L) {
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < WR; ++w) v += lds_cols[buf * (WR * T::TK) + w * T::TK + col];
                raw[(size_t)tok0 * g.H_kv + (size_t)h * L + j0 + col] = v;
            }
        }
    };

    // Workgroup barrier that orders LDS traffic only: the waves exchange nothing through global memory, and a wave's
    // outstanding global loads or stores are no reason to hold the others up.
    auto wg_barrier = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };
    // sweep 2: one compute wave stores the column sums of tile t once the barrier that ended tile t has passed
    auto flush_tile = [&](int t_) {
        if (SWEEP2 && wave == T::FLUSH_WAVE) flush_cols((t_ - t_begin) % 3, t_ * T::TK);
    };

    if (wave == WR) {
        // ================= loader wave: HBM -> LDS ring, AHEAD tiles ahead =================
        // Every instruction moves 64 x 16 bytes from per-lane global addresses to 1 KiB of consecutive LDS bytes
        // (global_load_lds_dwordx4): lane l fills chunk slot l % CPR of row l / CPR of the instruction's RPI rows,
        // so it fetches the chunk that belongs in that slot. Rows past the end are clamped to the last
        // row, never zero-filled: every tile that reaches past L - W is a masked tile, and the masked path
        // discards those logits.
        const int lrow = lane / T::CPR, pslot = lane % T::CPR;
        const int64_t row_elems = kv_tok_stride(g);
        const __bf16* head_base = k + kv_row_offset(g, item, tok0, L, h, 0);
        // byte offset of this lane's chunk inside the RPI rows of instruction `it`, for it & 3 (the slot rotation
        // repeats every 8 rows): a 32-bit lane offset on top of a uniform 64-bit base keeps the address arithmetic scalar
        unsigned lane_off[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
            lane_off[v] = (unsigned)(((int64_t)lrow * row_elems + T::chunk_in_slot(pslot, v * T::RPI + lrow) * 8) * 2);
        auto issue_tile = [&](int lt) {                 // workgroup-local tile index; past the end: the last tile again,
            const int t_ = t_begin + min(lt, n_loc - 1);   // into a slot whose tile has been consumed
            unsigned char* dst = lds + (lt % T::STAGES) * T::LDS_K;
            if ((t_ + 1) * T::TK <= L) {
                const char* tile_base = reinterpret_cast<const char*>(head_base + (int64_t)t_ * T::TK * row_elems);
#pragma unroll
                for (int it = 0; it < T::CH; ++it)
                    __builtin_amdgcn_global_load_lds(
                        (global_void_ptr)(tile_base + (int64_t)it * T::RPI * row_elems * 2 + lane_off[it & 3]),
                        (lds_void_ptr)(dst + it * 1024), 16, 0, 0);
            } else {
#pragma unroll
                for (int it = 0; it < T::CH; ++it) {
                    const int r_ = it * T::RPI + lrow;
                    const int j_ = min(t_ * T::TK + r_, L - 1);
                    __builtin_amdgcn_global_load_lds(
                        (global_void_ptr)(k + kv_row_offset(g, item, tok0, L, h, j_) + T::chunk_in_slot(pslot, r_) * 8),
                        (lds_void_ptr)(dst + it * 1024), 16, 0, 0);
                }
            }
        };
        // Loads complete in the order they were issued, so "at most (AHEAD - 1) tiles' worth outstanding" means
        // that the oldest tile in flight has landed; the barrier then hands it to the compute waves. (These are the
        // only vector-memory operations of this wave.)
        auto tile_landed_then_barrier = [&]() {
            __builtin_amdgcn_s_waitcnt(vmcnt_only((T::AHEAD - 1) * T::CH));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
        };
#pragma unroll
        for (int a = 0; a < T::AHEAD; ++a) issue_tile(a);
        tile_landed_then_barrier();                     // tile 0 is in the ring
#pragma unroll 1
        for (int lt = 0; lt < n_loc; ++lt) {
            // slot (lt + AHEAD) % STAGES held tile lt - 1, which every wave left at the barrier that ended it
            issue_tile(lt + T::AHEAD);
            tile_landed_then_barrier();                 // tile lt + 1 is in the ring; ends iteration lt
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));      // nothing may still be writing LDS when the wave ends
        return;
    }

    // ================= compute waves =================
    // stationary operand: this wave's window queries, as MFMA fragments
    // fragment (rb, kk): lane holds row row0 + rb*32 + l32, channels kk*16 + g2*8 .. +8
    bf16x8 qf[NB][T::KK];
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
        const int r = rowg0 + rb * 32 + l32;
        const bool live = r < R;
        const int qh = live ? r / g.W : 0, wrow = live ? r - qh * g.W : 0;
        const __bf16* src = q_win + (((size_t)item * g.H_q + (size_t)h * g.G + qh) * g.W + wrow) * D + g2 * 8;
#pragma unroll
        for (int kk = 0; kk < T::KK; ++kk) {
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (live) v = *reinterpret_cast<const bf16x8*>(src + kk * 16);
            qf[rb][kk] = v;
        }
    }
    if (SWEEP2)
        for (int r = tid; r < T::ROWS; r += 64 * WR)
            lds_rc[r] = row_base + r < rows_pad ? cst[(size_t)head * rows_pad + row_base + r] : INFINITY;

    // sweep 1: reference (base-2 units: logit * c) and sum of exp2(logit * c - reference) for row
    // row0 + rb*32 + l32 over this lane's keys. The reference is a logit that the row has met, not its running
    // maximum: softmax statistics are shift-invariant, and fp32 leaves more than a hundred binary orders between a
    // term of 1 and overflow. It is raised only when a block's terms grow past 2^64 (see reduce_end), so the common
    // path spends no vector work on maxima or on rescaling the sum. -inf: the lane has not seen a visible key yet.
    float run_m[NB], run_l[NB];
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) { run_m[rb] = -INFINITY; run_l[rb] = 0.f; }

    // The unit of work is a block: this wave's NB*32 rows x 32 keys (NB MFMA result tiles, KK MFMAs each). Its
    // logits then need the sweep's vector work (fma, exp2, add per logit), which costs about as much ALU time as
    // the MFMAs cost matrix-pipe time. The two are software-pipelined inside the wave: while the MFMAs of block
    // b + 1 accumulate into one register set, the reduction of block b runs on the other, interleaved k-step by
    // k-step (one MFMA per row tile, then one eighth of the reduction), so the ALU work sits in the shadow of the
    // matrix pipe. K fragments come from LDS through a small register ring, PF k-steps ahead, and the stream
    // runs on into the next block, whose tile is already in the LDS ring.
    constexpr int PF = 2;                               // fragment prefetch distance (k-steps)
    constexpr int RING = 4;
    static_assert(T::KK % RING == 0 && PF < RING, "the fragment ring must line up across blocks");
    constexpr int SLICE = 16 / (T::KK < 16 ? T::KK : 16);   // result elements reduced per k-step (per row tile)
    static_assert(T::KK <= 16 ? (SLICE * T::KK == 16) : true, "reduction slices must cover the 16 elements");
    f32x16 acc0[NB], acc1[NB];
    bf16x8 kfr[RING];
    // byte offset of chunk 2 kk + g2 of key row l32 (of any 32-key block: their first rows are multiples of 8) in its
    // rotated slot, for kk & 3; chunks 8 and up only add whole groups of 8 chunk slots
    int frag_off[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) frag_off[v] = l32 * T::ROW_BYTES + T::slot_of_chunk((2 * v) | g2, l32) * 16;
    auto frag_load = [&](int slot, int kb, int kk, int ring) {   // keys kb*32 + l32, channels kk*16 + g2*8 .. +8
        kfr[ring] = *reinterpret_cast<const bf16x8*>(lds + slot * T::LDS_K + kb * 32 * T::ROW_BYTES + frag_off[kk & 3] +
                                                     (kk >> 2) * 128);
    };

    // --- reduction of one block, cut into KK slices -------------------------------------------------------------
    float red_c[NB];                                    // sweep 1: the reference in use (run_m, or 0 while that is -inf)
    float red_s[2];                                     // partial sums of row tile 0 (two chains)
    float red_t[NB];                                    // sweep 1: partial sums of row tiles 1.. (slot 0 unused)
    // sweep 2: a lane always meets the same 16 rows of a row tile (c_row(i, g2)), so their constants stay in registers
    float rcv[NB][16];
    // The scale is read through this copy. The empty asm statements in run_block take it as an in/out operand, which
    // ties every slice of vector work to its place between two MFMAs (see there).
    float c_pin = c;
    // sweep 1, first block of a workgroup's plain tiles: take the reference from the logits themselves
    auto reference_from = [&](f32x16 (&a)[NB]) {
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            float mx = a[rb][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, a[rb][i]);
            run_m[rb] = mx * c;                         // c > 0: the scaled maximum is the maximum of the scaled logits
            red_c[rb] = run_m[rb];
        }
    };
    auto reduce_begin = [&](auto masked_tag, f32x16 (&a)[NB], int j0b) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        red_s[0] = red_s[1] = 0.f;
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) red_t[rb] = 0.f;
        if (!SWEEP2) {
            if (MASKED) {
                // tiles with invisible (row, key) pairs: plain running-maximum bookkeeping (a few tiles per head)
#pragma unroll
                for (int rb = 0; rb < NB; ++rb) {
                    const int lv = last_visible(g, L, R, rowg0 + rb * 32 + l32);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (j0b + c_row(i, g2) > lv) a[rb][i] = -INFINITY;
                    float mx = a[rb][0];
#pragma unroll
                    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, a[rb][i]);
                    const float m_new = fmaxf(run_m[rb], mx * c);
                    const float ms = (m_new == -INFINITY) ? 0.f : m_new;
                    run_l[rb] *= fast_exp2(run_m[rb] - ms);     // exp2(-inf) = 0 with run_l = 0: stays 0
                    run_m[rb] = m_new;
                    red_c[rb] = ms;
                }
            }
        } else if (MASKED) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (j0b + l32 > last_visible(g, L, R, rowg0 + rb * 32 + c_row(i, g2))) a[rb][i] = -INFINITY;
        }
    };
    auto reduce_part = [&](f32x16 (&a)[NB], int sl, int rb) {  // elements [sl*SLICE, (sl+1)*SLICE) of row tile rb
#pragma unroll
        for (int e = 0; e < SLICE; ++e) {
            const int i = sl * SLICE + e;
            if (SWEEP2) {
                red_s[i & 1] += fast_exp2(fmaf(a[rb][i], c_pin, -rcv[rb][i]));
            } else {
                if (rb == 0) red_s[i & 1] += fast_exp2(fmaf(a[rb][i], c_pin, -red_c[rb]));
                else         red_t[rb] += fast_exp2(fmaf(a[rb][i], c_pin, -red_c[rb]));
            }
        }
    };
    auto reduce_end = [&](f32x16 (&a)[NB], int cbuf, int kb) {
        if (SWEEP2) {
            // rows held by the other half of the wave; the other waves' rows are added by the loader wave
            // v_permlane32_swap trades lanes 32..63 of its first operand with lanes 0..31 of its second: afterwards
            // one register holds the lower-half sums in both halves, the other the upper-half sums. (Written as asm
            // because the two-result builtin got its results merged; the wait states in front cover the vector
            // write that produces the operands.)
            float v = red_s[0] + red_s[1];
#if defined(__HIP_DEVICE_COMPILE__)
            float v_hi = v;
            asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(v), "+v"(v_hi));
            v += v_hi;
#endif
            if (g2 == 0) lds_cols[cbuf * (WR * T::TK) + wave * T::TK + kb * 32 + l32] = v;
        } else {
            red_t[0] = red_s[0] + red_s[1];
            // Terms are exp2(logit - reference) with a reference that may lie below the block's maximum. A block sum
            // that has left [0, 2^64) (inf included) means the reference is stale for that row: raise it to the
            // block's maximum, rescale what was summed so far and sum the block again, now with terms <= 1. The
            // logits are still in the accumulator registers. Rare (the first block of a row is its reference, and
            // logits seldom climb 64 binary orders above it), so the test is one compare per row tile and block.
            float worst = red_t[0];
#pragma unroll
            for (int rb = 1; rb < NB; ++rb) worst = fmaxf(worst, red_t[rb]);
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(worst < 0x1p64f)) != 0, 0)) {
#pragma unroll
                for (int rb = 0; rb < NB; ++rb) {
                    if (!(red_t[rb] < 0x1p64f)) {
                        float mx = a[rb][0];
#pragma unroll
                        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, a[rb][i]);
                        const float m_new = fmaxf(run_m[rb], mx * c);    // finite: the row has a finite reference
                        run_l[rb] *= fast_exp2(run_m[rb] - m_new);
                        run_m[rb] = m_new;
                        red_c[rb] = m_new;
                        float sum = 0.f;
#pragma unroll
                        for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(a[rb][i], c, -m_new));
                        red_t[rb] = sum;
                    }
                }
            }
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) run_l[rb] += red_t[rb];
        }
    };

    // --- one pipelined step sequence: MFMAs of block (slot_m, kb_m) into `am`, reduction of `ar` ---------------
    // stream = true: fragments of the first PF k-steps are already in the ring, and the last PF steps pull the
    // head of the next block (slot_n, kb_n). stream = false: the block loads its own fragments.
    auto run_block = [&](auto do_mfma_tag, auto do_red_tag, auto stream_tag, f32x16 (&am)[NB], int slot_m, int kb_m,
                         int slot_n, int kb_n, f32x16 (&ar)[NB]) {
        constexpr bool DO_MFMA = decltype(do_mfma_tag)::value;
        constexpr bool DO_RED = decltype(do_red_tag)::value;
        constexpr bool STREAM = decltype(stream_tag)::value;
        if (DO_MFMA && !STREAM) {
#pragma unroll
            for (int kk = 0; kk < PF; ++kk) frag_load(slot_m, kb_m, kk, kk % RING);
        }
#pragma unroll
        for (int kk = 0; kk < T::KK; ++kk) {
            if (DO_MFMA) {
                if (kk + PF < T::KK) frag_load(slot_m, kb_m, kk + PF, (kk + PF) % RING);
                else if (STREAM)     frag_load(slot_n, kb_n, kk + PF - T::KK, (kk + PF) % RING);
            }
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) {
                if (DO_MFMA) {
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    const f32x16 cin = (kk == 0) ? zero : am[rb];
                    if (SWEEP2)   // C[row][key]: lane = key l32, rows c_row(i, g2)
                        am[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][kk], kfr[kk % RING], cin, 0, 0, 0);
                    else          // C[key][row]: lane = row l32, keys c_row(i, g2)
                        am[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[kk % RING], qf[rb][kk], cin, 0, 0, 0);
                }
                if (DO_RED && kk < 16) reduce_part(ar, kk, rb);
                // One MFMA, then SLICE logits of vector work (about as long as the MFMA occupies the matrix pipe),
                // then the next MFMA: a wave issues in order, so two MFMAs back to back would hold its vector work
                // up for a whole pass of the matrix pipe. The arithmetic has no side effects, and the compiler would
                // otherwise gather all MFMAs of the block in front of all the vector work; an empty asm statement
                // that takes the accumulator, the sums and the scale in and out fixes the order.
#if defined(__HIP_DEVICE_COMPILE__)
                if (DO_MFMA && DO_RED) {
                    if constexpr (NB == 1)      asm volatile("" : "+v"(c_pin), "+v"(am[rb]), "+v"(red_s[0]), "+v"(red_s[1]));
                    else if constexpr (NB == 2) asm volatile("" : "+v"(c_pin), "+v"(am[rb]), "+v"(red_s[0]), "+v"(red_s[1]), "+v"(red_t[1]));
                    else                        asm volatile("" : "+v"(c_pin), "+v"(am[rb]), "+v"(red_s[0]), "+v"(red_s[1]), "+v"(red_t[1]), "+v"(red_t[NB - 1]));
                }
#endif
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using Y = std::true_type;
    using N = std::false_type;

    // Tiles from t_plain_end on contain (row, key) pairs that need the visibility test: always the tail of a head.
    const int t_first_masked = g.causal ? (L - g.W + 1) / T::TK : L / T::TK;
    const int t_plain_end = min(max(t_first_masked, t_begin), t_end);
    auto slot_of = [&](int t) { return (t - t_begin) % T::STAGES; };

    wg_barrier();                                       // the first tile is in the ring (and lds_rc is filled)
    if (SWEEP2) {
#pragma unroll
        for (int rb = 0; rb < NB; ++rb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(lds_rc + row0 + g2 * 4 + rb * 32 + q4 * 8);
#pragma unroll
                for (int u = 0; u < 4; ++u) rcv[rb][q4 * 4 + u] = v[u];
            }
    }
    int t = t_begin;
    if (t < t_plain_end) {
        // ---- pipelined part: blocks (t, 0), (t, 1), (t + 1, 0), ... ; acc0 holds even blocks, acc1 odd ones
        run_block(Y{}, N{}, N{}, acc0, slot_of(t), 0, 0, 0, acc1);           // prologue: MFMAs of the first block
        if (!SWEEP2) reference_from(acc0);
        // its last steps did not prefetch: start the stream for the second block
        if (T::KB >= 2) {
            static_assert(T::KB == 1 || T::KB % 2 == 0, "the accumulator sets alternate by block parity");
#pragma unroll
            for (int kk = 0; kk < PF; ++kk) frag_load(slot_of(t), 1, kk, kk % RING);
            for (; t < t_plain_end; ++t) {
                const bool more = t + 1 < t_plain_end;
                const int cbuf = (t - t_begin) % 3;
#pragma unroll
                for (int kb = 0; kb < T::KB; ++kb) {
                    // block in flight on the matrix pipe: (t, kb + 1), or the first block of the next tile; the
                    // fragment stream then runs on into the block after that one
                    const bool wrap1 = kb + 1 >= T::KB, wrap2 = kb + 2 >= T::KB;
                    const int slot_m = wrap1 ? slot_of(t + 1) : slot_of(t), kb_m = wrap1 ? kb + 1 - T::KB : kb + 1;
                    const int slot_n = wrap2 ? slot_of(t + 1) : slot_of(t), kb_n = wrap2 ? kb + 2 - T::KB : kb + 2;
                    if ((kb & 1) == 0) {
                        reduce_begin(N{}, acc0, t * T::TK + kb * 32);
                        run_block(Y{}, Y{}, Y{}, acc1, slot_m, kb_m, slot_n, kb_n, acc0);
                        reduce_end(acc0, cbuf, kb);
                    } else {
                        reduce_begin(N{}, acc1, t * T::TK + kb * 32);
                        if (!wrap1 || more) run_block(Y{}, Y{}, Y{}, acc0, slot_m, kb_m, slot_n, kb_n, acc1);
                        else                run_block(N{}, Y{}, N{}, acc0, 0, 0, 0, 0, acc1);
                        reduce_end(acc1, cbuf, kb);
                    }
                }
                wg_barrier();
                flush_tile(t);
            }
        } else {
            // one block per tile: two tiles per trip so that the accumulator sets alternate statically. The MFMAs
            // run one tile ahead (tile t + 1 is visible since the last barrier); the fragment stream must not run
            // on into tile t + 2, which the loader is depositing right now, so every block loads its own.
            while (t < t_plain_end) {
                reduce_begin(N{}, acc0, t * T::TK);
                if (t + 1 < t_plain_end) run_block(Y{}, Y{}, N{}, acc1, slot_of(t + 1), 0, 0, 0, acc0);
                else                     run_block(N{}, Y{}, N{}, acc1, 0, 0, 0, 0, acc0);
                reduce_end(acc0, (t - t_begin) % 3, 0);
                wg_barrier();
                flush_tile(t);
                ++t;
                if (t >= t_plain_end) break;
                reduce_begin(N{}, acc1, t * T::TK);
                if (t + 1 < t_plain_end) run_block(Y{}, Y{}, N{}, acc0, slot_of(t + 1), 0, 0, 0, acc1);
                else                     run_block(N{}, Y{}, N{}, acc0, 0, 0, 0, 0, acc1);
                reduce_end(acc1, (t - t_begin) % 3, 0);
                wg_barrier();
                flush_tile(t);
                ++t;
            }
        }
    }
    // ---- masked tail (at most a few tiles per head): plain sequence, with the visibility test
    for (; t < t_end; ++t) {
        const int cbuf = (t - t_begin) % 3;
#pragma unroll
        for (int kb = 0; kb < T::KB; ++kb) {
            run_block(Y{}, N{}, N{}, acc0, slot_of(t), kb, 0, 0, acc1);
            reduce_begin(Y{}, acc0, t * T::TK + kb * 32);
            run_block(N{}, Y{}, N{}, acc1, 0, 0, 0, 0, acc0);
            reduce_end(acc0, cbuf, kb);
        }
        wg_barrier();
        flush_tile(t);
    }

    if (!SWEEP2) {
        // a row's keys are spread over the two halves of the wave
        float* my_stats = stats + ((size_t)head * nsplit + split) * rows_pad * 2;
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            const float m2 = __shfl_xor(run_m[rb], 32, 64), l2 = __shfl_xor(run_l[rb], 32, 64);
            merge_stats(run_m[rb], run_l[rb], m2, l2);
            if (g2 == 0) {
                const int r = rowg0 + rb * 32 + l32;
                my_stats[2 * r] = run_m[rb];
                my_stats[2 * r + 1] = run_l[rb];
            }
        }
    }
}

// per row: reference + log2(sum) over the key ranges (fixed order); +inf for padded rows, whose exp2 then vanishes.
// Row constants from log-sum-exp values that the caller already has (natural log of the softmax denominator of
// every window row, as an attention kernel that ran the window's queries returns them): replaces sweep 1.
static __global__ __launch_bounds__(64) void score_cst_from_lse_kernel(Geom g, const float* __restrict__ lse,
                                                                       int rows_pad, float* __restrict__ cst)
{
    const int blocks_per_head = (rows_pad + 63) / 64;
    const int head = blockIdx.x / blocks_per_head;
    const int r = (blockIdx.x - head * blocks_per_head) * 64 + threadIdx.x;
    if (r >= rows_pad) return;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    float out = INFINITY;
    if (r < g.G * g.W) {
        const int qh = r / g.W, wrow = r - qh * g.W;
        out = lse[((size_t)item * g.H_q + (size_t)h * g.G + qh) * g.W + wrow] * 1.44269504088896340736f;
    }
    cst[(size_t)head * rows_pad + r] = out;
}

// raw += raw_b: the column sums of the second row range of a split sweep 2 (fixed order: deterministic)
static __global__ __launch_bounds__(256) void score_add_kernel(float* __restrict__ raw, const float* __restrict__ raw_b, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) raw[i] += raw_b[i];
}

// which = 1: per-range row statistics into stats (sweep 1; the caller merges them into cst with launch_score_merge),
//            or the conversion of supplied log-sum-exp values straight into cst;
// which = 2: column sums (sweep 2) from the cst at cst_in. The two may use different (NB, WR) tilings and key-range
// counts: they only share the row pitch rows_pad of the statistics.
template <int D, int NB, int WR>
hipError_t launch_sweep(int which, const Geom& g, const void* q_win, const void* k, const int32_t* cu_seq,
                        int nsplit, int rows_pad, int row_base, float* stats, float* cst, float* raw, hipStream_t s,
                        const float* lse)
{
    using T = Tile<D, NB, WR>;
    const int n_heads = g.n_items * g.H_kv;
    const dim3 grid((unsigned)(n_heads * nsplit));
    static std::atomic<bool> attr_set{false};
    if (!attr_set && T::LDS_BYTES > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_kernel<D, NB, WR, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_kernel<D, NB, WR, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (which == 1) {
        const unsigned merge_blocks = (unsigned)(n_heads * ((rows_pad + 63) / 64));
        if (lse) {
            hipLaunchKernelGGL(score_cst_from_lse_kernel, dim3(merge_blocks), dim3(64), 0, s, g, lse, rows_pad, cst);
        } else {
            hipLaunchKernelGGL((score_kernel<D, NB, WR, false>), grid, dim3(T::THREADS), T::LDS_BYTES, s, g,
                               (const __bf16*)q_win, (const __bf16*)k, cu_seq, nsplit, rows_pad, 0, stats,
                               (const float*)nullptr, raw);
        }
    } else {
        hipLaunchKernelGGL((score_kernel<D, NB, WR, true>), grid, dim3(T::THREADS), T::LDS_BYTES, s, g,
                           (const __bf16*)q_win, (const __bf16*)k, cu_seq, nsplit, rows_pad, row_base, (float*)nullptr,
                           (const float*)cst, raw);
    }
    return hipGetLastError();
}

}  // namespace score_detail

// one translation unit per head_dim keeps the build parallel
hipError_t launch_score_d64(int which, const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, int rows_pad, int row_base, float* stats, float* cst, float* raw,
        hipStream_t s, const float* lse);
hipError_t launch_score_d128(int which, const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, int rows_pad, int row_base, float* stats, float* cst, float* raw,
        hipStream_t s, const float* lse);
hipError_t launch_score_d256(int which, const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, int rows_pad, int row_base, float* stats, float* cst, float* raw,
        hipStream_t s, const float* lse);

}  // namespace audiokv
