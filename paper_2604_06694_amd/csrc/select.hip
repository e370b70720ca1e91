// Stage 4: per-head top-k with a forced window tail (paper Sec. 1, Solution 2:
// Top-K selection on the importance scores; window w of Sec. 3.1 Eq. 1).
//
// One workgroup per head. Scores become order-preserving 32-bit keys held in
// registers (token t + 1024 e in register e of thread t: coalesced loads).
// The threshold is the largest T with #(key >= T) >= the number of tokens to
// keep. A long head first brackets it between two pivots taken from a sample
// of its keys and checks the counts (exact whatever the sample; a bracket that
// fails falls back); otherwise T is found bit by bit with counting passes over
// all keys until the keys that the remaining bits can still separate are few.
// Those go to a short list in LDS (a short head is its own list), where the
// remaining bits are set one per pass or eight per round (digit counts), and
// once at most 64 keys are undecided one wave ranks them against each other
// and reads the threshold off directly. Tokens above the threshold are kept,
// tokens equal to it are kept in index order until the budget is full: for a
// fixed register the lanes of a wave hold 64 consecutive tokens, so lane masks
// give every (register, wave) chunk its counts, one block-wide exclusive scan
// over the chunks gives their output offsets, and every kept token computes
// its own ascending output slot from the offsets and its rank in the lane
// mask. Integer-only (counts and integer adds in any order): bit-exact.
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

constexpr int kCompact = 8;          // undecided keys per thread once the candidates have been narrowed down
// Pivots from a sample: of 512 keys spread over the head, the two whose ranks lie kMargin on either side of the
// budget's quantile bracket the threshold except with a probability of about 1e-4 (kMargin is 4 sigma of the binomial
// spread of a 512-sample quantile) and hold about 2 * kMargin / 512 = 17 % of the keys between them (the short list
// holds 25 % of the longest head: 4.7 sigma of the spread of that share).
constexpr int kSamples = 512, kMargin = 44;
constexpr int kPivotBits = 20;       // a pivot need not be a key: its low bits stay zero, which shortens the search for it

template <int EPT>   // tokens per thread; the head must have at most EPT * kSelThreads candidates
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    Geom g, const float* __restrict__ scores, const int32_t* __restrict__ budgets,
    const int32_t* __restrict__ cu_b, const int32_t* __restrict__ cu_seq, int32_t* __restrict__ indices)
{
    __shared__ uint32_t narrowed[kCompact * kSelThreads];   // keys still undecided after narrowing (any order)
    __shared__ int pass_count[3];
    __shared__ int list_n, last_n;                   // fill counts of `narrowed` and `last_keys`
    __shared__ __attribute__((aligned(16))) uint32_t last_keys[64];
    __shared__ uint32_t ranked[2];                  // threshold and #(key > threshold) from the wave that ranks the last keys
    __shared__ int chunk_gt[EPT * kSelWaves], chunk_eq[EPT * kSelWaves];   // per (register, wave) chunk of 64 tokens
    __shared__ uint32_t samp[kSamples];
    __shared__ uint32_t pivot[2];
    __shared__ int above_hi;
    __shared__ __attribute__((aligned(16))) int hist[256];   // digit counts of the short list
    __shared__ int digit_pick[3];
    const int head = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const float* s = scores + (size_t)tok0 * g.H_kv + (size_t)h * L;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

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

    // Thread t holds tokens t, t + 1024, t + 2048, ...: the loads are coalesced straight into registers, a thread's
    // keys are spread over the whole sequence (so the undecided ones stay evenly spread, see below), and for a fixed
    // register the lanes of a wave hold 64 consecutive tokens (so one lane mask is 64 bits of a per-token bitmap).
    uint32_t key[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int j = tid + e * kSelThreads;
        // clamped address and a mask instead of a branch around the load: all loads of a thread are in flight together
        const float f = s[min(j, n_cand - 1)];
        key[e] = order_key(f) & (j < n_cand ? 0xffffffffu : 0u);   // 0 is below every real key and every trial
    }

    // k-th largest key: the largest T with #(key >= T) >= want, found bit by bit. c_lo = #(key >= T) and
    // c_up = #(key >= T + 2^bit) bracket the keys whose upper bits equal T's: the only ones later bits can still
    // tell apart. Once they are few they are moved to a short list, kCompact per thread, and the remaining passes
    // count only those; the keys above the bracket are a constant.
    if (tid < 3) pass_count[tid] = 0;
    if (tid == 3) { list_n = 0; last_n = 0; above_hi = 0; }
    if (tid < 64) last_keys[tid] = 0u;               // 0 is below every key that can reach the list
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    uint32_t T = 0;
    int c_lo = n_cand, c_up = 0;
    int parity = 0;
    // Move the keys for which `in_bracket` holds to the short list. Its order does not matter (the keys are only
    // counted), so a wave reserves room for all its keys with one LDS add and places them by lane-mask rank.
    auto to_short_list = [&](auto in_bracket) {
        int wave_total = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            wave_total += __builtin_popcountll(__builtin_amdgcn_ballot_w64(in_bracket(key[e])));
        int base = 0;
        if (lane == 0 && wave_total) base = atomicAdd(&list_n, wave_total);
        base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const bool in = in_bracket(key[e]);
            const unsigned long long m = __builtin_amdgcn_ballot_w64(in);
            const int pos = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, (uint32_t)base));
            if (in && pos < kCompact * kSelThreads) narrowed[pos] = key[e];   // keys beyond the list's end are dropped: the caller checks list_n
            base += __builtin_popcountll(m);
        }
        __syncthreads();
    };
    // One counting pass: `c` is this wave's count of keys >= trial (wave-uniform). The block-wide sum goes through
    // one LDS counter per pass (three in rotation: the counter of the next pass was last read two passes ago,
    // before the previous barrier, so it is cleared while this one is in use). Integer adds: order-free.
    auto decide = [&](uint32_t trial, int c, int c_above) {
        if (lane == 0) atomicAdd(&pass_count[parity], c);
        if (tid == 0) pass_count[parity == 2 ? 0 : parity + 1] = 0;
        __syncthreads();
        const int t = c_above + pass_count[parity];
        if (t >= want) { T = trial; c_lo = t; } else { c_up = t; }
        parity = parity == 2 ? 0 : parity + 1;
    };
    int bit = 31;
    // Heads of at most kCompact keys per thread are their own short list from the start (all 32 bits undecided).
    bool have_list = EPT <= kCompact;
    bool spread = false;                             // the listed keys lie between two pivots: no crowded digits
    if (EPT <= kCompact) bit = 32;
    if (EPT > kCompact && n_cand >= 12 * kSelThreads) {
        // Long head: instead of counting all keys once per bit until few are undecided, bracket the threshold between
        // two pivots taken from a sample and go on with the keys in between. Whatever the sample looks like the result
        // is exact: the counts are checked, and a bracket that misses the threshold or holds too many keys (heavy
        // ties, adversarial order) falls back to the bit-by-bit passes.
        const int full_regs = n_cand / kSelThreads;              // registers that hold a real key in every thread
        if (tid < kSamples) {
            // sample i: token 2 i or 2 i + 1 (both parities occur) of the block of 1024 tokens number e_i, where e_i
            // runs through [0, full_regs) in scrambled order; read once more from memory (it is in the cache) rather
            // than picked out of the registers
            const int hashed = (tid * 97) & (kSamples - 1);
            const int e_i = (hashed * full_regs) / kSamples;
            samp[tid] = order_key(s[2 * tid + ((hashed >> 4) & 1) + e_i * kSelThreads]);
        }
        __syncthreads();
        if (wave < 2) {
            // Two waves find one pivot each, the sample of rank r (0 = largest) cut to its upper kPivotBits bits: the
            // same bit-by-bit search as below, on 8 samples per lane and with no barrier (a wave is alone with its counts).
            const int centre = (int)(((long long)want * kSamples) / n_cand);   // sample rank of the budget's quantile
            const int r = wave == 0 ? centre - kMargin : centre + kMargin;
            uint32_t sk[kSamples / 64];
#pragma unroll
            for (int j = 0; j < kSamples / 64; ++j) sk[j] = samp[lane + 64 * j];
            uint32_t V = 0;
            for (int bb = 31; bb >= 32 - kPivotBits; --bb) {
                const uint32_t trial = V | (1u << bb);
                int c = 0;
#pragma unroll
                for (int j = 0; j < kSamples / 64; ++j) c += __builtin_popcountll(__builtin_amdgcn_ballot_w64(sk[j] >= trial));
                if (c > r) V = trial;                // r < 0: every trial passes: (almost) nothing is at or above V
            }
            if (lane == 0) pivot[1 - wave] = max(V, 1u);   // r >= kSamples: no trial passes; 1 is below every real key
        }
        __syncthreads();
        const uint32_t lo = pivot[0], hi = pivot[1];                         // lo <= hi
        {
            // keys at or above hi are only counted (per lane, then summed over the wave through lane masks) ...
            uint32_t per_lane = 0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) per_lane += key[e] >= hi ? 1u : 0u;
            int c_hi = 0;
#pragma unroll
            for (int bb = 0; EPT >> bb; ++bb)            // per_lane <= EPT
                c_hi += __builtin_popcountll(__builtin_amdgcn_ballot_w64((per_lane >> bb) & 1u)) << bb;
            if (lane == 0 && c_hi) atomicAdd(&above_hi, c_hi);
        }
        // ... and the keys in [lo, hi) go to the short list
        to_short_list([&](uint32_t kx) { return kx - lo < hi - lo; });   // nothing if lo == hi
        const int n_hi = above_hi, n_in = list_n;
        if (lo < hi && n_hi < want && want <= n_hi + n_in && n_in <= kCompact * kSelThreads) {   // uniform
            have_list = true;
            spread = true;
            // lo and hi - 1 agree above their highest differing bit d: those bits are the threshold's. Below, the
            // short list alone decides: for a trial T' in that range #(key >= T') is n_hi plus the listed keys >= T'
            // wherever that matters (a trial at or above hi must fail and does, one at or below lo must pass and does).
            const uint32_t x = lo ^ (hi - 1u);
            const int d = x ? 31 - __builtin_clz(x) : -1;
            T = d >= 0 ? (lo & ~((2u << d) - 1u)) : lo;
            bit = d + 1;                                 // the short passes start at bit d
            c_lo = n_hi + n_in;
            c_up = n_hi;
        } else {
            __syncthreads();                             // everybody has read list_n
            if (tid == 0) list_n = 0;                    // (the bit-by-bit passes below meet at barriers before it is used again)
        }
    }
    bool narrow = false;
    for (; !have_list && bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        // Wave-wide count, split between the two issue ports so that neither is the bottleneck: the even registers
        // through lane masks and population counts on the scalar unit (which the whole CU shares), the odd ones
        // through a per-lane counter on the vector unit, whose bits are then summed with a few lane masks.
        int c = 0;
        uint32_t per_lane = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            if (e & 1) per_lane += key[e] >= trial ? 1u : 0u;
            else c += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] >= trial));
        }
#pragma unroll
        for (int bb = 0; (EPT / 2) >> bb; ++bb)      // per_lane <= EPT / 2
            c += __builtin_popcountll(__builtin_amdgcn_ballot_w64((per_lane >> bb) & 1u)) << bb;
        decide(trial, c, 0);
        // Few undecided keys left (uniform decision)? T >> bit != 0 keeps the padding key 0 out of the bracket.
        if (EPT > kCompact && bit > 0 && (T >> bit) != 0u && c_lo - c_up <= kCompact * kSelThreads) { narrow = true; break; }
    }
    if (narrow) {
        // the real keys in [T, T + 2^bit): those whose upper bits equal T's
        const uint32_t hi_part = T >> bit;
        to_short_list([&](uint32_t kx) { return (kx >> bit) == hi_part; });
        have_list = true;
    }
    if (have_list) {
        const int n_und = c_lo - c_up;               // == list_n
        const int c_above = c_up;                    // keys above the bracket: counted in every later pass
        uint32_t ckey[kCompact];
#pragma unroll
        for (int e = 0; e < kCompact; ++e) {
            const int i = tid + e * kSelThreads;
            if constexpr (EPT <= kCompact) ckey[e] = e < EPT ? key[e < EPT ? e : 0] : 0u;   // (0 where there is no token)
            else ckey[e] = i < n_und ? narrowed[i] : 0u;
        }
        // (validity of a listed key is its index, tid + e * 1024 < n_und, in both cases: the value 0 also passes for
        // a key whose upper bits equal T's when those are all zero)
        // Undecided bits are [0, bit - 1]. They are settled one per pass while they are exponent bits of keys that
        // may crowd into a few digits, and eight per round otherwise (bits 22 and lower, or any bits of keys that lie
        // between two pivots: LDS adds to one address serialise, adds spread over the digits do not): the listed keys whose
        // upper bits equal T's are counted by their next eight bits in LDS (integer adds), and one wave finds the
        // largest digit D with c_up + #(digit >= D) >= want from the suffix sums: what eight passes would set.
        // As soon as at most 64 keys are undecided, one wave ranks them (below).
        bool rank_last = false;
        while (bit > 0) {
            if (bit <= 31 && c_lo - c_up <= 64) { rank_last = true; break; }   // uniform
            if (bit >= 8 && bit <= (spread ? 31 : 23)) {
                const int sh = bit - 8;
                const uint32_t prefix = T >> bit;
#pragma unroll
                for (int e = 0; e < kCompact; ++e)
                    if (tid + e * kSelThreads < n_und && (ckey[e] >> bit) == prefix)
                        atomicAdd(&hist[(ckey[e] >> sh) & 255u], 1);
                __syncthreads();
                if (wave == 0) {
                    const int4 h4 = reinterpret_cast<const int4*>(hist)[lane];          // digits 4 lane .. 4 lane + 3
                    const int s3 = h4.w, s2 = s3 + h4.z, s1 = s2 + h4.y, s0 = s1 + h4.x;   // sums up to the lane's last digit
                    int incl = s0;                                                     // + all higher lanes
#pragma unroll
                    for (int o = 1; o < 64; o <<= 1) {
                        const int t = __shfl_down(incl, o, 64);
                        if (lane + o < 64) incl += t;
                    }
                    const int base = c_up + incl - s0;       // keys above the bracket + digits above this lane's
                    const int S[5] = {base + s0, base + s1, base + s2, base + s3, base};   // #(key >= T | D << sh), D = 4 lane + K
#pragma unroll
                    for (int K = 0; K < 4; ++K)
                        if (S[K] >= want && S[K + 1] < want) {   // exactly one (lane, K): S falls from c_lo >= want to c_up < want
                            digit_pick[0] = 4 * lane + K; digit_pick[1] = S[K]; digit_pick[2] = S[K + 1];
                        }
                    reinterpret_cast<int4*>(hist)[lane] = make_int4(0, 0, 0, 0);        // for the next round
                }
                __syncthreads();
                T |= (uint32_t)digit_pick[0] << sh;
                c_lo = digit_pick[1];
                c_up = digit_pick[2];
                bit = sh;
                continue;
            }
            --bit;
            const uint32_t trial = T | (1u << bit);
            int c = 0;
#pragma unroll
            for (int e = 0; e < kCompact; ++e) c += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ckey[e] >= trial));
            decide(trial, c, c_above);
        }
        if (rank_last) {
            // At most 64 keys share T's upper bits: the remaining bits of the threshold are those of the r-th largest
            // of them, r = want - c_up. One wave holds them a key per lane and ranks each against all the others.
            const uint32_t hi2 = T >> bit;
            int wt = 0;
#pragma unroll
            for (int e = 0; e < kCompact; ++e)
                wt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(tid + e * kSelThreads < n_und && (ckey[e] >> bit) == hi2));
            int b2 = 0;
            if (lane == 0 && wt) b2 = atomicAdd(&last_n, wt);
            b2 = __builtin_amdgcn_readfirstlane(b2);
#pragma unroll
            for (int e = 0; e < kCompact; ++e) {
                const bool in = tid + e * kSelThreads < n_und && (ckey[e] >> bit) == hi2;
                const unsigned long long m = __builtin_amdgcn_ballot_w64(in);
                const int pos = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, (uint32_t)b2));
                if (in && pos < 64) last_keys[pos] = ckey[e];
                b2 += __builtin_popcountll(m);
            }
            __syncthreads();
            if (wave == 0) {
                const int n_last = c_lo - c_up;      // == last_n, 1..64; the rest of last_keys is 0
                const uint32_t mine_k = last_keys[lane];
                const int r = want - c_up;           // 1 <= r <= n_last
                int gt = 0, ge = 0;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    const uint4 v = reinterpret_cast<const uint4*>(last_keys)[jj];
                    gt += (v.x > mine_k ? 1 : 0) + (v.y > mine_k ? 1 : 0) + (v.z > mine_k ? 1 : 0) + (v.w > mine_k ? 1 : 0);
                    ge += (v.x >= mine_k ? 1 : 0) + (v.y >= mine_k ? 1 : 0) + (v.z >= mine_k ? 1 : 0) + (v.w >= mine_k ? 1 : 0);
                }
                // the r-th largest value v has #(key > v) < r <= #(key >= v); every lane that holds v says so
                const bool is_thr = lane < n_last && gt < r && r <= ge;
                const unsigned long long who = __builtin_amdgcn_ballot_w64(is_thr);
                const int first = __builtin_ctzll(who | (1ull << 63));
                if (lane == first) { ranked[0] = mine_k; ranked[1] = (uint32_t)(c_up + gt); }
            }
            __syncthreads();
            T = ranked[0];
            c_up = (int)ranked[1];
        }
    }
    // tokens strictly above T all stay; tokens equal to T stay in index order while room is left
    const int need_eq = want - c_up;                 // c_up = #(key > T); >= 1 by construction of T

    // For a fixed register e, wave w holds the 64 consecutive tokens [e*1024 + w*64, +64): chunk e*16 + w in token
    // order. Count the chunk's tokens above and equal to T from lane masks (lane e collects the counts of register e) ...
    int my_gt = 0, my_eq = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int cg = __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] > T));
        const int ce = __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] == T));
        // lane e of my_gt / my_eq <- the wave-uniform counts of register e
        asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(my_gt) : "s"(cg), "n"(e));
        asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(my_eq) : "s"(ce), "n"(e));
    }
    if (lane < EPT) { chunk_gt[lane * kSelWaves + wave] = my_gt; chunk_eq[lane * kSelWaves + wave] = my_eq; }
    __syncthreads();
    // ... turn the counts into exclusive prefixes over the chunks (one scan for both) ...
    if (wave == 0) {
        constexpr int kChunks = EPT * kSelWaves;     // <= 512
        constexpr int kPer = kChunks / 64;           // consecutive chunks per lane
        int cg[kPer], ce[kPer], sg = 0, se = 0;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            cg[u] = chunk_gt[lane * kPer + u]; ce[u] = chunk_eq[lane * kPer + u];
            sg += cg[u]; se += ce[u];
        }
        int ig = sg, ie = se;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int tg = __shfl_up(ig, o, 64), te = __shfl_up(ie, o, 64);
            if (lane >= o) { ig += tg; ie += te; }
        }
        int eg = ig - sg, ee = ie - se;              // counts in the lanes before this one
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            chunk_gt[lane * kPer + u] = eg; chunk_eq[lane * kPer + u] = ee;
            eg += cg[u]; ee += ce[u];
        }
    }
    __syncthreads();
    // ... and let every kept token compute its output slot: tokens above T before it, plus the kept ties before it.
    // The slots of a wave's tokens are consecutive, so each store instruction writes one run of the output.
    if (lane < EPT) { my_gt = chunk_gt[lane * kSelWaves + wave]; my_eq = chunk_eq[lane * kSelWaves + wave]; }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const bool is_gt = key[e] > T, is_eq = key[e] == T;
        const unsigned long long mg = __builtin_amdgcn_ballot_w64(is_gt);
        const unsigned long long me = __builtin_amdgcn_ballot_w64(is_eq);
        const int gt_pre = __builtin_amdgcn_readlane(my_gt, e), eq_pre = __builtin_amdgcn_readlane(my_eq, e);
        if (me == 0) {
            // no tie with the threshold among the chunk's 64 tokens (the usual case): the kept ties before any of
            // them are a chunk-wide number, folded into the base of the lane-mask rank
            const int pos = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32),
                                __builtin_amdgcn_mbcnt_lo((uint32_t)mg, (uint32_t)(gt_pre + min(eq_pre, need_eq))));
            if (is_gt && pos < want) out[pos] = tid + e * kSelThreads;
        } else {
            const int gt_before = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mg, (uint32_t)gt_pre));
            const int eq_before = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, (uint32_t)eq_pre));
            const int pos = gt_before + min(eq_before, need_eq);
            if ((is_gt || (is_eq && eq_before < need_eq)) && pos < want) out[pos] = tid + e * kSelThreads;
        }
    }
}

// Heads longer than 32 * 1024 tokens: the keys do not fit the registers of one workgroup, so every counting pass
// streams the scores again (they stay in L2: 4 bytes per token), and the output pass walks the sequence in rounds of
// 32 consecutive tokens per thread. Same threshold, same tie rule, same ascending order; slower per token than the
// register kernel (32 full passes), meant for the rare very long head.
__global__ __launch_bounds__(kSelThreads) void select_stream_kernel(
    Geom g, const float* __restrict__ scores, const int32_t* __restrict__ budgets,
    const int32_t* __restrict__ cu_b, const int32_t* __restrict__ cu_seq, int32_t* __restrict__ indices)
{
    __shared__ int slots[4 * kSelWaves];
    __shared__ uint32_t short_list[kCompact * kSelThreads];
    __shared__ int list_n;
    const int head = blockIdx.x;
    const int item = head / g.H_kv, h = head - item * g.H_kv;
    const int tok0 = cu_seq[item];
    const int L = cu_seq[item + 1] - tok0;
    const float* s = scores + (size_t)tok0 * g.H_kv + (size_t)h * L;
    const int tid = threadIdx.x;

    const int W = min(g.W, L);
    const int n_cand = L - W;
    const int room = cu_b[head + 1] - cu_b[head];
    const int b = min(min(max(budgets[head], W), L), room);
    const int want = max(b - W, 0);
    int32_t* out = indices + cu_b[head];
    for (int w = tid; w < W; w += kSelThreads)
        if (want + w < room) out[want + w] = n_cand + w;
    if (want <= 0) return;

    // the largest T with #(key >= T) >= want, bit by bit; c_up ends as #(key > T): the count of the last trial that
    // failed, which is T + 1 (all lower bits of T are ones from there down)
    uint32_t T = 0;
    int c_lo = n_cand, c_up = 0, parity = 0;
    int bit = 31;
    bool narrow = false;
    for (; bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        int c = 0;
        for (int j0 = tid; j0 < n_cand; j0 += 16 * kSelThreads) {      // 16 loads in flight: clamped address, masked count
            float f[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) f[u] = s[min(j0 + u * kSelThreads, n_cand - 1)];
#pragma unroll
            for (int u = 0; u < 16; ++u) c += (j0 + u * kSelThreads < n_cand && order_key(f[u]) >= trial) ? 1 : 0;
        }
        const int t = block_count(c, slots, parity);
        parity ^= 1;
        if (t >= want) { T = trial; c_lo = t; } else { c_up = t; }
        // the keys that the remaining bits can still tell apart are those whose upper bits equal T's: once they fit
        // the short list, one more streaming pass collects them and the rest of the search never touches memory
        if (bit > 0 && c_lo - c_up <= kCompact * kSelThreads) { narrow = true; break; }
    }
    if (narrow) {
        const uint32_t hi_part = T >> bit;
        if (tid == 0) list_n = 0;
        __syncthreads();
        for (int j0 = tid; j0 < n_cand; j0 += 16 * kSelThreads) {
            float f[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) f[u] = s[min(j0 + u * kSelThreads, n_cand - 1)];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const uint32_t key = order_key(f[u]);
                const bool mine = j0 + u * kSelThreads < n_cand && (key >> bit) == hi_part;
                // the order of the list does not matter (it is only counted): one LDS add per wave and step
                const unsigned long long m = __builtin_amdgcn_ballot_w64(mine);
                int base = 0;
                if (m) {
                    if ((tid & 63) == 0) base = atomicAdd(&list_n, __builtin_popcountll(m));
                    base = __shfl(base, 0, 64);
                    const int pos = base + __builtin_popcountll(m & ((1ull << (tid & 63)) - 1ull));
                    if (mine && pos < kCompact * kSelThreads) short_list[pos] = key;   // (the counts say it always fits)
                }
            }
        }
        __syncthreads();
        const int n_und = c_lo - c_up;                   // == list_n
        const int c_above = c_up;
        uint32_t ckey[kCompact];
#pragma unroll
        for (int e = 0; e < kCompact; ++e) {
            const int i = tid + e * kSelThreads;
            ckey[e] = i < n_und ? short_list[i] : 0u;
        }
        for (--bit; bit >= 0; --bit) {
            const uint32_t trial = T | (1u << bit);
            int c = 0;
#pragma unroll
            for (int e = 0; e < kCompact; ++e) c += (tid + e * kSelThreads < n_und && ckey[e] >= trial) ? 1 : 0;
            const int t = c_above + block_count(c, slots, parity);
            parity ^= 1;
            if (t >= want) T = trial; else c_up = t;
        }
    }
    const int need_eq = want - c_up;

    int gt_base = 0, eq_base = 0;                    // tokens > T and == T in the rounds before this one
    for (int base = 0; base < n_cand; base += 32 * kSelThreads) {
        const int j0 = base + tid * 32;
        uint32_t mg = 0, me = 0;
        float f[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) f[u] = s[min(j0 + u, n_cand - 1)];
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const uint32_t key = order_key(f[u]);
            const bool live = j0 + u < n_cand;
            mg |= (live && key > T ? 1u : 0u) << u;
            me |= (live && key == T ? 1u : 0u) << u;
        }
        int gt_before, eq_before;
        block_exscan2(__builtin_popcount(mg), __builtin_popcount(me), slots + 2 * kSelWaves, gt_before, eq_before);
        int gt_round = 0, eq_round = 0;
        for (int w = 0; w < kSelWaves; ++w) { gt_round += slots[2 * kSelWaves + w]; eq_round += slots[3 * kSelWaves + w]; }
        gt_before += gt_base;
        eq_before += eq_base;
        uint32_t m = mg | me;
        while (m) {
            const int bpos = __builtin_ctz(m);
            m &= m - 1;
            if ((mg >> bpos) & 1u) {
                out[gt_before + min(eq_before, need_eq)] = j0 + bpos;
                ++gt_before;
            } else {
                if (eq_before < need_eq) out[gt_before + eq_before] = j0 + bpos;
                ++eq_before;
            }
        }
        gt_base += gt_round;
        eq_base += eq_round;
        __syncthreads();                             // the scan slots are rewritten by the next round
    }
}

}  // namespace

bool select_supported(int L) { return L >= 1; }

hipError_t launch_select(const Geom& g, const float* scores, const int32_t* budgets, const int32_t* cu_budgets,
                         const int32_t* cu_seqlens, int max_L, int32_t* indices, hipStream_t s)
{
    const int n_heads = g.n_items * g.H_kv;
    const int ept_needed = (max_L + kSelThreads - 1) / kSelThreads;
#define AUDIOKV_LAUNCH_SELECT(E)                                                                        \
    do {                                                                                                \
        hipLaunchKernelGGL((select_kernel<E>), dim3(n_heads), dim3(kSelThreads), 0, s, g, scores,       \
                           budgets, cu_budgets, cu_seqlens, indices);                                   \
    } while (0)
    if (ept_needed <= 4) AUDIOKV_LAUNCH_SELECT(4);
    else if (ept_needed <= 8) AUDIOKV_LAUNCH_SELECT(8);
    else if (ept_needed <= 16) AUDIOKV_LAUNCH_SELECT(16);
    else if (ept_needed <= 32) AUDIOKV_LAUNCH_SELECT(32);
    else   // longer heads than the registers and the LDS staging of one workgroup hold
        hipLaunchKernelGGL(select_stream_kernel, dim3(n_heads), dim3(kSelThreads), 0, s, g, scores, budgets, cu_budgets,
                           cu_seqlens, indices);
#undef AUDIOKV_LAUNCH_SELECT
    return hipGetLastError();
}

}  // namespace audiokv
