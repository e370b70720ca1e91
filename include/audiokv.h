/*
 * audiokv.h - C ABI of the MI355X (gfx950) implementation of AudioKV's
 * prefill-time KV-cache eviction path.
 *
 * The path, per (sequence, layer) "item":
 *   1. score     observation-window importance of every cached token
 *   2. allocate  per-KV-head cache budgets from head criticality weights
 *   3. smooth    Spectral Score Smoothing of each head's score sequence
 *   4. select    per-head top-k at the allocated budget
 *   5. compact   gather of the retained K/V rows into a packed cache
 * plus audiokv_evict, which runs 1-5 in one call.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * - Plain C. Every function returns an int32 status: AUDIOKV_OK (0) or a
 *   negative AUDIOKV_E_* code; audiokv_last_error() gives the text of the last
 *   failure on the calling thread (library-owned, valid until the next call).
 * - "device" pointers are HIP device memory owned by the caller; "host"
 *   pointers are ordinary host memory. The library allocates no device memory
 *   and keeps no data between calls: scratch comes from the caller's
 *   `workspace` (size from audiokv_workspace_bytes). (audiokv_evict owns one
 *   helper stream and two events, see there.)
 * - Calls validate their arguments on the host, enqueue kernels on `stream`
 *   (a hipStream_t passed as void*; NULL = the default stream) and return
 *   without synchronising. Inputs, outputs and workspace must stay alive, and
 *   the workspace must not be shared with a concurrent call, until the stream
 *   has drained. On a validation error nothing is enqueued.
 * - An empty batch (n_items = 0) is accepted by every entry point: the call
 *   returns AUDIOKV_OK and enqueues nothing (sizes come back as 0).
 * - Deterministic: equal inputs give bit-identical outputs.
 *
 * Batch layout
 * ------------
 * A call handles `n_items` items. Item i has L_i cached tokens;
 * `seqlens_host[i] = L_i` (host, int32) and `cu_seqlens_dev[i]` (device, int32,
 * n_items + 1 entries) is the exclusive prefix sum of the L_i. Heads are
 * numbered globally: head (i, h) has index i * n_kv_heads + h.
 *   K, V    bf16. Item i starts at element cu_seqlens[i] * n_kv_heads * head_dim.
 *           kv_layout 0: item block is [n_kv_heads][L_i][head_dim];
 *           kv_layout 1: item block is [L_i][n_kv_heads][head_dim].
 *           Any other arrangement with contiguous rows: explicit strides in
 *           audiokv_params (kv_stride_item / _head / _tok).
 *   q_win   bf16 [n_items][n_q_heads][window][head_dim]: the queries of the
 *           last `window` prompt positions (row w sits at position L_i - window + w).
 *           Query head q belongs to KV head q / (n_q_heads / n_kv_heads).
 *   scores  fp32; head (i, h) occupies L_i floats starting at
 *           cu_seqlens[i] * n_kv_heads + h * L_i.
 *   budgets int32 [n_heads]; cu_budgets int32 [n_heads + 1] (exclusive scan).
 *   indices int32 [sum of budgets]; head g's kept token indices (within its
 *           item, ascending) start at cu_budgets[g].
 *   k_out, v_out  bf16 [sum of budgets][head_dim], row t of head g at
 *           cu_budgets[g] + t.
 */
#ifndef AUDIOKV_H
#define AUDIOKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AUDIOKV_OK                     0
#define AUDIOKV_E_INVALID_ARG        (-1)  /* null pointer, inconsistent sizes, parameter out of range */
#define AUDIOKV_E_UNSUPPORTED        (-2)  /* valid request outside what the kernels implement */
#define AUDIOKV_E_WORKSPACE_TOO_SMALL (-3)
#define AUDIOKV_E_HIP                (-4)  /* a HIP runtime call failed */

#define AUDIOKV_POOL_AVG 0
#define AUDIOKV_POOL_MAX 1

#define AUDIOKV_LAYOUT_HEAD_MAJOR  0   /* [H_kv][L][d] per item */
#define AUDIOKV_LAYOUT_TOKEN_MAJOR 1   /* [L][H_kv][d] per item */

#define AUDIOKV_CUTOFF_FRACTION     0  /* k* = floor(cutoff * floor(L/2)): a fixed fraction of the bins            */
#define AUDIOKV_CUTOFF_ENERGY       1  /* smallest k* whose cumulative spectral energy reaches cutoff * total      */
#define AUDIOKV_CUTOFF_ENERGY_NO_DC 2  /* the same with both sums starting at bin 1 (k* >= 1)                      */

#define AUDIOKV_SCOPE_ITEM   0  /* each item's heads share that item's budget pool        */
#define AUDIOKV_SCOPE_GLOBAL 1  /* all heads of all items share one pool (equal L required) */

/* Static description of the attention geometry and of the scoring options.
 * Set `size = sizeof(audiokv_params)`; a mismatch is AUDIOKV_E_INVALID_ARG. */
typedef struct audiokv_params {
    uint32_t size;
    int32_t  n_q_heads;      /* H_q, a multiple of n_kv_heads                          */
    int32_t  n_kv_heads;     /* H_kv                                                   */
    int32_t  head_dim;       /* d: 64, 128 or 256                                      */
    int32_t  window;         /* W >= 1: observation window, also the forced-kept tail  */
    int32_t  pool_kernel;    /* odd >= 1; 1 disables pooling                           */
    int32_t  pool_mode;      /* AUDIOKV_POOL_AVG (zero padding, divisor = kernel) or _MAX */
    int32_t  causal;         /* 1: window row w sees keys j <= L - W + w; 0: all keys  */
    int32_t  kv_layout;      /* AUDIOKV_LAYOUT_*                                       */
    float    softmax_scale;  /* 0 selects 1/sqrt(head_dim)                             */
    float    floor_frac;     /* beta in [0,1]: uniform floor r = floor(beta*(n_keep-W))*/
    int32_t  cutoff_mode;    /* AUDIOKV_CUTOFF_*: how the `cutoff_frac` argument of smooth / evict sets k* */
    int32_t  taper_bins;     /* T >= 0: bins of cosine roll-off after k* (0: hard mask) */
    /* Explicit K/V strides, in elements; all three 0 (the default) selects the packed layout of `kv_layout`.
     * Otherwise token j of KV head h of item i starts at element
     *     i * kv_stride_item + h * kv_stride_head + j * kv_stride_tok
     * of both `k` and `v` (kv_layout is then ignored; cu_seqlens still gives the lengths and the layout of the
     * scores). A row is head_dim contiguous elements; every stride must be a multiple of 8 elements (rows are
     * moved as 16-byte vectors), kv_stride_tok >= head_dim, and kv_stride_item > 0 when n_items > 1. Rows of
     * different (item, head, token) must not overlap. This is how a padded prefill cache [B][H_kv][L_max][d]
     * (kv_stride_item = H_kv*L_max*d, kv_stride_head = L_max*d, kv_stride_tok = d) or a slice of a larger
     * buffer is passed without a copy. Used by score, compact, evict (and their variants); q_win, the outputs
     * and the compacted cache read by decode_attend are always packed. */
    int64_t  kv_stride_item;
    int64_t  kv_stride_head;
    int64_t  kv_stride_tok;
} audiokv_params;

/* Packed version: major * 10000 + minor * 100 + patch. */
int32_t audiokv_version(void);

/* Text of the last error on this thread ("" if none). Never NULL. */
const char* audiokv_last_error(void);

/* Host-only helper: n_keep = floor(ratio * L + 0.5), the per-head mean number
 * of kept tokens. Budgets of a pool of n heads sum to exactly n_keep * n. */
int32_t audiokv_n_keep(double ratio, int32_t L);

/* Host-only: total kept rows (sum of all budgets) for a batch, known before
 * any kernel runs because budgets sum exactly to n_keep per head on average:
 * sum_i n_keep(ratio, L_i) * n_kv_heads. Sizes indices / k_out / v_out. */
int32_t audiokv_total_kept(const audiokv_params* params, int32_t n_items,
                           const int32_t* seqlens_host, double ratio, int64_t* out_rows);

/* Host-only: bytes of device workspace that any entry point needs for this
 * batch (one size covers all of them, audiokv_evict included). No GPU call. */
int32_t audiokv_workspace_bytes(const audiokv_params* params, int32_t n_items,
                                const int32_t* seqlens_host, size_t* out_bytes);

/* Stage 1 - observation-window importance score (paper Sec. 3.3: the per-head
 * importance sequence s in R^L, attention averaged over an observation window;
 * Sec. 2: local pooling of such scores).
 * For KV head h: every query head q of its group and window row w gives
 * P = softmax_j(scale * <q_win[q,w], K[h,j]>) over the keys it may see;
 * raw[h,j] = sum_{q,w} P[j]; scores[h,j] = pool(raw[h])[j].
 * Arithmetic: bf16 inputs, fp32 accumulation (MFMA), fp32 softmax.
 * Requires L_i >= window for every item. */
int32_t audiokv_score(const audiokv_params* params,
                      const void* q_win, const void* k,
                      const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                      float* scores,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Stage 1 when the row statistics already exist (same passage as
 * audiokv_score). The prefill attention kernel that ran the last `window`
 * queries normally returns, per query row, the log-sum-exp of its scaled
 * logits; given those, the first of the two passes over K (which only
 * rebuilds them) is skipped. lse_dev: fp32 [n_items][n_q_heads][window],
 * natural log of sum_j exp(scale * <q, K[j]>) over the keys the row may see
 * (the same mask and scale as params). Everything else as audiokv_score; the
 * scores match audiokv_score to the accuracy of the supplied values. */
int32_t audiokv_score_lse(const audiokv_params* params,
                          const void* q_win, const void* k, const float* lse_dev,
                          const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                          float* scores,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Stage 2 - head-wise budget allocation (paper Sec. 3.1 Eq. 1:
 * b = w + r + B_score * S / sum S; Sec. 3.2 Eq. 12: floor of the proportional
 * share), made to sum exactly to the pool total.
 * Heads are split into `n_segments` pools of `heads_per_segment` consecutive
 * heads; pool s has sequence length seqlens_host[s] (= cu_seqlens_dev[s+1] -
 * cu_seqlens_dev[s]). Per-sequence budgets: n_segments = n_items,
 * heads_per_segment = n_kv_heads. The paper's global form over all layers of
 * one sequence: n_segments = 1, heads_per_segment = layers * n_kv_heads.
 * weights_dev: fp32 >= 0, [n_segments * heads_per_segment * weight_group];
 * weight_group > 1 means weights are per query head and are summed within
 * each group of `weight_group` consecutive entries first.
 * Per pool (float64 on the device, same operation order as the reference
 * definition): n_keep = floor(ratio*L + .5); f = W + floor(beta*(n_keep - W));
 * shares of n*(n_keep - f) proportional to S, capped at L - f with the excess
 * re-spread over uncapped heads; floors; leftover units to the largest
 * fractional parts (ties: lower head). b_h = f + share_h in [f, L].
 * cu_budgets is the exclusive scan over ALL heads of the call. Requires
 * W <= n_keep <= L, ratio in (0, 1]. */
int32_t audiokv_allocate(const audiokv_params* params,
                         const float* weights_dev,
                         int32_t n_segments, int32_t heads_per_segment, int32_t weight_group,
                         const int32_t* cu_seqlens_dev, const int32_t* seqlens_host,
                         double ratio,
                         int32_t* budgets_dev, int32_t* cu_budgets_dev, void* stream);

/* Stage 3 - Spectral Score Smoothing (paper Sec. 3.3, Eqs. 13-20):
 * F = RFFT(s) over exactly L_i points; F~ = F * w; s~ = IRFFT(F~, L_i);
 * out = (1-alpha) s + alpha s~. The mask w (Eqs. 17-18) keeps bins i <= k*,
 * rolls off over the next params->taper_bins bins as
 * w_i = (1 + cos(pi (i - k*) / (T + 1))) / 2 (the cosine transition band
 * mentioned after Eq. 17; T = 0 is the hard mask) and is zero beyond.
 * params->cutoff_mode chooses k*:
 *   AUDIOKV_CUTOFF_FRACTION  k* = floor(cutoff_frac * floor(L_i/2)),
 *                            cutoff_frac in [0,1] (1 keeps every bin: identity);
 *   AUDIOKV_CUTOFF_ENERGY    Eqs. 14-16: the smallest k* with
 *                            sum_{i<=k*} |F_i|^2 >= cutoff_frac * sum_i |F_i|^2
 *                            over the one-sided spectrum, per head, cutoff_frac
 *                            (the ratio rho of Eq. 16) in (0,1]; energies are
 *                            fp32 squares accumulated in float64;
 *   AUDIOKV_CUTOFF_ENERGY_NO_DC  the same with both sums starting at bin 1.
 * alpha in [0,1] (0: bitwise copy). scores_out may alias scores_in. fp32
 * arithmetic with float64-generated twiddles. Lengths up to 131072 (longer:
 * AUDIOKV_E_UNSUPPORTED unless alpha = 0); lengths that are not powers of two,
 * and all lengths above 32768, need the workspace. */
int32_t audiokv_smooth(const audiokv_params* params,
                       const float* scores_in,
                       const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                       double cutoff_frac, double alpha,
                       float* scores_out,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The cutoff bin k* that audiokv_smooth would use for every head, without the
 * filtering (paper Sec. 3.3, Eqs. 14-16 for the energy modes): kstar_dev is
 * int32 [n_items * n_kv_heads] on the device. Same arguments, lengths and
 * workspace as audiokv_smooth. */
int32_t audiokv_smooth_cutoffs(const audiokv_params* params,
                               const float* scores_in,
                               const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                               double cutoff_frac,
                               int32_t* kstar_dev,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Stage 4 - per-head top-k (paper Sec. 1, Solution 2: Top-K selection on the
 * importance scores). Head g keeps budgets[g] tokens: the last `window`
 * positions always, and the budgets[g] - window highest scores among positions
 * [0, L - window); equal scores (-0 == +0) go to the lower index. Indices are
 * written ascending. Scores must be finite. Requires
 * window <= budgets[g] <= L (not checked on the device beyond clamping). */
int32_t audiokv_select(const audiokv_params* params,
                       const float* scores,
                       const int32_t* budgets_dev, const int32_t* cu_budgets_dev,
                       const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                       int32_t* indices_dev,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Stage 5 - compaction (paper Sec. 1 / Sec. 4.6: only retained tokens stay in
 * the cache). Copies row indices[cu_budgets[g] + t] of head g's K and V to
 * row cu_budgets[g] + t of k_out / v_out, bit for bit. total_rows = sum of
 * budgets (host value, see audiokv_total_kept). */
int32_t audiokv_compact(const audiokv_params* params,
                        const void* k, const void* v,
                        const int32_t* indices_dev, const int32_t* cu_budgets_dev,
                        const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                        int64_t total_rows,
                        void* k_out, void* v_out, void* stream);

/* Stages 1-5 in one call on one stream. `alloc_scope` chooses the budget
 * pools (AUDIOKV_SCOPE_ITEM: per item; AUDIOKV_SCOPE_GLOBAL: one pool over all
 * n_items * n_kv_heads heads, all L_i equal). weights_dev: fp32
 * [n_items * n_kv_heads], one per KV head. Intermediate scores live in the
 * workspace. Outputs as in the per-stage calls; the result equals the five
 * calls composed. The budget allocation does not depend on the scores, nor do
 * the tables that smoothing needs for lengths that are not powers of two: for
 * pools of 32 heads or more, or when such tables are needed, they are forked
 * onto a helper stream owned by the library (created on first use, default
 * priority) and joined back into `stream` with events after the scoring
 * (smaller pools are allocated on `stream` itself, in the launch that merges
 * the softmax statistics between the two scoring sweeps); everything is
 * ordered after prior work on
 * `stream` and before later work on it. Calls on different streams may be in
 * flight together (separate workspaces and outputs), also from several host
 * threads: the helper stream and its two events are shared, so the part of a
 * call between the fork and the join holds a lock. */
int32_t audiokv_evict(const audiokv_params* params,
                      const void* q_win, const void* k, const void* v,
                      const float* weights_dev, int32_t alloc_scope,
                      const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                      double ratio, double cutoff_frac, double alpha,
                      void* k_out, void* v_out, int32_t* indices_dev,
                      int32_t* budgets_dev, int32_t* cu_budgets_dev,
                      void* workspace, size_t workspace_bytes, void* stream);

/* audiokv_evict with the window rows' log-sum-exp supplied (see
 * audiokv_score_lse): identical otherwise, one pass over K instead of two. */
int32_t audiokv_evict_lse(const audiokv_params* params,
                          const void* q_win, const void* k, const void* v, const float* lse_dev,
                          const float* weights_dev, int32_t alloc_scope,
                          const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                          double ratio, double cutoff_frac, double alpha,
                          void* k_out, void* v_out, int32_t* indices_dev,
                          int32_t* budgets_dev, int32_t* cu_budgets_dev,
                          void* workspace, size_t workspace_bytes, void* stream);

/* audiokv_evict for callers that cannot allocate device memory or pass a workspace: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation. Same arguments and same results as audiokv_evict,
 * without `workspace`: the scratch is a static device array of AUDIOKV_NOALLOC_SCRATCH_BYTES inside the library
 * (every GPU the library runs on holds its own copy until the process ends). A batch whose
 * audiokv_workspace_bytes exceeds that size is rejected with AUDIOKV_E_WORKSPACE_TOO_SMALL and nothing is enqueued
 * (one layer of 4 KV heads x 32768 tokens needs about 1.2 MB). The call creates no stream or event and calls no
 * allocating routine; all kernels, the budget allocation included, go to `stream` in order. The array is shared by
 * all calls on a GPU: calls whose kernels may overlap on one GPU (different streams or host threads) race on it and
 * must be serialised by the caller. Nothing in it needs to start at zero: every kernel writes what it later reads. */
#define AUDIOKV_NOALLOC_SCRATCH_BYTES (8u << 20)
int32_t audiokv_evict_noalloc(const audiokv_params* params,
                              const void* q_win, const void* k, const void* v,
                              const float* weights_dev, int32_t alloc_scope,
                              const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                              double ratio, double cutoff_frac, double alpha,
                              void* k_out, void* v_out, int32_t* indices_dev,
                              int32_t* budgets_dev, int32_t* cu_budgets_dev,
                              void* stream);

/* The step after the path: one decoding step on the compacted cache (paper
 * Sec. 1 and Sec. 4.6: generation proceeds on the retained tokens only).
 * q_dev: bf16 [n_items][n_q_heads][head_dim], one new query per head;
 * k_cache / v_cache / cu_budgets_dev: as written by audiokv_compact /
 * audiokv_evict. out_dev: fp32 [n_items][n_q_heads][head_dim],
 *   out[i][j] = sum_t softmax_t(scale * <q[i][j], K_g[t]>) * V_g[t]
 * over the budgets[g] rows of KV head g = i * n_kv_heads + j / (n_q_heads /
 * n_kv_heads). total_rows (host) is the sum of all budgets
 * (audiokv_total_kept): it sizes the launch and the workspace
 * (audiokv_decode_workspace_bytes); cache rows at or beyond total_rows are
 * never read. A head with budget 0 yields zeros. n_q_heads / n_kv_heads <= 16. */
int32_t audiokv_decode_workspace_bytes(const audiokv_params* params, int32_t n_items, int64_t total_rows,
                                       size_t* out_bytes);
int32_t audiokv_decode_attend(const audiokv_params* params,
                              const void* q_dev, const void* k_cache, const void* v_cache,
                              const int32_t* cu_budgets_dev, int32_t n_items, int64_t total_rows,
                              float* out_dev,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid, not part of the method (used by the benchmark to time the
 * kernels of audiokv_evict where they run). While enabled, audiokv_evict records
 * HIP events on the caller's stream between its kernels; audiokv_profile_read
 * waits for the most recent such call to finish and writes the elapsed
 * milliseconds of each interval to ms_out[AUDIOKV_PROFILE_STAGES] (host):
 * 0 allocate, 1 score sweep 1 (row statistics), 2 score sweep 2 (column sums),
 * 3 pooling + spectral smoothing, 4 select, 5 compact. Process-wide state (the
 * events are created by the first enable and kept); not thread-safe. */
#define AUDIOKV_PROFILE_STAGES 6
int32_t audiokv_profile_enable(int32_t enable);
int32_t audiokv_profile_read(float* ms_out);

#ifdef __cplusplus
}
#endif
#endif /* AUDIOKV_H */
