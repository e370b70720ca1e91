// The C ABI of include/audiokv.h: host-side validation, workspace carving and
// kernel enqueues. Nothing here allocates device memory or synchronises.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "common.h"

using namespace audiokv;

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int32_t hip_fail(hipError_t e, const char* what) {
    return fail(AUDIOKV_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Batch {
    int n_items = 0;
    int max_L = 0, min_L = 0;
    long long total_tokens = 0;
    bool uniform = true;
};

// window_min: smallest legal window for the calling entry point (score needs >= 1, select accepts 0)
int32_t check_params(const audiokv_params* p, int window_min) {
    if (!p) return fail(AUDIOKV_E_INVALID_ARG, "params is NULL");
    if (p->size != sizeof(audiokv_params))
        return fail(AUDIOKV_E_INVALID_ARG, "params.size = %u, this library expects %zu", p->size, sizeof(audiokv_params));
    if (p->n_kv_heads < 1 || p->n_q_heads < 1 || p->n_q_heads % p->n_kv_heads != 0)
        return fail(AUDIOKV_E_INVALID_ARG, "n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)",
                    p->n_q_heads, p->n_kv_heads);
    if (p->head_dim != 64 && p->head_dim != 128 && p->head_dim != 256)
        return fail(AUDIOKV_E_UNSUPPORTED, "head_dim %d: only 64, 128 and 256 are built", p->head_dim);
    if (p->window < window_min) return fail(AUDIOKV_E_INVALID_ARG, "window %d < %d", p->window, window_min);
    if (p->pool_kernel < 1 || p->pool_kernel % 2 == 0 || p->pool_kernel > 1025)
        return fail(AUDIOKV_E_INVALID_ARG, "pool_kernel %d must be odd, in [1, 1025]", p->pool_kernel);
    if (p->pool_mode != AUDIOKV_POOL_AVG && p->pool_mode != AUDIOKV_POOL_MAX)
        return fail(AUDIOKV_E_INVALID_ARG, "pool_mode %d", p->pool_mode);
    if (p->cutoff_mode < AUDIOKV_CUTOFF_FRACTION || p->cutoff_mode > AUDIOKV_CUTOFF_ENERGY_NO_DC)
        return fail(AUDIOKV_E_INVALID_ARG, "cutoff_mode %d", p->cutoff_mode);
    if (p->taper_bins < 0) return fail(AUDIOKV_E_INVALID_ARG, "taper_bins %d must be >= 0", p->taper_bins);
    if (p->kv_layout != AUDIOKV_LAYOUT_HEAD_MAJOR && p->kv_layout != AUDIOKV_LAYOUT_TOKEN_MAJOR)
        return fail(AUDIOKV_E_INVALID_ARG, "kv_layout %d", p->kv_layout);
    if (p->causal != 0 && p->causal != 1) return fail(AUDIOKV_E_INVALID_ARG, "causal %d", p->causal);
    if (!(p->softmax_scale >= 0.f) || !std::isfinite(p->softmax_scale))
        return fail(AUDIOKV_E_INVALID_ARG, "softmax_scale must be finite and >= 0 (0 selects 1/sqrt(d))");
    if (!(p->floor_frac >= 0.f && p->floor_frac <= 1.f))
        return fail(AUDIOKV_E_INVALID_ARG, "floor_frac must lie in [0, 1]");
    if (p->kv_stride_tok != 0 || p->kv_stride_head != 0 || p->kv_stride_item != 0) {
        // explicit strides: rows stay contiguous in head_dim and 16-byte aligned
        if (p->kv_stride_tok < p->head_dim || p->kv_stride_head < 1 || p->kv_stride_item < 0)
            return fail(AUDIOKV_E_INVALID_ARG, "kv strides (item %lld, head %lld, token %lld): with explicit strides the "
                        "token stride must be >= head_dim, the head stride > 0 and the item stride >= 0",
                        (long long)p->kv_stride_item, (long long)p->kv_stride_head, (long long)p->kv_stride_tok);
        if (p->kv_stride_tok % 8 != 0 || p->kv_stride_head % 8 != 0 || p->kv_stride_item % 8 != 0)
            return fail(AUDIOKV_E_INVALID_ARG, "kv strides (item %lld, head %lld, token %lld) must be multiples of 8 "
                        "elements: K/V rows are moved as 16-byte vectors",
                        (long long)p->kv_stride_item, (long long)p->kv_stride_head, (long long)p->kv_stride_tok);
    }
    return AUDIOKV_OK;
}

int32_t check_batch(const audiokv_params* p, int32_t n_items, const int32_t* seqlens_host, Batch* b) {
    if (n_items < 1) return fail(AUDIOKV_E_INVALID_ARG, "n_items %d < 1", n_items);
    if (!seqlens_host) return fail(AUDIOKV_E_INVALID_ARG, "seqlens_host is NULL");
    b->n_items = n_items;
    b->max_L = 0;
    b->min_L = INT32_MAX;
    b->total_tokens = 0;
    for (int i = 0; i < n_items; ++i) {
        const int L = seqlens_host[i];
        if (L < 1 || L < p->window)
            return fail(AUDIOKV_E_INVALID_ARG, "item %d: length %d must be >= max(1, window = %d)", i, L, p->window);
        b->max_L = L > b->max_L ? L : b->max_L;
        b->min_L = L < b->min_L ? L : b->min_L;
        b->total_tokens += L;
    }
    b->uniform = b->max_L == b->min_L;
    if (p->kv_stride_tok != 0 && n_items > 1 && p->kv_stride_item == 0)
        return fail(AUDIOKV_E_INVALID_ARG, "explicit kv strides with %d items need kv_stride_item > 0", n_items);
    if (b->total_tokens * p->n_kv_heads > (long long)INT32_MAX)
        return fail(AUDIOKV_E_UNSUPPORTED, "batch too large: %lld tokens x %d heads exceeds 2^31 scores",
                    b->total_tokens, p->n_kv_heads);
    if ((long long)n_items * p->n_kv_heads > (1 << 20))
        return fail(AUDIOKV_E_UNSUPPORTED, "too many heads in one call");
    return AUDIOKV_OK;
}

Geom make_geom(const audiokv_params* p, int n_items) {
    Geom g;
    g.n_items = n_items;
    g.H_q = p->n_q_heads;
    g.H_kv = p->n_kv_heads;
    g.G = p->n_q_heads / p->n_kv_heads;
    g.D = p->head_dim;
    g.W = p->window;
    g.pool_kernel = p->pool_kernel;
    g.pool_mode = p->pool_mode;
    g.causal = p->causal;
    g.layout = p->kv_layout;
    const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / std::sqrt((float)p->head_dim);
    g.c_log2 = scale * 1.44269504088896340736f;
    g.cutoff_mode = p->cutoff_mode;
    g.taper_bins = p->taper_bins;
    g.s_item = p->kv_stride_item;
    g.s_head = p->kv_stride_head;
    g.s_tok = p->kv_stride_tok;
    return g;
}

struct Workspace {
    size_t stats_off = 0, raw_off = 0, raw2_off = 0, smooth_off = 0, fft_off = 0, total = 0;
    bool raw2 = false;
};

Workspace plan_workspace(const audiokv_params* p, const Batch& b, const int32_t* seqlens_host) {
    Workspace w;
    const int n_heads = b.n_items * p->n_kv_heads;
    const int rows = (p->n_q_heads / p->n_kv_heads) * (p->window > 0 ? p->window : 1);
    const int rows_pad = score_padded_rows(rows, p->head_dim);
    const int nsplit = score_num_splits(p->n_kv_heads, b.n_items, seqlens_host, rows, p->head_dim);
    size_t off = 0;
    w.stats_off = off;
    // partial row statistics [head][split][rows_pad][2], then the merged per-row constants [head][rows_pad]
    off += align_up((size_t)n_heads * (rows_pad > 0 ? rows_pad : 1) * (2 * (size_t)nsplit + 1) * sizeof(float), 256);
    w.raw_off = off;
    off += align_up((size_t)b.total_tokens * p->n_kv_heads * sizeof(float), 256);
    w.raw2 = score_needs_second_raw(rows, p->head_dim);     // second row range of a split sweep 2
    w.raw2_off = off;
    if (w.raw2) off += align_up((size_t)b.total_tokens * p->n_kv_heads * sizeof(float), 256);
    w.smooth_off = off;
    off += align_up((size_t)b.total_tokens * p->n_kv_heads * sizeof(float), 256);
    w.fft_off = off;          // arbitrary-length spectral smoothing (empty when every length is a power of two)
    off += align_up(smooth_workspace_bytes(seqlens_host, b.n_items, p->n_kv_heads), 256);
    w.total = off;
    return w;
}

int32_t check_ratio(const audiokv_params* p, const Batch& b, const int32_t* seqlens_host, double ratio) {
    if (!(ratio > 0.0 && ratio <= 1.0)) return fail(AUDIOKV_E_INVALID_ARG, "ratio %g must lie in (0, 1]", ratio);
    for (int i = 0; i < b.n_items; ++i) {
        const int nk = audiokv_n_keep(ratio, seqlens_host[i]);
        if (nk < p->window || nk > seqlens_host[i])
            return fail(AUDIOKV_E_INVALID_ARG,
                        "item %d: n_keep = round(%g * %d) = %d must lie in [window = %d, L]", i, ratio,
                        seqlens_host[i], nk, p->window);
    }
    return AUDIOKV_OK;
}

int32_t check_smooth_args(const audiokv_params* p, double cutoff_frac, double alpha) {
    if (!(cutoff_frac >= 0.0 && cutoff_frac <= 1.0)) return fail(AUDIOKV_E_INVALID_ARG, "cutoff_frac %g must lie in [0, 1]", cutoff_frac);
    if (p->cutoff_mode != AUDIOKV_CUTOFF_FRACTION && !(cutoff_frac > 0.0))
        return fail(AUDIOKV_E_INVALID_ARG, "energy ratio %g must lie in (0, 1]", cutoff_frac);
    if (!(alpha >= 0.0 && alpha <= 1.0)) return fail(AUDIOKV_E_INVALID_ARG, "alpha %g must lie in [0, 1]", alpha);
    return AUDIOKV_OK;
}

int32_t check_smooth_lengths(const Batch& b, const int32_t* seqlens_host, double alpha) {
    if (alpha == 0.0) return AUDIOKV_OK;
    for (int i = 0; i < b.n_items; ++i)
        if (!smooth_supported(seqlens_host[i]))
            return fail(AUDIOKV_E_UNSUPPORTED, "item %d: spectral smoothing of length %d is not built "
                        "(lengths up to 131072)", i, seqlens_host[i]);
    return AUDIOKV_OK;
}

int32_t check_score_shape(const audiokv_params* p) {
    const int rows = (p->n_q_heads / p->n_kv_heads) * p->window;
    if (score_padded_rows(rows, p->head_dim) == 0)
        return fail(AUDIOKV_E_UNSUPPORTED, "group * window = %d rows at head_dim %d exceeds what the score kernels hold "
                    "in registers (576 rows at d <= 128, 256 rows at d = 256)", rows, p->head_dim);
    return AUDIOKV_OK;
}

// stage timing for the benchmark: events 0..6 bracket the six kernels of audiokv_evict
struct Profile {
    bool enabled = false;
    bool created = false;
    bool recorded = false;
    hipEvent_t ev[AUDIOKV_PROFILE_STAGES + 2] = {};    // last slot: between the two score sweeps
} g_prof;

// audiokv_evict forks the (tiny, score-independent) allocation onto a helper stream so that it runs under the
// score kernels instead of in front of them. Created on first use, kept for the life of the process.
struct Helper {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    std::mutex mu;      // one fork ... join sequence at a time: the stream and the two events are shared by all callers
} g_helper;

hipError_t ensure_helper() {        // called with g_helper.mu held
    if (g_helper.stream) return hipSuccess;
    hipError_t e = hipStreamCreateWithFlags(&g_helper.stream, hipStreamNonBlocking);   // default priority
    if (e == hipSuccess) e = hipEventCreateWithFlags(&g_helper.fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&g_helper.join, hipEventDisableTiming);
    return e;
}

#define AUDIOKV_TRY(expr)                  \
    do {                                   \
        const int32_t rc__ = (expr);       \
        if (rc__ != AUDIOKV_OK) return rc__; \
    } while (0)
#define AUDIOKV_HIP(expr, what)                      \
    do {                                             \
        const hipError_t e__ = (expr);               \
        if (e__ != hipSuccess) return hip_fail(e__, what); \
    } while (0)

}  // namespace

extern "C" {

int32_t audiokv_version(void) { return 100; }   // 0.1.0

const char* audiokv_last_error(void) { return g_err; }

int32_t audiokv_n_keep(double ratio, int32_t L) {
    volatile double prod = ratio * (double)L;    // volatile: no fused multiply-add on the host either
    return (int32_t)std::floor(prod + 0.5);
}

int32_t audiokv_total_kept(const audiokv_params* params, int32_t n_items, const int32_t* seqlens_host,
                           double ratio, int64_t* out_rows)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (!out_rows) return fail(AUDIOKV_E_INVALID_ARG, "out_rows is NULL");
    if (n_items == 0) { *out_rows = 0; return AUDIOKV_OK; }
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    AUDIOKV_TRY(check_ratio(params, b, seqlens_host, ratio));
    int64_t tot = 0;
    for (int i = 0; i < n_items; ++i) tot += (int64_t)audiokv_n_keep(ratio, seqlens_host[i]) * params->n_kv_heads;
    *out_rows = tot;
    return AUDIOKV_OK;
}

int32_t audiokv_workspace_bytes(const audiokv_params* params, int32_t n_items, const int32_t* seqlens_host,
                                size_t* out_bytes)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (!out_bytes) return fail(AUDIOKV_E_INVALID_ARG, "out_bytes is NULL");
    if (n_items == 0) { *out_bytes = 0; return AUDIOKV_OK; }
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    *out_bytes = plan_workspace(params, b, seqlens_host).total;
    return AUDIOKV_OK;
}

namespace {
int32_t score_entry(const audiokv_params* params, const void* q_win, const void* k, const float* lse_dev,
                    const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                    float* scores, void* workspace, size_t workspace_bytes, void* stream)
{
    AUDIOKV_TRY(check_params(params, 1));
    if (n_items == 0) return AUDIOKV_OK;           // an empty batch: nothing to enqueue
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    if (!q_win || !k || !cu_seqlens_dev || !scores || !workspace)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_score: NULL pointer argument");
    if (!aligned16(q_win) || !aligned16(k)) return fail(AUDIOKV_E_INVALID_ARG, "q_win and k must be 16-byte aligned");
    AUDIOKV_TRY(check_score_shape(params));
    const Workspace w = plan_workspace(params, b, seqlens_host);
    if (workspace_bytes < w.total)
        return fail(AUDIOKV_E_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
    const Geom g = make_geom(params, n_items);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    float* stats = reinterpret_cast<float*>(ws + w.stats_off);
    float* raw = params->pool_kernel == 1 ? scores : reinterpret_cast<float*>(ws + w.raw_off);
    AUDIOKV_HIP(launch_score(g, q_win, k, cu_seqlens_dev, seqlens_host, stats, raw, s, nullptr, lse_dev,
                             w.raw2 ? reinterpret_cast<float*>(ws + w.raw2_off) : nullptr,
                             (size_t)b.total_tokens * params->n_kv_heads), "score kernels");
    if (params->pool_kernel != 1)
        AUDIOKV_HIP(launch_pool(g, raw, cu_seqlens_dev, b.max_L, scores, s), "pool kernel");
    return AUDIOKV_OK;
}
}  // namespace

int32_t audiokv_score(const audiokv_params* params, const void* q_win, const void* k,
                      const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                      float* scores, void* workspace, size_t workspace_bytes, void* stream)
{
    return score_entry(params, q_win, k, nullptr, cu_seqlens_dev, seqlens_host, n_items, scores, workspace,
                       workspace_bytes, stream);
}

int32_t audiokv_score_lse(const audiokv_params* params, const void* q_win, const void* k, const float* lse_dev,
                          const int32_t* cu_seqlens_dev, const int32_t* seqlens_host, int32_t n_items,
                          float* scores, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!lse_dev && n_items != 0) return fail(AUDIOKV_E_INVALID_ARG, "audiokv_score_lse: NULL lse_dev");
    return score_entry(params, q_win, k, lse_dev, cu_seqlens_dev, seqlens_host, n_items, scores, workspace,
                       workspace_bytes, stream);
}

int32_t audiokv_allocate(const audiokv_params* params, const float* weights_dev, int32_t n_segments,
                         int32_t heads_per_segment, int32_t weight_group, const int32_t* cu_seqlens_dev,
                         const int32_t* seqlens_host, double ratio, int32_t* budgets_dev,
                         int32_t* cu_budgets_dev, void* stream)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (n_segments == 0) return AUDIOKV_OK;
    if (n_segments < 1 || heads_per_segment < 1 || weight_group < 1)
        return fail(AUDIOKV_E_INVALID_ARG, "n_segments, heads_per_segment and weight_group must be >= 1");
    if (heads_per_segment > 1536)
        return fail(AUDIOKV_E_UNSUPPORTED, "heads_per_segment %d > 1536", heads_per_segment);
    if (!weights_dev || !cu_seqlens_dev || !seqlens_host || !budgets_dev || !cu_budgets_dev)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_allocate: NULL pointer argument");
    if (!(ratio > 0.0 && ratio <= 1.0)) return fail(AUDIOKV_E_INVALID_ARG, "ratio %g must lie in (0, 1]", ratio);
    long long total = 0;
    for (int s2 = 0; s2 < n_segments; ++s2) {
        const int L = seqlens_host[s2];
        if (L < 1) return fail(AUDIOKV_E_INVALID_ARG, "segment %d: length %d", s2, L);
        const int nk = audiokv_n_keep(ratio, L);
        if (nk < params->window || nk > L)
            return fail(AUDIOKV_E_INVALID_ARG, "segment %d: n_keep = %d must lie in [window = %d, L = %d]", s2, nk,
                        params->window, L);
        total += (long long)nk * heads_per_segment;
    }
    if (total > (long long)INT32_MAX) return fail(AUDIOKV_E_UNSUPPORTED, "sum of budgets exceeds 2^31");
    const Geom g = make_geom(params, n_segments);
    AUDIOKV_HIP(launch_allocate(g, weights_dev, n_segments, heads_per_segment, weight_group, cu_seqlens_dev, ratio,
                                (double)params->floor_frac, budgets_dev, cu_budgets_dev,
                                static_cast<hipStream_t>(stream)),
                "allocate kernel");
    return AUDIOKV_OK;
}

namespace {
int32_t smooth_entry(const audiokv_params* params, const float* scores_in, const int32_t* cu_seqlens_dev,
                     const int32_t* seqlens_host, int32_t n_items, double cutoff_frac, double alpha,
                     float* scores_out, int32_t* kstar_dev, bool cutoffs_only, void* workspace,
                     size_t workspace_bytes, void* stream)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (n_items == 0) return AUDIOKV_OK;
    audiokv_params p2 = *params;
    p2.window = 0;                                // lengths are not tied to the window here
    Batch b;
    AUDIOKV_TRY(check_batch(&p2, n_items, seqlens_host, &b));
    if (!scores_in || !cu_seqlens_dev || (cutoffs_only ? !kstar_dev : !scores_out))
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_smooth: NULL pointer argument");
    AUDIOKV_TRY(check_smooth_args(params, cutoff_frac, alpha));
    AUDIOKV_TRY(check_smooth_lengths(b, seqlens_host, alpha));
    void* fft_ws = nullptr;
    const size_t fft_bytes = alpha != 0.0 ? smooth_workspace_required(seqlens_host, n_items, params->n_kv_heads) : 0;
    if (workspace && alpha != 0.0) fft_ws = workspace;      // optional room beyond the required part is put to use
    if (fft_bytes > 0) {
        // the stand-alone call uses the transform's scratch only, carved from the start of the workspace: whatever
        // audiokv_workspace_bytes returns for the batch covers it (that size also holds the scores of the fused path)
        if (!workspace || workspace_bytes < fft_bytes)
            return fail(AUDIOKV_E_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed (lengths that are not powers "
                        "of two use a global-memory transform)", workspace ? workspace_bytes : (size_t)0, fft_bytes);
        fft_ws = workspace;
    }
    const Geom g = make_geom(params, n_items);
    AUDIOKV_HIP(launch_smooth(g, scores_in, false, cu_seqlens_dev, seqlens_host, n_items, cutoff_frac, alpha,
                              scores_out, fft_ws, fft_ws ? workspace_bytes : (size_t)0, kstar_dev, cutoffs_only,
                              static_cast<hipStream_t>(stream)),
                "smooth kernel");
    return AUDIOKV_OK;
}
}  // namespace

int32_t audiokv_smooth(const audiokv_params* params, const float* scores_in, const int32_t* cu_seqlens_dev,
                       const int32_t* seqlens_host, int32_t n_items, double cutoff_frac, double alpha,
                       float* scores_out, void* workspace, size_t workspace_bytes, void* stream)
{
    return smooth_entry(params, scores_in, cu_seqlens_dev, seqlens_host, n_items, cutoff_frac, alpha, scores_out,
                        nullptr, false, workspace, workspace_bytes, stream);
}

int32_t audiokv_smooth_cutoffs(const audiokv_params* params, const float* scores_in, const int32_t* cu_seqlens_dev,
                               const int32_t* seqlens_host, int32_t n_items, double cutoff_frac,
                               int32_t* kstar_dev, void* workspace, size_t workspace_bytes, void* stream)
{
    // alpha = 1: the transform has to run for the energy modes
    return smooth_entry(params, scores_in, cu_seqlens_dev, seqlens_host, n_items, cutoff_frac, 1.0, nullptr,
                        kstar_dev, true, workspace, workspace_bytes, stream);
}

int32_t audiokv_select(const audiokv_params* params, const float* scores, const int32_t* budgets_dev,
                       const int32_t* cu_budgets_dev, const int32_t* cu_seqlens_dev, const int32_t* seqlens_host,
                       int32_t n_items, int32_t* indices_dev, void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    AUDIOKV_TRY(check_params(params, 0));
    if (n_items == 0) return AUDIOKV_OK;
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    if (!scores || !budgets_dev || !cu_budgets_dev || !cu_seqlens_dev || !indices_dev)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_select: NULL pointer argument");
    if (!select_supported(b.max_L))
        return fail(AUDIOKV_E_UNSUPPORTED, "select: length %d is not supported", b.max_L);
    const Geom g = make_geom(params, n_items);
    AUDIOKV_HIP(launch_select(g, scores, budgets_dev, cu_budgets_dev, cu_seqlens_dev, b.max_L, indices_dev,
                              static_cast<hipStream_t>(stream)),
                "select kernel");
    return AUDIOKV_OK;
}

int32_t audiokv_compact(const audiokv_params* params, const void* k, const void* v, const int32_t* indices_dev,
                        const int32_t* cu_budgets_dev, const int32_t* cu_seqlens_dev, const int32_t* seqlens_host,
                        int32_t n_items, int64_t total_rows, void* k_out, void* v_out, void* stream)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (n_items == 0) return AUDIOKV_OK;
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    if (!k || !v || !indices_dev || !cu_budgets_dev || !cu_seqlens_dev || !k_out || !v_out)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_compact: NULL pointer argument");
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
        return fail(AUDIOKV_E_INVALID_ARG, "k, v, k_out and v_out must be 16-byte aligned");
    if (total_rows < 0 || total_rows > b.total_tokens * params->n_kv_heads)
        return fail(AUDIOKV_E_INVALID_ARG, "total_rows %lld outside [0, tokens x heads]", (long long)total_rows);
    const Geom g = make_geom(params, n_items);
    AUDIOKV_HIP(launch_compact(g, k, v, indices_dev, cu_budgets_dev, cu_seqlens_dev, total_rows, k_out, v_out,
                               static_cast<hipStream_t>(stream)),
                "compact kernel");
    return AUDIOKV_OK;
}

namespace {
int32_t evict_entry(const audiokv_params* params, const void* q_win, const void* k, const void* v,
                    const float* lse_dev,
                    const float* weights_dev, int32_t alloc_scope, const int32_t* cu_seqlens_dev,
                    const int32_t* seqlens_host, int32_t n_items, double ratio, double cutoff_frac, double alpha,
                    void* k_out, void* v_out, int32_t* indices_dev, int32_t* budgets_dev, int32_t* cu_budgets_dev,
                    void* workspace, size_t workspace_bytes, void* stream, bool in_line = false)
{
    AUDIOKV_TRY(check_params(params, 1));
    if (n_items == 0) return AUDIOKV_OK;
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    if (!q_win || !k || !v || !weights_dev || !cu_seqlens_dev || !k_out || !v_out || !indices_dev || !budgets_dev ||
        !cu_budgets_dev || !workspace)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_evict: NULL pointer argument");
    if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
        return fail(AUDIOKV_E_INVALID_ARG, "q_win, k, v, k_out and v_out must be 16-byte aligned");
    if (alloc_scope != AUDIOKV_SCOPE_ITEM && alloc_scope != AUDIOKV_SCOPE_GLOBAL)
        return fail(AUDIOKV_E_INVALID_ARG, "alloc_scope %d", alloc_scope);
    if (alloc_scope == AUDIOKV_SCOPE_GLOBAL && !b.uniform)
        return fail(AUDIOKV_E_INVALID_ARG, "a global budget pool needs equal lengths (got %d..%d)", b.min_L, b.max_L);
    AUDIOKV_TRY(check_ratio(params, b, seqlens_host, ratio));
    AUDIOKV_TRY(check_smooth_args(params, cutoff_frac, alpha));
    AUDIOKV_TRY(check_smooth_lengths(b, seqlens_host, alpha));
    AUDIOKV_TRY(check_score_shape(params));
    if (!select_supported(b.max_L)) return fail(AUDIOKV_E_UNSUPPORTED, "select: length %d is not supported", b.max_L);
    const int n_heads = n_items * params->n_kv_heads;
    if (alloc_scope == AUDIOKV_SCOPE_GLOBAL && n_heads > 1536)
        return fail(AUDIOKV_E_UNSUPPORTED, "global pool of %d heads > 1536", n_heads);
    const Workspace w = plan_workspace(params, b, seqlens_host);
    if (workspace_bytes < w.total)
        return fail(AUDIOKV_E_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);

    const Geom g = make_geom(params, n_items);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    float* stats = reinterpret_cast<float*>(ws + w.stats_off);
    float* raw = reinterpret_cast<float*>(ws + w.raw_off);
    float* smoothed = reinterpret_cast<float*>(ws + w.smooth_off);
    int64_t total_rows = 0;
    for (int i = 0; i < n_items; ++i) total_rows += (int64_t)audiokv_n_keep(ratio, seqlens_host[i]) * params->n_kv_heads;

    const int n_seg = alloc_scope == AUDIOKV_SCOPE_GLOBAL ? 1 : n_items;
    const int hps = alloc_scope == AUDIOKV_SCOPE_GLOBAL ? n_heads : params->n_kv_heads;
    // in_line: everything on the caller's stream, no library-owned stream or event is touched (or created)
    const bool prof = !in_line && g_prof.enabled && g_prof.created;
    // Work that does not depend on the scores goes to the helper stream, beside the score sweeps: the allocation, and
    // for lengths that are not powers of two the chirp tables and filter spectra of the smoothing (35 us of small
    // kernels). A small pool alone is allocated faster than a fork and a join are issued (55 us of host time): then
    // everything stays in line.
    const bool chirp = alpha != 0.0 && smooth_workspace_required(seqlens_host, n_items, params->n_kv_heads) > 0;
    const bool side = !in_line && !prof && (hps >= 32 || chirp);
    const bool side_filters = side && chirp;
    std::unique_lock<std::mutex> helper_lock(g_helper.mu, std::defer_lock);
    if (side) helper_lock.lock();
#define AUDIOKV_MARK(i) do { if (prof) AUDIOKV_HIP(hipEventRecord(g_prof.ev[i], s), "hipEventRecord"); } while (0)
    AUDIOKV_MARK(0);
    // In line and without stage timing, the allocation rides along with the launch that merges the row statistics
    // between the two sweeps (one launch less on the critical path of a call); with the caller's log-sum-exp there
    // is no such launch.
    const AllocateJob alloc_job{weights_dev, n_seg, hps, 1, cu_seqlens_dev, ratio, (double)params->floor_frac,
                                budgets_dev, cu_budgets_dev};
    const bool ride = !side && !prof && !lse_dev;
    if (!side && !ride) {
        // (stage timing wants one kernel per interval: then, too, the allocation stays in line)
        AUDIOKV_HIP(launch_allocate(g, weights_dev, n_seg, hps, 1, cu_seqlens_dev, ratio, (double)params->floor_frac,
                                    budgets_dev, cu_budgets_dev, s), "allocate kernel");
    } else if (side) {
        AUDIOKV_HIP(ensure_helper(), "helper stream");
        AUDIOKV_HIP(hipEventRecord(g_helper.fork, s), "hipEventRecord");
        AUDIOKV_HIP(hipStreamWaitEvent(g_helper.stream, g_helper.fork, 0), "hipStreamWaitEvent");
        AUDIOKV_HIP(launch_allocate(g, weights_dev, n_seg, hps, 1, cu_seqlens_dev, ratio, (double)params->floor_frac,
                                    budgets_dev, cu_budgets_dev, g_helper.stream), "allocate kernel");
        // the chirp tables and filter spectra of lengths that are not powers of two depend on the lengths and the
        // cutoff only: half a dozen small kernels that also fit under the score sweeps
        if (side_filters)
            AUDIOKV_HIP(launch_smooth_filters(g, cu_seqlens_dev, seqlens_host, n_items, cutoff_frac, ws + w.fft_off,
                                              g_helper.stream), "chirp-z filter kernels");
        AUDIOKV_HIP(hipEventRecord(g_helper.join, g_helper.stream), "hipEventRecord");
    }
    AUDIOKV_MARK(1);
    AUDIOKV_HIP(launch_score(g, q_win, k, cu_seqlens_dev, seqlens_host, stats, raw, s,
                             prof ? g_prof.ev[AUDIOKV_PROFILE_STAGES + 1] : nullptr, lse_dev,
                             w.raw2 ? reinterpret_cast<float*>(ws + w.raw2_off) : nullptr,
                             (size_t)b.total_tokens * params->n_kv_heads, ride ? &alloc_job : nullptr), "score kernels");
    AUDIOKV_MARK(2);
    if (side) {
        // budgets (needed by select) and filters (needed by smooth) are ready; by now the helper's work is long done
        AUDIOKV_HIP(hipStreamWaitEvent(s, g_helper.join, 0), "hipStreamWaitEvent");
        helper_lock.unlock();
    }
    AUDIOKV_HIP(launch_smooth(g, raw, params->pool_kernel != 1, cu_seqlens_dev, seqlens_host, n_items, cutoff_frac,
                              alpha, smoothed, ws + w.fft_off, w.total - w.fft_off, nullptr, false, s, side_filters),
                "smooth kernel");
    AUDIOKV_MARK(3);
    AUDIOKV_HIP(launch_select(g, smoothed, budgets_dev, cu_budgets_dev, cu_seqlens_dev, b.max_L, indices_dev, s),
                "select kernel");
    AUDIOKV_MARK(4);
    AUDIOKV_HIP(launch_compact(g, k, v, indices_dev, cu_budgets_dev, cu_seqlens_dev, total_rows, k_out, v_out, s),
                "compact kernel");
    AUDIOKV_MARK(5);
#undef AUDIOKV_MARK
    if (prof) g_prof.recorded = true;
    return AUDIOKV_OK;
}
}  // namespace

int32_t audiokv_evict(const audiokv_params* params, const void* q_win, const void* k, const void* v,
                      const float* weights_dev, int32_t alloc_scope, const int32_t* cu_seqlens_dev,
                      const int32_t* seqlens_host, int32_t n_items, double ratio, double cutoff_frac, double alpha,
                      void* k_out, void* v_out, int32_t* indices_dev, int32_t* budgets_dev, int32_t* cu_budgets_dev,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    return evict_entry(params, q_win, k, v, nullptr, weights_dev, alloc_scope, cu_seqlens_dev, seqlens_host, n_items,
                       ratio, cutoff_frac, alpha, k_out, v_out, indices_dev, budgets_dev, cu_budgets_dev, workspace,
                       workspace_bytes, stream);
}

int32_t audiokv_evict_lse(const audiokv_params* params, const void* q_win, const void* k, const void* v,
                          const float* lse_dev,
                          const float* weights_dev, int32_t alloc_scope, const int32_t* cu_seqlens_dev,
                          const int32_t* seqlens_host, int32_t n_items, double ratio, double cutoff_frac, double alpha,
                          void* k_out, void* v_out, int32_t* indices_dev, int32_t* budgets_dev,
                          int32_t* cu_budgets_dev, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!lse_dev && n_items != 0) return fail(AUDIOKV_E_INVALID_ARG, "audiokv_evict_lse: NULL lse_dev");
    return evict_entry(params, q_win, k, v, lse_dev, weights_dev, alloc_scope, cu_seqlens_dev, seqlens_host, n_items,
                       ratio, cutoff_frac, alpha, k_out, v_out, indices_dev, budgets_dev, cu_budgets_dev, workspace,
                       workspace_bytes, stream);
}

// ---- audiokv_evict_noalloc: the workspace is a static device array -------------------------------------------------
// One copy per GPU, at its own address; the host-side name `scratch` is only a handle for hipGetSymbolAddress.
namespace {
__attribute__((used)) static __device__ __align__(256) unsigned char scratch[AUDIOKV_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
struct ScratchAddr {
    std::mutex mu;
    void* ptr[kMaxDevices] = {};
} g_scratch;

// device address of `scratch` on the current device (looked up once per device, with that device current)
int32_t scratch_of_current_device(void** out) {
    int dev = -1;
    AUDIOKV_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(AUDIOKV_E_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch.mu);
    if (!g_scratch.ptr[dev]) {
        void* p = nullptr;
        AUDIOKV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (!p) return fail(AUDIOKV_E_HIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch.ptr[dev] = p;
    }
    *out = g_scratch.ptr[dev];
    return AUDIOKV_OK;
}
}  // namespace

int32_t audiokv_evict_noalloc(const audiokv_params* params, const void* q_win, const void* k, const void* v,
                              const float* weights_dev, int32_t alloc_scope, const int32_t* cu_seqlens_dev,
                              const int32_t* seqlens_host, int32_t n_items, double ratio, double cutoff_frac,
                              double alpha, void* k_out, void* v_out, int32_t* indices_dev, int32_t* budgets_dev,
                              int32_t* cu_budgets_dev, void* stream)
{
    AUDIOKV_TRY(check_params(params, 1));
    if (n_items == 0) return AUDIOKV_OK;
    Batch b;
    AUDIOKV_TRY(check_batch(params, n_items, seqlens_host, &b));
    const size_t need = plan_workspace(params, b, seqlens_host).total;
    if (need > (size_t)AUDIOKV_NOALLOC_SCRATCH_BYTES)
        return fail(AUDIOKV_E_WORKSPACE_TOO_SMALL, "audiokv_evict_noalloc: this batch needs %zu bytes of scratch, the static "
                    "array holds %zu (use audiokv_evict with a workspace)", need, (size_t)AUDIOKV_NOALLOC_SCRATCH_BYTES);
    void* ws = nullptr;
    AUDIOKV_TRY(scratch_of_current_device(&ws));
    return evict_entry(params, q_win, k, v, nullptr, weights_dev, alloc_scope, cu_seqlens_dev, seqlens_host, n_items,
                       ratio, cutoff_frac, alpha, k_out, v_out, indices_dev, budgets_dev, cu_budgets_dev, ws,
                       (size_t)AUDIOKV_NOALLOC_SCRATCH_BYTES, stream, /*in_line=*/true);
}

int32_t audiokv_decode_workspace_bytes(const audiokv_params* params, int32_t n_items, int64_t total_rows,
                                       size_t* out_bytes)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (!out_bytes || n_items < 0 || total_rows < 0 || total_rows > (int64_t)INT32_MAX)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_decode_workspace_bytes: NULL pointer, n_items < 0 or total_rows out of range");
    if (n_items == 0) { *out_bytes = 0; return AUDIOKV_OK; }
    *out_bytes = decode_workspace_bytes(make_geom(params, n_items), total_rows);
    return AUDIOKV_OK;
}

int32_t audiokv_decode_attend(const audiokv_params* params, const void* q_dev, const void* k_cache,
                              const void* v_cache, const int32_t* cu_budgets_dev, int32_t n_items,
                              int64_t total_rows, float* out_dev, void* workspace, size_t workspace_bytes,
                              void* stream)
{
    AUDIOKV_TRY(check_params(params, 0));
    if (n_items == 0) return AUDIOKV_OK;
    if (!q_dev || !k_cache || !v_cache || !cu_budgets_dev || !out_dev || !workspace)
        return fail(AUDIOKV_E_INVALID_ARG, "audiokv_decode_attend: NULL pointer argument");
    if (n_items < 1 || total_rows < 0 || total_rows > (int64_t)INT32_MAX)
        return fail(AUDIOKV_E_INVALID_ARG, "n_items must be >= 1 and total_rows in [0, 2^31)");
    if (!decode_supported(params->n_q_heads / params->n_kv_heads))
        return fail(AUDIOKV_E_UNSUPPORTED, "decode: %d query heads per KV head > 16", params->n_q_heads / params->n_kv_heads);
    const Geom g = make_geom(params, n_items);
    const size_t need = decode_workspace_bytes(g, total_rows);
    if (workspace_bytes < need)
        return fail(AUDIOKV_E_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    AUDIOKV_HIP(launch_decode(g, q_dev, k_cache, v_cache, cu_budgets_dev, total_rows, out_dev, workspace,
                              static_cast<hipStream_t>(stream)),
                "decode kernels");
    return AUDIOKV_OK;
}

int32_t audiokv_profile_enable(int32_t enable)
{
    if (enable && !g_prof.created) {
        for (auto& e : g_prof.ev) AUDIOKV_HIP(hipEventCreate(&e), "hipEventCreate");
        g_prof.created = true;
    }
    g_prof.enabled = enable != 0;
    g_prof.recorded = false;
    return AUDIOKV_OK;
}

int32_t audiokv_profile_read(float* ms_out)
{
    if (!ms_out) return fail(AUDIOKV_E_INVALID_ARG, "ms_out is NULL");
    if (!g_prof.created || !g_prof.recorded)
        return fail(AUDIOKV_E_INVALID_ARG, "no profiled audiokv_evict call to read");
    AUDIOKV_HIP(hipEventSynchronize(g_prof.ev[5]), "hipEventSynchronize");
    hipEvent_t mid = g_prof.ev[AUDIOKV_PROFILE_STAGES + 1];
    // intervals: [0,1] allocate, [1,mid] sweep 1, [mid,2] sweep 2, [2,3] smooth, [3,4] select, [4,5] compact
    hipEvent_t a[AUDIOKV_PROFILE_STAGES] = {g_prof.ev[0], g_prof.ev[1], mid, g_prof.ev[2], g_prof.ev[3], g_prof.ev[4]};
    hipEvent_t b[AUDIOKV_PROFILE_STAGES] = {g_prof.ev[1], mid, g_prof.ev[2], g_prof.ev[3], g_prof.ev[4], g_prof.ev[5]};
    for (int i = 0; i < AUDIOKV_PROFILE_STAGES; ++i)
        AUDIOKV_HIP(hipEventElapsedTime(&ms_out[i], a[i], b[i]), "hipEventElapsedTime");
    return AUDIOKV_OK;
}

}  // extern "C"
