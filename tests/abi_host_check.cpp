// Host-side exercise of the C ABI for a sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer on the host code
// of the library): argument validation, size queries, rounding, empty batches. No kernel is launched and no device
// memory is touched: every call either runs on the host only or is refused before its first HIP call.
// Built and run by tests/test_host_sanitizers.py; exits 0 when every check holds.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "audiokv.h"

static int g_failed = 0;
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::fprintf(stderr, "FAILED %s:%d: %s (last error: %s)\n", __FILE__, __LINE__, #cond, audiokv_last_error()); \
            ++g_failed;                                                      \
        }                                                                    \
    } while (0)

static audiokv_params make(int hq, int hkv, int d, int w) {
    audiokv_params p;
    std::memset(&p, 0, sizeof(p));
    p.size = sizeof(p);
    p.n_q_heads = hq; p.n_kv_heads = hkv; p.head_dim = d; p.window = w;
    p.pool_kernel = 7; p.causal = 1; p.floor_frac = 0.1f;
    return p;
}

int main() {
    CHECK(audiokv_version() >= 100);
    CHECK(audiokv_last_error() != nullptr);
    // rounding of ratio * L: half up, in one rounded multiply and one rounded add
    CHECK(audiokv_n_keep(0.4, 2048) == 819);
    CHECK(audiokv_n_keep(0.5, 3) == 2);
    CHECK(audiokv_n_keep(1.0, 32768) == 32768);

    audiokv_params p = make(28, 4, 128, 32);
    int64_t rows = -1;
    size_t bytes = 0;
    const int32_t lens2[2] = {2048, 5000};
    CHECK(audiokv_total_kept(&p, 2, lens2, 0.3, &rows) == AUDIOKV_OK && rows == (614 + 1500) * 4);
    CHECK(audiokv_workspace_bytes(&p, 2, lens2, &bytes) == AUDIOKV_OK && bytes > 2u * 4u * (2048u + 5000u) * 4u);

    // every geometry the score planner knows, ragged batches of many sizes: the planner's arithmetic under UBSan
    const int geoms[][4] = {{28, 4, 128, 32}, {28, 4, 128, 64}, {32, 4, 128, 32}, {8, 2, 256, 32}, {8, 8, 64, 8},
                            {16, 1, 128, 16}, {36, 4, 128, 64}, {16, 1, 256, 16}, {64, 8, 64, 64}, {1, 1, 64, 1}};
    for (const auto& gm : geoms) {
        audiokv_params q = make(gm[0], gm[1], gm[2], gm[3]);
        for (int n = 1; n <= 48; n += 7) {
            std::vector<int32_t> lens(n);
            for (int i = 0; i < n; ++i) lens[i] = gm[3] + 1 + (i * 7919 + n * 104729) % 33000;
            size_t b = 0;
            const int32_t rc = audiokv_workspace_bytes(&q, n, lens.data(), &b);
            CHECK(rc == AUDIOKV_OK && b > 0);
            int64_t r = 0;
            CHECK(audiokv_total_kept(&q, n, lens.data(), 1.0, &r) == AUDIOKV_OK && r > 0);
        }
    }

    // invalid parameters are codes, never crashes
    { audiokv_params q = make(28, 5, 128, 32);  CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }
    { audiokv_params q = make(28, 4, 96, 32);   CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_UNSUPPORTED); }
    { audiokv_params q = p; q.pool_kernel = 4;  CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }
    { audiokv_params q = p; q.floor_frac = 1.5f; CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }
    { audiokv_params q = p; q.kv_layout = 7;    CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }
    { audiokv_params q = p; q.size = 12;        CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }
    { audiokv_params q = p; q.kv_stride_tok = 132; q.kv_stride_head = 4096 * 128;
      CHECK(audiokv_workspace_bytes(&q, 1, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }
    { audiokv_params q = p; q.kv_stride_tok = 128; q.kv_stride_head = 8192 * 128;
      CHECK(audiokv_workspace_bytes(&q, 1, lens2, &bytes) == AUDIOKV_OK);
      CHECK(audiokv_workspace_bytes(&q, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG); }      // no item stride
    CHECK(audiokv_workspace_bytes(nullptr, 2, lens2, &bytes) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_workspace_bytes(&p, 2, nullptr, &bytes) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_workspace_bytes(&p, 2, lens2, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_workspace_bytes(&p, -1, lens2, &bytes) == AUDIOKV_E_INVALID_ARG);
    const int32_t short_len[1] = {16};
    CHECK(audiokv_total_kept(&p, 1, short_len, 0.5, &rows) == AUDIOKV_E_INVALID_ARG);        // L below the window
    CHECK(audiokv_total_kept(&p, 2, lens2, 0.001, &rows) == AUDIOKV_E_INVALID_ARG);          // n_keep below the window
    CHECK(std::strlen(audiokv_last_error()) > 0);

    // entry points that would enqueue kernels: NULL pointers and bad arguments are refused before any HIP call
    CHECK(audiokv_score(&p, nullptr, nullptr, nullptr, lens2, 2, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_score_lse(&p, nullptr, nullptr, nullptr, nullptr, lens2, 2, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_allocate(&p, nullptr, 1, 4, 1, nullptr, lens2, 0.4, nullptr, nullptr, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_allocate(&p, nullptr, 1, 4000, 1, nullptr, lens2, 0.4, nullptr, nullptr, nullptr) == AUDIOKV_E_UNSUPPORTED);
    CHECK(audiokv_smooth(&p, nullptr, nullptr, lens2, 2, 0.125, 1.0, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_smooth_cutoffs(&p, nullptr, nullptr, lens2, 2, 0.5, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_select(&p, nullptr, nullptr, nullptr, nullptr, lens2, 2, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_compact(&p, nullptr, nullptr, nullptr, nullptr, nullptr, lens2, 2, 10, nullptr, nullptr, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_evict(&p, nullptr, nullptr, nullptr, nullptr, 0, nullptr, lens2, 2, 0.4, 0.125, 1.0, nullptr, nullptr,
                        nullptr, nullptr, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_evict_lse(&p, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, lens2, 2, 0.4, 0.125, 1.0, nullptr,
                            nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_evict_noalloc(&p, nullptr, nullptr, nullptr, nullptr, 0, nullptr, lens2, 2, 0.4, 0.125, 1.0, nullptr,
                                nullptr, nullptr, nullptr, nullptr, nullptr) != AUDIOKV_OK);
    {   // a batch beyond the static scratch is refused by size, before anything else is looked at
        std::vector<int32_t> big(28, 32768);
        audiokv_params q = make(28, 4, 128, 64);
        CHECK(audiokv_evict_noalloc(&q, nullptr, nullptr, nullptr, nullptr, 1, nullptr, big.data(), 28, 0.4, 0.125, 1.0,
                                    nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == AUDIOKV_E_WORKSPACE_TOO_SMALL);
    }
    int dummy = 0;                       // non-null, never dereferenced: the argument checks come first
    void* x = &dummy;
    CHECK(audiokv_evict(&p, x, x, x, (const float*)x, 5, (const int32_t*)x, lens2, 2, 0.4, 0.125, 1.0, x, x, (int32_t*)x,
                        (int32_t*)x, (int32_t*)x, x, 1u << 30, nullptr) == AUDIOKV_E_INVALID_ARG);   // alloc_scope 5, misaligned
    CHECK(audiokv_decode_attend(&p, nullptr, nullptr, nullptr, nullptr, 1, 10, nullptr, nullptr, 0, nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_decode_workspace_bytes(&p, 1, -5, &bytes) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_decode_workspace_bytes(&p, 28, 1468000, &bytes) == AUDIOKV_OK && bytes > 0);
    float ms[AUDIOKV_PROFILE_STAGES];
    CHECK(audiokv_profile_read(nullptr) == AUDIOKV_E_INVALID_ARG);
    CHECK(audiokv_profile_read(ms) == AUDIOKV_E_INVALID_ARG);                                 // nothing recorded

    // empty batches: accepted everywhere, nothing is enqueued, sizes come back as 0
    CHECK(audiokv_total_kept(&p, 0, nullptr, 0.4, &rows) == AUDIOKV_OK && rows == 0);
    CHECK(audiokv_workspace_bytes(&p, 0, nullptr, &bytes) == AUDIOKV_OK && bytes == 0);
    CHECK(audiokv_score(&p, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_score_lse(&p, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_allocate(&p, nullptr, 0, 4, 1, nullptr, nullptr, 0.4, nullptr, nullptr, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_smooth(&p, nullptr, nullptr, nullptr, 0, 0.125, 1.0, nullptr, nullptr, 0, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_select(&p, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_compact(&p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_evict(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, 0, 0.4, 0.125, 1.0, nullptr, nullptr,
                        nullptr, nullptr, nullptr, nullptr, 0, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_evict_noalloc(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, nullptr, 0, 0.4, 0.125, 1.0, nullptr,
                                nullptr, nullptr, nullptr, nullptr, nullptr) == AUDIOKV_OK);
    CHECK(audiokv_decode_attend(&p, nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, 0, nullptr) == AUDIOKV_OK);

    if (g_failed) { std::fprintf(stderr, "%d check(s) failed\n", g_failed); return 1; }
    std::puts("abi_host_check: all checks passed");
    return 0;
}
