// Host-side planning for the score kernels: which (row blocks per wave, row-splitting
// waves) instantiation covers G*W window rows, and into how many key ranges a head is cut.
#include "score_impl.h"

namespace audiokv {

namespace {

struct Plan { int NB, WR, rows_pad, tile_keys; };

// Instantiated row-block counts per head_dim (must match score_d*.hip).
const int kNB64[] = {1, 2, 4, 8};
const int kNB128[] = {1, 2, 4, 7, 8};
const int kNB256[] = {1, 2, 4};

bool make_plan(int rows, int D, Plan* out) {
    const int* nbs; int n_nb;
    if (D == 64) { nbs = kNB64; n_nb = 4; }
    else if (D == 128) { nbs = kNB128; n_nb = 5; }
    else if (D == 256) { nbs = kNB256; n_nb = 3; }
    else return false;
    bool found = false;
    Plan best{};
    for (int WR = 4; WR >= 2; WR >>= 1) {            // prefer more row-splitting waves on equal padding
        for (int i = 0; i < n_nb; ++i) {
            const int pad = nbs[i] * 16 * WR;
            if (pad < rows) continue;
            if (!found || pad < best.rows_pad) {
                const int kb = (D == 256) ? 2 : 4;
                best = Plan{nbs[i], WR, pad, 16 * kb * (4 / WR)};
                found = true;
            }
            break;                                    // larger NB only pads more
        }
    }
    if (found) *out = best;
    return found;
}

}  // namespace

int score_padded_rows(int rows, int D) {
    Plan p;
    return make_plan(rows, D, &p) ? p.rows_pad : 0;
}

int score_num_splits(int n_heads_total, int max_L, int rows, int D) {
    Plan p;
    if (!make_plan(rows, D, &p) || n_heads_total <= 0) return 1;
    const int tiles = (max_L + p.tile_keys - 1) / p.tile_keys;
    const int target_groups = 1024;                   // ~4 workgroups per CU of a 256-CU part
    int ns = (target_groups + n_heads_total - 1) / n_heads_total;
    ns = ns < 1 ? 1 : ns;
    ns = ns > 64 ? 64 : ns;
    ns = ns > tiles ? tiles : ns;
    return ns < 1 ? 1 : ns;
}

hipError_t launch_score(const Geom& g, const void* q_win, const void* k, const int32_t* cu_seqlens,
                        int max_L, float* stats_ws, float* raw_out, hipStream_t s, hipEvent_t between_sweeps)
{
    Plan p;
    const int rows = g.G * g.W;
    if (!make_plan(rows, g.D, &p)) return hipErrorInvalidValue;
    const int nsplit = score_num_splits(g.n_items * g.H_kv, max_L, rows, g.D);
    switch (g.D) {
        case 64:  return launch_score_d64(g, p.NB, p.WR, q_win, k, cu_seqlens, nsplit, stats_ws, raw_out, s, between_sweeps);
        case 128: return launch_score_d128(g, p.NB, p.WR, q_win, k, cu_seqlens, nsplit, stats_ws, raw_out, s, between_sweeps);
        case 256: return launch_score_d256(g, p.NB, p.WR, q_win, k, cu_seqlens, nsplit, stats_ws, raw_out, s, between_sweeps);
    }
    return hipErrorInvalidValue;
}

}  // namespace audiokv
