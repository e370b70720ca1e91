// Host-side planning for the score kernels: which (row blocks per wave, row-splitting
// waves) instantiation covers G*W window rows, and into how many key ranges a head is cut.
#include "score_impl.h"

namespace audiokv {

namespace {

struct Plan { int NB, WR, rows_pad, tile_keys; };

// Instantiated (32-row blocks per wave, waves per workgroup) pairs, by padded row count (must match score_d*.hip).
struct Combo { int NB, WR; };
const Combo kCombos128[] = {{1, 1}, {1, 2}, {1, 4}, {1, 7}, {2, 4}, {2, 7}, {2, 8}};   // d = 64, 128
const Combo kCombos256[] = {{1, 1}, {1, 2}, {1, 4}, {1, 7}, {1, 8}};                   // d = 256

bool make_plan(int rows, int D, Plan* out) {
    const Combo* cs; int n;
    if (D == 64 || D == 128) { cs = kCombos128; n = 7; }
    else if (D == 256) { cs = kCombos256; n = 5; }
    else return false;
    for (int i = 0; i < n; ++i) {                     // sorted by padded rows: the first that fits pads least
        const int pad = cs[i].NB * 32 * cs[i].WR;
        if (pad >= rows) {
            *out = Plan{cs[i].NB, cs[i].WR, pad, (D == 256) ? 32 : 32 * AUDIOKV_SCORE_KB};
            return true;
        }
    }
    return false;
}

}  // namespace

int score_padded_rows(int rows, int D) {
    Plan p;
    return make_plan(rows, D, &p) ? p.rows_pad : 0;
}

int score_num_splits(int n_heads_total, int max_L, int rows, int D) {
    Plan p;
    if (!make_plan(rows, D, &p) || n_heads_total <= 0) return 1;
    // A head is cut into key ranges so that the grid fills the 256 CUs in whole rounds: pick the split
    // count that minimises rounds x (tiles per workgroup + fixed prologue cost, in tiles).
    const int tiles = (max_L + p.tile_keys - 1) / p.tile_keys;
    // resident workgroups: two per CU when a wave holds one row tile (128 registers, 59 KB of LDS) or the
    // workgroup is small, one when the eight waves take all the registers
    const int slots = 256 * ((p.NB == 1 && D <= 128) || p.WR < 7 ? 2 : 1);
    const int overhead = 3;
    int best = 1;
    long long best_cost = -1;
    const int ns_max = tiles < 64 ? tiles : 64;
    for (int ns = 1; ns <= ns_max; ++ns) {
        const long long groups = (long long)n_heads_total * ns;
        const long long rounds = (groups + slots - 1) / slots;
        const long long cost = rounds * ((tiles + ns - 1) / ns + overhead);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = ns; }
    }
    return best;
}

hipError_t launch_score(const Geom& g, const void* q_win, const void* k, const int32_t* cu_seqlens,
                        int max_L, float* stats_ws, float* raw_out, hipStream_t s, hipEvent_t between_sweeps,
                        const float* lse)
{
    Plan p;
    const int rows = g.G * g.W;
    if (!make_plan(rows, g.D, &p)) return hipErrorInvalidValue;
    const int nsplit = score_num_splits(g.n_items * g.H_kv, max_L, rows, g.D);
    switch (g.D) {
        case 64:  return launch_score_d64(g, p.NB, p.WR, q_win, k, cu_seqlens, nsplit, stats_ws, raw_out, s, between_sweeps, lse);
        case 128: return launch_score_d128(g, p.NB, p.WR, q_win, k, cu_seqlens, nsplit, stats_ws, raw_out, s, between_sweeps, lse);
        case 256: return launch_score_d256(g, p.NB, p.WR, q_win, k, cu_seqlens, nsplit, stats_ws, raw_out, s, between_sweeps, lse);
    }
    return hipErrorInvalidValue;
}

}  // namespace audiokv
