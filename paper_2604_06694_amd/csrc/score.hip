// Host-side planning for the score kernels: which (row blocks per wave, row-splitting waves) instantiation
// covers G*W window rows in each of the two sweeps, and into how many key ranges a head is cut.
#include "score_impl.h"

namespace audiokv {

namespace {

struct Plan { int NB, WR, rows_pad, tile_keys; };

// Instantiated (32-row blocks per wave, waves per workgroup) pairs in order of preference per sweep: the first
// that holds the rows is taken (all must exist in score_d*.hip). The sweeps differ where their register needs do:
// three row tiles per wave fit the registers of sweep 1 (and let two 4-wave workgroups share a CU at 256 rows),
// but spill in sweep 2, which also carries the row constants.
struct Combo { int NB, WR; };
const Combo kSweep1_128[] = {{1, 1}, {1, 2}, {1, 4}, {1, 7}, {3, 3}, {2, 7}, {3, 6}};   // d = 64, 128
const Combo kSweep2_128[] = {{1, 1}, {1, 2}, {1, 4}, {1, 7}, {2, 4}, {2, 7}, {2, 8}};
const Combo kCombos256[] = {{1, 1}, {1, 2}, {1, 4}, {1, 7}, {1, 8}};                    // d = 256, both sweeps

bool make_plan(int rows, int D, int sweep, Plan* out) {
    const Combo* cs; int n;
    if (D == 64 || D == 128) { cs = sweep == 1 ? kSweep1_128 : kSweep2_128; n = 7; }
    else if (D == 256) { cs = kCombos256; n = 5; }
    else return false;
    for (int i = 0; i < n; ++i) {
        const int pad = cs[i].NB * 32 * cs[i].WR;
        if (pad >= rows) {
            *out = Plan{cs[i].NB, cs[i].WR, pad, (D == 256) ? 32 : 32 * AUDIOKV_SCORE_KB};
            return true;
        }
    }
    return false;
}

int num_splits(const Plan& p, int H_kv, int n_items, const int32_t* seqlens_host, int D) {
    // A head is cut into key ranges so that the grid fills the 256 CUs evenly: the split count minimises the time of
    // the launch in units of one tile, with a fixed prologue cost per workgroup (in tiles).
    // resident workgroups per CU: two when the waves are few or hold one row tile each (128 registers), or when
    // the workgroup is four waves of three row tiles; one when eight waves take all the registers
    const bool two = (p.NB == 1 && D <= 128) || p.WR < 4 || (p.NB == 3 && p.WR == 3);
    const int slots = 256 * (two ? 2 : 1);
    // what a workgroup costs before its first and after its last tile (query fragments, filling the ring, the row
    // statistics or constants), in tiles: about 200 keys' worth, fitted to measured launches
    const int overhead = p.tile_keys >= 64 ? 3 : 7;
    int max_tiles = 1;
    bool uniform = true;
    for (int i = 0; i < n_items; ++i) {
        const int t = (seqlens_host[i] + p.tile_keys - 1) / p.tile_keys;
        if (t > max_tiles) max_tiles = t;
        if (seqlens_host[i] != seqlens_host[0]) uniform = false;
    }
    int best = 1;
    long long best_cost = -1;
    const int ns_max = max_tiles < 64 ? max_tiles : 64;
    for (int ns = 1; ns <= ns_max; ++ns) {
        long long cost;
        if (uniform) {
            // equal workgroups run in whole rounds
            const long long groups = (long long)n_items * H_kv * ns;
            const long long rounds = (groups + slots - 1) / slots;
            cost = rounds * ((max_tiles + ns - 1) / ns + overhead);
        } else {
            // Ragged lengths: a head's ranges are as long as the head is (tiles of the head / ns), and workgroups
            // start as others end. The launch takes about the average load of a slot, plus part of the longest
            // workgroup for the ones that start last, plus, when the last round of workgroups fills only part of the
            // slots, that round's average workgroup for the slots left idle (all in twice the unit, to keep halves).
            long long total = 0, longest = 0;
            const long long groups = (long long)n_items * H_kv * ns;   // launched, whether or not they hold tiles
            for (int i = 0; i < n_items; ++i) {
                const int t = (seqlens_host[i] + p.tile_keys - 1) / p.tile_keys;
                if (t <= 0) continue;
                const int tps = (t + ns - 1) / ns;
                const int used = (t + tps - 1) / tps;          // ranges of this head that hold tiles
                total += (long long)H_kv * (t + (long long)used * overhead);
                if (tps + overhead > longest) longest = tps + overhead;
            }
            cost = 2 * ((total + slots - 1) / slots) + longest;
            const long long rem = groups % slots;
            if (groups > slots && rem) cost += 2 * (total / groups) * (slots - rem) / slots;
        }
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = ns; }
    }
    return best;
}

}  // namespace

// Sweep 2 cannot hold more than 448 rows without spilling (its row constants come on top of the accumulators), so
// more rows are covered by two launches: the first 448 with the widest tiling, the rest with the smallest that fits;
// the second writes its column sums to a buffer of its own, added to the first afterwards.
constexpr int kSweep2MaxRows = 448;

bool sweep2_is_split(int rows, int D) { return D <= 128 && rows > kSweep2MaxRows; }

int score_padded_rows(int rows, int D) {
    Plan p1, p2;
    if (!make_plan(rows, D, 1, &p1)) return 0;
    if (sweep2_is_split(rows, D)) {
        if (!make_plan(rows - kSweep2MaxRows, D, 2, &p2)) return 0;
        const int pad2 = kSweep2MaxRows + p2.rows_pad;
        return p1.rows_pad > pad2 ? p1.rows_pad : pad2;
    }
    if (!make_plan(rows, D, 2, &p2)) return 0;
    return p1.rows_pad > p2.rows_pad ? p1.rows_pad : p2.rows_pad;
}

bool score_needs_second_raw(int rows, int D) { return sweep2_is_split(rows, D); }

// key ranges per head of sweep 1: what sizes the statistics in the workspace
int score_num_splits(int H_kv, int n_items, const int32_t* seqlens_host, int rows, int D) {
    Plan p;
    if (!make_plan(rows, D, 1, &p) || n_items <= 0 || H_kv <= 0) return 1;
    return num_splits(p, H_kv, n_items, seqlens_host, D);
}

hipError_t launch_score(const Geom& g, const void* q_win, const void* k, const int32_t* cu_seqlens,
                        const int32_t* seqlens_host, float* stats_ws, float* raw_out, hipStream_t s, hipEvent_t between_sweeps,
                        const float* lse, float* raw_second, size_t raw_elems, const AllocateJob* ride_along)
{
    Plan p1;
    const int rows = g.G * g.W;
    if (!make_plan(rows, g.D, 1, &p1)) return hipErrorInvalidValue;
    const int n_heads = g.n_items * g.H_kv;
    const int rows_pad = score_padded_rows(rows, g.D);
    if (rows_pad == 0) return hipErrorInvalidValue;
    const int ns1 = num_splits(p1, g.H_kv, g.n_items, seqlens_host, g.D);
    float* cst = stats_ws + (size_t)n_heads * ns1 * rows_pad * 2;
    auto sweep = [&](int which, const Plan& p, int ns, int row_base, float* raw) -> hipError_t {
        switch (g.D) {
            case 64:  return launch_score_d64(which, g, p.NB, p.WR, q_win, k, cu_seqlens, ns, rows_pad, row_base, stats_ws, cst, raw, s, lse);
            case 128: return launch_score_d128(which, g, p.NB, p.WR, q_win, k, cu_seqlens, ns, rows_pad, row_base, stats_ws, cst, raw, s, lse);
            case 256: return launch_score_d256(which, g, p.NB, p.WR, q_win, k, cu_seqlens, ns, rows_pad, row_base, stats_ws, cst, raw, s, lse);
        }
        return hipErrorInvalidValue;
    };
    hipError_t e = sweep(1, p1, ns1, 0, raw_out);
    if (e != hipSuccess) return e;
    if (!lse) {
        e = launch_score_merge(g, stats_ws, ns1, rows_pad, cst, ride_along, s);
        if (e != hipSuccess) return e;
    }
    if (between_sweeps) {
        e = hipEventRecord(between_sweeps, s);
        if (e != hipSuccess) return e;
    }
    Plan p2;
    if (!sweep2_is_split(rows, g.D)) {
        if (!make_plan(rows, g.D, 2, &p2)) return hipErrorInvalidValue;
        return sweep(2, p2, num_splits(p2, g.H_kv, g.n_items, seqlens_host, g.D), 0, raw_out);
    }
    if (!raw_second) return hipErrorInvalidValue;
    Plan p2b;
    if (!make_plan(kSweep2MaxRows, g.D, 2, &p2) || !make_plan(rows - kSweep2MaxRows, g.D, 2, &p2b)) return hipErrorInvalidValue;
    e = sweep(2, p2, num_splits(p2, g.H_kv, g.n_items, seqlens_host, g.D), 0, raw_out);
    if (e != hipSuccess) return e;
    e = sweep(2, p2b, num_splits(p2b, g.H_kv, g.n_items, seqlens_host, g.D), kSweep2MaxRows, raw_second);
    if (e != hipSuccess) return e;
    const unsigned blocks = (unsigned)((raw_elems + 256 * 8 - 1) / (256 * 8));
    hipLaunchKernelGGL(score_detail::score_add_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, s, raw_out,
                       (const float*)raw_second, raw_elems);
    return hipGetLastError();
}

}  // namespace audiokv
