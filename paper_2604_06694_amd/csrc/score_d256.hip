// Score kernels for head_dim = 256 (row-block counts instantiated: 1 2 4; row-splitting waves: 2 or 4).
#include "score_impl.h"

namespace audiokv {

hipError_t launch_score_d256(const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, float* stats, float* raw, hipStream_t s, hipEvent_t between)
{
    using namespace score_detail;
    if (NB == 1 && WR == 2) return launch_both_sweeps<256, 1, 2>(g, q_win, k, cu_seq, nsplit, stats, raw, s, between);
    if (NB == 1 && WR == 4) return launch_both_sweeps<256, 1, 4>(g, q_win, k, cu_seq, nsplit, stats, raw, s, between);
    if (NB == 2 && WR == 2) return launch_both_sweeps<256, 2, 2>(g, q_win, k, cu_seq, nsplit, stats, raw, s, between);
    if (NB == 2 && WR == 4) return launch_both_sweeps<256, 2, 4>(g, q_win, k, cu_seq, nsplit, stats, raw, s, between);
    if (NB == 4 && WR == 2) return launch_both_sweeps<256, 4, 2>(g, q_win, k, cu_seq, nsplit, stats, raw, s, between);
    if (NB == 4 && WR == 4) return launch_both_sweeps<256, 4, 4>(g, q_win, k, cu_seq, nsplit, stats, raw, s, between);
    return hipErrorInvalidValue;
}

}  // namespace audiokv
