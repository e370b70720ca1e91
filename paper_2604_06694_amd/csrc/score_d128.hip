// Score kernels for head_dim = 128. Instantiated (32-row blocks per wave, waves per workgroup): 1,1 1,2 1,4 1,7 2,4 3,3 2,7 2,8 3,6.
#include "score_impl.h"

namespace audiokv {

hipError_t launch_score_d128(int which, const Geom& g, int NB, int WR, const void* q_win, const void* k,
        const int32_t* cu_seq, int nsplit, int rows_pad, int row_base, float* stats, float* cst, float* raw,
        hipStream_t s, const float* lse)
{
    using namespace score_detail;
    if (NB == 1 && WR == 1) return launch_sweep<128, 1, 1>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 1 && WR == 2) return launch_sweep<128, 1, 2>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 1 && WR == 4) return launch_sweep<128, 1, 4>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 1 && WR == 7) return launch_sweep<128, 1, 7>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 2 && WR == 4) return launch_sweep<128, 2, 4>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 3 && WR == 3) return launch_sweep<128, 3, 3>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 2 && WR == 7) return launch_sweep<128, 2, 7>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 2 && WR == 8) return launch_sweep<128, 2, 8>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    if (NB == 3 && WR == 6) return launch_sweep<128, 3, 6>(which, g, q_win, k, cu_seq, nsplit, rows_pad, row_base, stats, cst, raw, s, lse);
    return hipErrorInvalidValue;
}

}  // namespace audiokv
