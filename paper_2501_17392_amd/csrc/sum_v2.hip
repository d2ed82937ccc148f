// Instantiates the plain sum / mean kernels for 2-dword loads.
#include "ops.hpp"

brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v2(int cols, int ru, int nt, int pipe,
                                                                 int rs)
{
    return brace_dev::pick_cols<brace_dev::SumOp, 2>(cols, ru, nt, pipe, rs);
}
