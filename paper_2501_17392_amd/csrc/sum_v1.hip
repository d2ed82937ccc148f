// Instantiates the plain sum / mean kernels for 1-dword loads.
#include "ops.hpp"

brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v1(int cols, int ru, int nt, int pipe,
                                                                 int rs)
{
    return brace_dev::pick_cols<brace_dev::SumOp, 1>(cols, ru, nt, pipe, rs);
}
