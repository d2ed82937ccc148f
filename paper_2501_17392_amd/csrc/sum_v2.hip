// Instantiates the plain sum / mean kernels for 2-dword loads.
#include "ops.hpp"

brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v2(int cols, int ru, int nt, int pipe,
                                                                 int rs)
{
    return brace_dev::pick_cols<brace_dev::SumOp, 2>(cols, ru, nt, pipe, rs);
}

// The staged (burst-write) kernels for 2- and 4-dword loads live here too: this is the
// smallest of the three translation units.
brace_dev::stream_staged_kernel_t<brace_dev::SumOp> brace_sum_pick_staged(int v, int cols, int pipe)
{
    return v == 4 ? brace_dev::pick_staged<brace_dev::SumOp, 4>(cols, pipe)
                  : brace_dev::pick_staged<brace_dev::SumOp, 2>(cols, pipe);
}
