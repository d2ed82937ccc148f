// Instantiates the BRACE vote kernels for 4-dword loads (one translation unit per op and
// load width so that they compile in parallel).
#include "ops.hpp"

brace_dev::stream_kernel_t<brace_dev::VoteOp> brace_vote_pick_v4(int cols, int ru, int nt, int pipe,
                                                                 int rs)
{
    return brace_dev::pick_cols<brace_dev::VoteOp, 4>(cols, ru, nt, pipe, rs);
}
