// Instantiates the BRACE vote kernels for 2-dword loads (one translation unit per op and
// load width so that they compile in parallel).
#include "ops.hpp"

brace_dev::stream_kernel_t<brace_dev::VoteOp> brace_vote_pick_v2(int cols, int ru, int nt, int pipe,
                                                                 int rs)
{
    return brace_dev::pick_cols<brace_dev::VoteOp, 2>(cols, ru, nt, pipe, rs);
}

// The staged (burst-write) kernels for 2- and 4-dword loads live here too: this is the
// smallest of the three translation units.
brace_dev::stream_staged_kernel_t<brace_dev::VoteOp> brace_vote_pick_staged(int v, int cols, int pipe)
{
    return v == 4 ? brace_dev::pick_staged<brace_dev::VoteOp, 4>(cols, pipe)
                  : brace_dev::pick_staged<brace_dev::VoteOp, 2>(cols, pipe);
}
