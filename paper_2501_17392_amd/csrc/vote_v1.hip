// Instantiates the streaming vote kernel for 1-dword loads (one translation unit per load
// width so that the widths compile in parallel).
#include "vote_kernel.hpp"

brace_dev::vote_kernel_t brace_vote_pick_v1(int cols, int ru, int nt, int pipe)
{
    return brace_dev::pick_cols<1>(cols, ru, nt, pipe);
}
