// Instantiates the plain sum / mean kernels for 1-dword loads.
#include "ops.hpp"

brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v1(int cols, int ru, int nt, int pipe,
                                                                 int rs)
{
    return brace_dev::pick_cols<brace_dev::SumOp, 1>(cols, ru, nt, pipe, rs);
}

// The ring-order fp32 sum for every load width lives here too: this translation unit has
// the fewest other kernels.
brace_dev::ring_sum_kernel_t brace_ring_pick(int v, int cols, int staged)
{
    switch (v) {
    case 4: return brace_dev::pick_ring<4>(cols, staged != 0);
    case 2: return brace_dev::pick_ring<2>(cols, staged != 0);
    default: return brace_dev::pick_ring<1>(cols, false);
    }
}
