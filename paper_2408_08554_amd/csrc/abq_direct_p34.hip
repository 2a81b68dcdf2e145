// Kernel instantiations of the direct decode kernel for weight widths 3 and 4 (one translation unit per
// pair of widths so that they compile in parallel).
#include "abq_direct_kernels.h"

namespace abq {

hipError_t direct_launch_p34(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    return p == 3 ? direct_launch_p<3>(gp, MR, R, raw, grid, waves, s) : direct_launch_p<4>(gp, MR, R, raw, grid, waves, s);
}

}  // namespace abq
