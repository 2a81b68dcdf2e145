// Kernel instantiations of the direct decode kernel for weight widths 1 and 2 (one translation unit per
// pair of widths so that they compile in parallel).
#include "abq_direct_kernels.h"

namespace abq {

hipError_t direct_launch_p12(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    return p == 1 ? direct_launch_p<1>(gp, MR, R, raw, grid, waves, s) : direct_launch_p<2>(gp, MR, R, raw, grid, waves, s);
}

}  // namespace abq
