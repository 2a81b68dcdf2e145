// Kernel instantiations of the shared-operand decode kernel for weight widths 1 to 4.
#include "abq_shared_a_kernels.h"

namespace abq {

hipError_t shared_a_launch_p1234(int p, const SharedAParams& gp, int phases, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    switch (p) {
        case 1: return shared_a_launch_p<1>(gp, phases, R, raw, grid, waves, s);
        case 2: return shared_a_launch_p<2>(gp, phases, R, raw, grid, waves, s);
        case 3: return shared_a_launch_p<3>(gp, phases, R, raw, grid, waves, s);
        default: return shared_a_launch_p<4>(gp, phases, R, raw, grid, waves, s);
    }
}

}  // namespace abq
