// Kernel instantiations of the shared-operand decode kernel for weight widths 5 to 8.
#include "abq_shared_a_kernels.h"

namespace abq {

hipError_t shared_a_launch_p5678(int p, const SharedAParams& gp, int phases, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    switch (p) {
        case 5: return shared_a_launch_p<5>(gp, phases, R, raw, grid, waves, s);
        case 6: return shared_a_launch_p<6>(gp, phases, R, raw, grid, waves, s);
        case 7: return shared_a_launch_p<7>(gp, phases, R, raw, grid, waves, s);
        default: return shared_a_launch_p<8>(gp, phases, R, raw, grid, waves, s);
    }
}

}  // namespace abq
