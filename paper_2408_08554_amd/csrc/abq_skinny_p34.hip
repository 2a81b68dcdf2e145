// Kernel instantiations of the streaming decode kernel for weight widths 3 and 4 (one translation unit per
// pair of widths so that they compile in parallel).
#include "abq_skinny_kernels.h"

namespace abq {

hipError_t skinny_launch_p34(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    return p == 3 ? launch_pd<3, 4>(prm, grid, waves, lds_bytes, s) : launch_pd<4, 4>(prm, grid, waves, lds_bytes, s);
}

hipError_t grouped_launch_p34(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s)
{
    return p == 3 ? launch_grouped_pd<3, 4>(gp, raw, grid, waves, lds_bytes, s)
                  : launch_grouped_pd<4, 4>(gp, raw, grid, waves, lds_bytes, s);
}

}  // namespace abq
