// Kernel instantiations of the streaming decode kernel for weight widths 7 and 8 (one translation unit per
// pair of widths so that they compile in parallel).
#include "abq_skinny_kernels.h"

namespace abq {

hipError_t skinny_launch_p78(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    return p == 7 ? launch_pd<7, 2>(prm, grid, waves, lds_bytes, s) : launch_pd<8, 2>(prm, grid, waves, lds_bytes, s);
}

hipError_t grouped_launch_p78(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s)
{
    return p == 7 ? launch_grouped_pd<7, 2>(gp, raw, grid, waves, lds_bytes, s)
                  : launch_grouped_pd<8, 2>(gp, raw, grid, waves, lds_bytes, s);
}

}  // namespace abq
