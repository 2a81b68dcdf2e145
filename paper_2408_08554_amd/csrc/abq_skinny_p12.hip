// Kernel instantiations of the streaming decode kernel for weight widths 1 and 2 (one translation unit per
// pair of widths so that they compile in parallel).
#include "abq_skinny_kernels.h"

namespace abq {

hipError_t skinny_launch_p12(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    return p == 1 ? launch_pd<1, 8>(prm, grid, waves, lds_bytes, s) : launch_pd<2, 8>(prm, grid, waves, lds_bytes, s);
}

hipError_t grouped_launch_p12(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s)
{
    return p == 1 ? launch_grouped_pd<1, 8>(gp, raw, grid, waves, lds_bytes, s)
                  : launch_grouped_pd<2, 8>(gp, raw, grid, waves, lds_bytes, s);
}

}  // namespace abq
