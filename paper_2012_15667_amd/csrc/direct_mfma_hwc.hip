// Direct convolution on the matrix cores, x[N][H][W][C] -> y[N][P][Q][K] instantiations.
#include "direct_mfma_impl.h"

namespace iolb {

hipError_t launch_direct_mfma_hwc(const float* x, const float* wt, float* y, const DirectGeom& g, hipStream_t st)
{
    return launch_direct_mfma_layout<true>(x, wt, y, g, st);
}

}  // namespace iolb
