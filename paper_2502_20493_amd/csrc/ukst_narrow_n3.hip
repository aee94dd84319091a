// Narrow-channel kernels for kernel side n = 3 (one translation unit per n keeps the build parallel).
#include "ukst_narrow_kernel.h"

namespace ukst {

hipError_t launch_narrow_n3(const Geom& g, const float* x, const float* w, float* y,
                             hipStream_t stream)
{
    return narrow::launch_ci<3>(g, x, w, y, stream);
}

}  // namespace ukst
