// MFMA path (placeholder until the implicit-GEMM kernels land): reports "not supported" so that
// UKST_PATH_AUTO resolves to the direct path and UKST_PATH_MFMA returns UKST_ERR_UNSUPPORTED.
#include "ukst_internal.h"

namespace ukst {
bool mfma_supported(const Geom&, int) { return false; }
hipError_t launch_mfma(const Geom&, const void*, const void*, float*, int, hipStream_t)
{
    return hipErrorNotSupported;
}
const char* mfma_kernel_name(const Geom&, int) { return ""; }
}  // namespace ukst
