// Narrow-channel path (fp32, Cin <= 4, Cout <= 4): which shapes it takes, and the dispatch on the
// kernel side n to the translation unit that holds those kernels.
#include "ukst_internal.h"

namespace ukst {

hipError_t launch_narrow_n1(const Geom&, const float*, const float*, float*, hipStream_t);
hipError_t launch_narrow_n2(const Geom&, const float*, const float*, float*, hipStream_t);
hipError_t launch_narrow_n3(const Geom&, const float*, const float*, float*, hipStream_t);
hipError_t launch_narrow_n4(const Geom&, const float*, const float*, float*, hipStream_t);
hipError_t launch_narrow_n5(const Geom&, const float*, const float*, float*, hipStream_t);

bool narrow_supported(const Geom& g, int dtype)
{
    // buffer offsets are 32-bit byte offsets inside the image of one batch item
    const long long xbytes = 4LL * g.Cin * g.H * g.W, ybytes = 4LL * g.Cout * g.OH * g.OW;
    return dtype == 0 && g.Cin <= 4 && g.Cout <= 4 && g.n <= 5 && xbytes < (1LL << 30) &&
           ybytes < (1LL << 30) && g.P < (1 << 20);
}

hipError_t launch_narrow(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream)
{
    const float* xf = (const float*)x;
    const float* wf = (const float*)w;
    switch (g.n) {
        case 1: return launch_narrow_n1(g, xf, wf, y, stream);
        case 2: return launch_narrow_n2(g, xf, wf, y, stream);
        case 3: return launch_narrow_n3(g, xf, wf, y, stream);
        case 4: return launch_narrow_n4(g, xf, wf, y, stream);
        case 5: return launch_narrow_n5(g, xf, wf, y, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ukst
