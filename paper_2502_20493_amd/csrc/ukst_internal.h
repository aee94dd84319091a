// Internal declarations shared by the HIP translation units of libukst (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ukst {

// Problem description in "quad space".
//
// Shift output coordinates by the padding: qy = oy + P, qx = ox + P.  A quad (k, m) is the 2x2
// group of shifted coordinates rows {2k-1, 2k} x cols {2m-1, 2m}.  Its four members are exactly
// the four parity classes of Algorithm 2 (row 2k-1 -> r = 1, row 2k -> r = 0; same for columns),
// and all four read the same ceil(n/2) x ceil(n/2) input window whose first pixel is
// (k - P, m - P): for member row q the first input row is ceil((q - 2P)/2) = k - P either way.
// Class (r, s) uses the taps w[r + 2u][s + 2v] of that window (Eqs. 1-4), so across the quad
// every one of the n*n taps is used exactly once.  Members that fall outside the output (first /
// last row or column of an odd-sized output) are predicated off, never stored.
struct Geom {
    int B, Cin, Cout, H, W, n, P;
    int OH, OW;
    int k_min, m_min;  // first quad row / column that owns an in-range output
    int KH, KW;        // number of quad rows / columns
};

inline Geom make_geom(int B, int Cin, int Cout, int H, int W, int n, int P)
{
    Geom g;
    g.B = B; g.Cin = Cin; g.Cout = Cout; g.H = H; g.W = W; g.n = n; g.P = P;
    g.OH = 2 * H + 2 * P - n;
    g.OW = 2 * W + 2 * P - n;
    g.k_min = (P + 1) >> 1;                      // smallest k with 2k >= P
    g.m_min = (P + 1) >> 1;
    g.KH = ((P + g.OH - 1 + 1) >> 1) - g.k_min + 1;  // largest k: ceil((P+OH-1)/2)
    g.KW = ((P + g.OW - 1 + 1) >> 1) - g.m_min + 1;
    return g;
}

// Launchers.  Each returns hipSuccess or the launch error; none synchronises.
hipError_t launch_direct(const Geom& g, const void* x, const void* w, float* y, int dtype,
                         hipStream_t stream);
const char* direct_kernel_name(const Geom& g, int dtype);

// Narrow-channel kernel (fp32, Cin and Cout <= 4): register-blocked quads, buffer addressing.
bool narrow_supported(const Geom& g, int dtype);
hipError_t launch_narrow(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream);

// Thin-output kernel (fp32, Cout <= 4, many input channels): channel-split reduction on the VALUs.
bool thin_supported(const Geom& g, int dtype);
hipError_t launch_thin(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream);

bool mfma_supported(const Geom& g, int dtype);
hipError_t launch_mfma(const Geom& g, const void* x, const void* w, float* y, int dtype,
                       hipStream_t stream);
const char* mfma_kernel_name(const Geom& g, int dtype);

// true if the kernel mfma_kernel_name() names also needs x aligned to 16 bytes (w always is)
bool mfma_needs_aligned_x(const Geom& g, int dtype);

// fp32-operand MFMA kernels (used by the functions above for dtype 0): the general one, and the
// one for layers with at most 4 output channels, where the parity classes fill the MFMA columns
bool mfma_f32_supported(const Geom& g);
hipError_t launch_mfma_f32(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream);
bool thin_mfma_supported(const Geom& g, int dtype);
hipError_t launch_thin_mfma(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream);

}  // namespace ukst
