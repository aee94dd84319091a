// Internal declarations shared by the HIP translation units of libukst (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

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
// Optional fused epilogue, applied to the finished sum on its way to memory:
// y = act(sum + bias[co]); bias == nullptr means no bias, act 0 none, 1 ReLU, 2 tanh.
struct Epilogue {
    const float* bias;
    int act;
};

// The part of the geometry the kernels take as their argument.
struct GeomBase {
    int B, Cin, Cout, H, W, n, P;
    int OH, OW;
    int k_min, m_min;  // first quad row / column that owns an in-range output
    int KH, KW;        // number of quad rows / columns
};

// Host side: geometry plus the epilogue of this call.  Kernels receive the epilogue as their LAST
// argument (or last member of their argument block), so that the argument layout, and with it
// the code, of the instances that do not use it stays what it is without one.
struct Geom : GeomBase {
    Epilogue ep;
};

// true if the stores have anything to apply (uniform over the launch)
__host__ __device__ inline bool has_epilogue(const Epilogue& e) { return e.bias != nullptr || e.act != 0; }

// tanh(v) = 1 - 2 / (exp(2v) + 1): saturates to +-1 without overflow trouble (exp -> inf gives 1,
// exp -> 0 gives -1); hardware exp2 and reciprocal, absolute error of a few 1e-7
__device__ __forceinline__ float fast_tanh(float v)
{
    const float e = __builtin_amdgcn_exp2f(v * 2.8853900817779268f);  // exp(2v) = 2^(2v log2 e)
    return fmaf(-2.f, __builtin_amdgcn_rcpf(e + 1.f), 1.f);
}
// activation known at compile time (kernels with long drains branch once, outside their loops)
template <int ACT>
__device__ __forceinline__ float epilogue_t(float v, float b)
{
    v += b;
    if constexpr (ACT == 1) v = fmaxf(v, 0.f);
    if constexpr (ACT == 2) v = fast_tanh(v);
    return v;
}
__device__ __forceinline__ float epilogue(float v, float b, int act)
{
    return act == 1 ? epilogue_t<1>(v, b) : act == 2 ? epilogue_t<2>(v, b) : epilogue_t<0>(v, b);
}
// calls f(integral_constant<int, act>) for the run-time activation code (uniform branch)
template <class F>
__device__ __forceinline__ void with_activation(int act, F&& f)
{
    if (act == 1) f(std::integral_constant<int, 1>{});
    else if (act == 2) f(std::integral_constant<int, 2>{});
    else f(std::integral_constant<int, 0>{});
}

// Exact division of n < 2^31 by a run-time constant: q = umulhi(n, M) >> sh.
struct FastDiv { unsigned M; int sh; unsigned d; };
inline FastDiv make_fastdiv(unsigned d)
{
    FastDiv f;
    f.d = d; f.M = 0; f.sh = 0;
    if (d <= 1) return f;
    int l = 0;
    while ((1ull << l) < d) ++l;
    f.M = (unsigned)(((1ull << (31 + l)) / d) + 1);
    f.sh = l - 1;
    return f;
}
__device__ __forceinline__ int fdiv(int n, const FastDiv& f)
{
    return f.d == 1 ? n : (int)(__umulhi((unsigned)n, f.M) >> f.sh);
}

// Workgroups are handed to the 8 XCDs round-robin.  Renumber them so that each XCD (one L2)
// works on a contiguous run of tiles and neighbouring tiles' halos hit the same L2.
__device__ __forceinline__ int xcd_contiguous(int bid, int nb)
{
    constexpr int X = 8;
    const int xcd = bid % X, idx = bid / X;
    const int fl = nb / X, rem = nb % X;
    return xcd * fl + (xcd < rem ? xcd : rem) + idx;
}

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
    g.ep.bias = nullptr;
    g.ep.act = 0;
    return g;
}

// Scratch memory of one call, owned by the caller (the library never allocates).  Launchers that
// use scratch compute the bytes they need from the shape alone.  With `query` set they record that
// figure in `need` and launch nothing; otherwise they return kWorkspaceTooSmall when `bytes` is
// below it.  ptr == nullptr asks for kernels that need no scratch where such kernels exist.
struct Workspace {
    void* ptr = nullptr;
    size_t bytes = 0;
    bool query = false;
    size_t need = 0;
};
constexpr hipError_t kWorkspaceTooSmall = hipErrorOutOfMemory;  // reported as UKST_ERR_WORKSPACE
// rounds a scratch sub-buffer size up so that the next one starts 256-byte aligned
inline size_t ws_align(size_t b) { return (b + 255) & ~(size_t)255; }

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
                       Workspace& ws, hipStream_t stream);
const char* mfma_kernel_name(const Geom& g, int dtype);

// bf16 operands, n = 4, even P: the same implicit GEMM on quads aligned to the output
bool mfma_aligned_supported(const Geom& g, int dtype);
hipError_t launch_mfma_aligned(const Geom& g, const void* x, const void* w, float* y, int dtype,
                               hipStream_t stream);

// true if the kernel mfma_kernel_name() names also needs x aligned to 16 bytes (w always is)
bool mfma_needs_aligned_x(const Geom& g, int dtype);

// fp32-operand MFMA kernels (used by the functions above for dtype 0): the general one, and the
// one for layers with at most 4 output channels, where the parity classes fill the MFMA columns
bool mfma_f32_supported(const Geom& g, int dtype);
hipError_t launch_mfma_f32(const Geom& g, const void* x, const void* w, float* y, int dtype, Workspace& ws,
                           hipStream_t stream);
bool thin_mfma_supported(const Geom& g, int dtype);
hipError_t launch_thin_mfma(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream);

// Stride-k transpose convolution (dilated == 0) / dilation-k convolution (dilated == 1), any shape
hipError_t launch_general(int dilated, int B, int Cin, int Cout, int H, int W, int n, int P, int k,
                          int OH, int OW, const void* x, const void* w, float* y, int dtype,
                          hipStream_t stream);

// Backward pass (vector-ALU kernels, any shape; dtype 0: fp32, 1: bf16 operands, fp32 result)
hipError_t launch_grad_input(const Geom& g, const void* dy, const void* w, float* dx, int dtype,
                             Workspace& ws, hipStream_t stream);
hipError_t launch_grad_weight(const Geom& g, const void* x, const void* dy, float* dw, int dtype,
                              Workspace& ws, hipStream_t stream);
// Input gradient of bf16 layers with 4 x 4 kernels and at least 65 input channels: bf16 MFMA with a
// channel's 16 taps as the contraction (weights packed once per call into the workspace)
bool grad_input_window_supported(const Geom& g, int dtype);
hipError_t launch_grad_input_window(const Geom& g, const void* dy, const void* w, float* dx, Workspace& ws,
                                    hipStream_t stream);
// Both gradients of narrow fp32 layers (Cin, Cout <= 4, 2 <= n <= 5, maps at least 32 wide):
// register-blocked strips, edges by buffer addressing.  which 0: (p0, p1) = (dy, w) -> dx, no scratch;
// which 1: (p0, p1) = (x, dy) -> dw, one copy of dw per block in the workspace
bool grad_narrow_supported(const Geom& g, int dtype);
hipError_t launch_grad_narrow(int which, const Geom& g, const void* p0, const void* p1, float* out, Workspace& ws,
                              hipStream_t stream);
// which: 0 gradient w.r.t. the input, 1 w.r.t. the kernel
const char* grad_kernel_name(const Geom& g, int which, int dtype);

}  // namespace ukst
