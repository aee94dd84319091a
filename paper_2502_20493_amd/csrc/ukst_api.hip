// C-ABI boundary of libukst: argument validation, geometry, path selection.  See include/ukst.h.
#include "../../include/ukst.h"
#include "ukst_internal.h"
#include <atomic>

namespace {

// Scratch of ukst_conv_transpose2d_grad_weight_static: one array per GPU, part of the loaded code
// object, held until the process ends.  The name is a host-side stand-in; the device address is
// looked up once per device (hipGetSymbolAddress) and kept here.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// device address of `scratch` on the current device, or nullptr (with *err set) on failure
void* static_scratch(hipError_t* err)
{
    int dev = -1;
    if ((*err = hipGetDevice(&dev)) != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        // two threads may both get here: they find the same address
        if ((*err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return nullptr;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    return p;
}

int validate_shape(int B, int Cin, int Cout, int H, int W, int n, int P)
{
    if (B < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1 || n < 1 || P < 0) return UKST_ERR_SHAPE;
    // sizes are ints: keep 2H+2P and friends inside int32
    if (H > (1 << 28) || W > (1 << 28) || P > (1 << 28)) return UKST_ERR_SHAPE;
    if (2 * H + 2 * P - n < 1 || 2 * W + 2 * P - n < 1) return UKST_ERR_SHAPE;
    return UKST_OK;
}

// Taps of one output row (or column) that meet an in-range input row: tap a of output o lands on
// upsampled coordinate o + a - P, which holds input row (o + a - P)/2 when even and inside.
unsigned long long exact_line_taps(int L, int OL, int n, int P)
{
    unsigned long long t = 0;
    for (int o = 0; o < OL; ++o)
        for (int a = 0; a < n; ++a) {
            const int u = o + a - P;
            if (u >= 0 && (u & 1) == 0 && u / 2 < L) ++t;
        }
    return t;
}

// Taps Algorithm 2 executes per line: ceil(n/2) for class 0 outputs, floor(n/2) for class 1.
unsigned long long nominal_line_taps(int OL, int n, int P)
{
    unsigned long long t = 0;
    for (int o = 0; o < OL; ++o) t += (unsigned)((n - ((o + P) & 1) + 1) >> 1);
    return t;
}

// Output size of the generalised operations, 0 on invalid arguments.
// stride-k transpose convolution: the map is upsampled to k(H-1)+1, padded by P, n x n window;
// dilation-k convolution: the kernel is upsampled to k(n-1)+1, the input padded by P.
bool general_shape(int dilated, int H, int W, int n, int P, int k, int* OH, int* OW)
{
    if (H < 1 || W < 1 || n < 1 || P < 0 || k < 1 || k > UKST_MAX_STEP) return false;
    if (H > (1 << 24) || W > (1 << 24) || P > (1 << 24)) return false;
    const long long oh = dilated ? (long long)H + 2 * P - (long long)k * (n - 1)
                                 : (long long)k * (H - 1) + 2 * P - n + 2;
    const long long ow = dilated ? (long long)W + 2 * P - (long long)k * (n - 1)
                                 : (long long)k * (W - 1) + 2 * P - n + 2;
    if (oh < 1 || ow < 1 || oh > 0x3fffffffLL || ow > 0x3fffffffLL) return false;
    *OH = (int)oh;
    *OW = (int)ow;
    return true;
}

// taps of one output line that meet an in-range input pixel (kind 0), that the segregated
// algorithm executes (kind 1: its class's taps, padding included), or that the naive definition
// multiplies (kind 2: every tap of the full or upsampled kernel)
unsigned long long general_line_taps(int dilated, int L, int OL, int n, int P, int k, int kind)
{
    unsigned long long t = 0;
    for (int o = 0; o < OL; ++o) {
        if (kind == 2) { t += dilated ? (unsigned)(k * (n - 1) + 1) : (unsigned)n; continue; }
        for (int a = 0; a < n; ++a) {
            if (dilated) {
                const int i = o + k * a - P;
                if (kind == 1 || (i >= 0 && i < L)) ++t;
            } else {
                const int u = o + a - P;
                if (((u % k) + k) % k != 0) continue;  // an inserted zero
                const int i = (u - (((u % k) + k) % k)) / k;
                if (kind == 1 || (u >= 0 && i < L)) ++t;
            }
        }
    }
    return t;
}

int general_checked(int dilated, const void* x, const void* w, void* y, int B, int Cin, int Cout, int H,
                    int W, int n, int P, int k, int dtype, void* stream)
{
    if (!x || !w || !y) return UKST_ERR_NULL;
    if (B < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1 || n < 1 || P < 0 || k < 1) return UKST_ERR_SHAPE;
    if (dtype != UKST_F32 && dtype != UKST_BF16_F32 && dtype != UKST_BF16_BF16) return UKST_ERR_DTYPE;
    if (dtype == UKST_BF16_BF16 || n > UKST_MAX_N || k > UKST_MAX_STEP) return UKST_ERR_UNSUPPORTED;
    int OH = 0, OW = 0;
    if (!general_shape(dilated, H, W, n, P, k, &OH, &OW)) return UKST_ERR_SHAPE;
    const uintptr_t esz = dtype == UKST_F32 ? 4 : 2;
    if ((((uintptr_t)x | (uintptr_t)w) & (esz - 1)) || ((uintptr_t)y & 3)) return UKST_ERR_UNSUPPORTED;
    const hipError_t e = ukst::launch_general(dilated, B, Cin, Cout, H, W, n, P, k, OH, OW, x, w, (float*)y,
                                              dtype, (hipStream_t)stream);
    return e == hipSuccess ? UKST_OK : e == hipErrorInvalidConfiguration ? UKST_ERR_UNSUPPORTED : UKST_ERR_LAUNCH;
}

int resolve_path(const ukst::Geom& g, int dtype, int path)
{
    if (path == UKST_PATH_DIRECT) return UKST_PATH_DIRECT;
    if (path == UKST_PATH_MFMA) return ukst::mfma_supported(g, dtype) ? UKST_PATH_MFMA : -1;
    // AUTO: the matrix cores pay off once both channel counts fill an MFMA tile, or, for layers
    // with very few output channels, once the parity classes can fill its columns instead
    if (ukst::mfma_supported(g, dtype) &&
        ((g.Cin >= 16 && g.Cout >= 16) || ukst::thin_mfma_supported(g, dtype)))
        return UKST_PATH_MFMA;
    return UKST_PATH_DIRECT;
}

}  // namespace

extern "C" {

int ukst_version(void) { return 200; }

const char* ukst_status_string(int status)
{
    switch (status) {
        case UKST_OK: return "ok";
        case UKST_ERR_NULL: return "null pointer argument";
        case UKST_ERR_SHAPE: return "invalid shape: a dimension < 1, P < 0, or empty output";
        case UKST_ERR_DTYPE: return "unknown dtype";
        case UKST_ERR_UNSUPPORTED: return "unsupported: kernel side above UKST_MAX_N or path cannot run this shape";
        case UKST_ERR_LAUNCH: return "HIP launch error";
        case UKST_ERR_WORKSPACE: return "workspace missing, misaligned or smaller than ukst_workspace_bytes";
        default: return "unknown status";
    }
}

int ukst_output_shape(int H, int W, int n, int P, int* OH, int* OW)
{
    if (!OH || !OW) return UKST_ERR_NULL;
    if (H < 1 || W < 1 || n < 1 || P < 0 || H > (1 << 28) || W > (1 << 28) || P > (1 << 28))
        return UKST_ERR_SHAPE;
    if (2 * H + 2 * P - n < 1 || 2 * W + 2 * P - n < 1) return UKST_ERR_SHAPE;
    *OH = 2 * H + 2 * P - n;
    *OW = 2 * W + 2 * P - n;
    return UKST_OK;
}

unsigned long long ukst_mac_count(int B, int Cin, int Cout, int H, int W, int n, int P, int kind)
{
    if (validate_shape(B, Cin, Cout, H, W, n, P) != UKST_OK) return 0;
    const int OH = 2 * H + 2 * P - n, OW = 2 * W + 2 * P - n;
    unsigned long long rows, cols;
    if (kind == 0) {
        rows = exact_line_taps(H, OH, n, P);
        cols = exact_line_taps(W, OW, n, P);
    } else if (kind == 1) {
        rows = nominal_line_taps(OH, n, P);
        cols = nominal_line_taps(OW, n, P);
    } else if (kind == 2) {
        rows = (unsigned long long)OH * n;
        cols = (unsigned long long)OW * n;
    } else {
        return 0;
    }
    return (unsigned long long)B * Cin * Cout * rows * cols;
}

int ukst_select_path(int B, int Cin, int Cout, int H, int W, int n, int P, int dtype)
{
    const int st = validate_shape(B, Cin, Cout, H, W, n, P);
    if (st != UKST_OK) return -st;
    if (dtype != UKST_F32 && dtype != UKST_BF16_F32 && dtype != UKST_BF16_BF16) return -UKST_ERR_DTYPE;
    if (n > UKST_MAX_N) return -UKST_ERR_UNSUPPORTED;
    return resolve_path(ukst::make_geom(B, Cin, Cout, H, W, n, P), dtype, UKST_PATH_AUTO);
}

// Validation shared by the forward entry points and the workspace query; on UKST_OK `g` holds the
// geometry with the epilogue and `chosen` the kernel family.
static int forward_checked(const void* x, const void* w, const float* bias, int act, const void* y,
                           int B, int Cin, int Cout, int H, int W, int n, int P, int dtype, int path,
                           ukst::Geom& g, int& chosen)
{
    if (!x || !w || !y) return UKST_ERR_NULL;
    const int st = validate_shape(B, Cin, Cout, H, W, n, P);
    if (st != UKST_OK) return st;
    if (dtype != UKST_F32 && dtype != UKST_BF16_F32 && dtype != UKST_BF16_BF16) return UKST_ERR_DTYPE;
    if (n > UKST_MAX_N) return UKST_ERR_UNSUPPORTED;
    if (path != UKST_PATH_AUTO && path != UKST_PATH_DIRECT && path != UKST_PATH_MFMA)
        return UKST_ERR_UNSUPPORTED;
    if (act != UKST_ACT_NONE && act != UKST_ACT_RELU && act != UKST_ACT_TANH)
        return UKST_ERR_UNSUPPORTED;
    g = ukst::make_geom(B, Cin, Cout, H, W, n, P);
    g.ep.bias = bias;
    g.ep.act = act;
    // element alignment is required of every buffer; the matrix-core kernels move the weights
    // (and bf16 activations) in 16-byte pieces and need those buffers aligned to that
    const uintptr_t esz = dtype == UKST_F32 ? 4 : 2, osz = dtype == UKST_BF16_BF16 ? 2 : 4;
    if (((uintptr_t)x | (uintptr_t)w) & (esz - 1) || ((uintptr_t)y & (osz - 1)) || ((uintptr_t)bias & 3))
        return UKST_ERR_UNSUPPORTED;
    chosen = resolve_path(g, dtype, path);
    const bool x16 = chosen == UKST_PATH_MFMA && ukst::mfma_needs_aligned_x(g, dtype);
    const bool wide_ok = (((uintptr_t)w | (x16 ? (uintptr_t)x : 0)) & 15) == 0;
    if (chosen == UKST_PATH_MFMA && !wide_ok) chosen = (path == UKST_PATH_AUTO) ? UKST_PATH_DIRECT : -1;
    return chosen < 0 ? UKST_ERR_UNSUPPORTED : UKST_OK;
}

static int status_of(hipError_t e)
{
    return e == hipSuccess ? UKST_OK : e == ukst::kWorkspaceTooSmall ? UKST_ERR_WORKSPACE : UKST_ERR_LAUNCH;
}

static int workspace_checked(const void* workspace, size_t bytes)
{
    if (workspace == nullptr) return bytes == 0 ? UKST_OK : UKST_ERR_WORKSPACE;
    return ((uintptr_t)workspace & 255) == 0 ? UKST_OK : UKST_ERR_WORKSPACE;
}

static int run_checked(const void* x, const void* w, const float* bias, int act, void* y, int B,
                       int Cin, int Cout, int H, int W, int n, int P, int dtype, int path,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    ukst::Geom g;
    int chosen = -1;
    const int st = forward_checked(x, w, bias, act, y, B, Cin, Cout, H, W, n, P, dtype, path, g, chosen);
    if (st != UKST_OK) return st;
    ukst::Workspace ws;
    ws.ptr = workspace;
    ws.bytes = workspace_bytes;
    hipError_t e;
    if (chosen == UKST_PATH_MFMA)
        e = ukst::launch_mfma(g, x, w, (float*)y, dtype, ws, (hipStream_t)stream);
    else
        e = ukst::launch_direct(g, x, w, (float*)y, dtype, (hipStream_t)stream);
    return status_of(e);
}

int ukst_conv_transpose2d_path(const void* x, const void* w, void* y, int B, int Cin, int Cout,
                               int H, int W, int n, int P, int dtype, int path, void* stream)
{
    return run_checked(x, w, nullptr, UKST_ACT_NONE, y, B, Cin, Cout, H, W, n, P, dtype, path, nullptr,
                       0, stream);
}

int ukst_conv_transpose2d_bias_act(const void* x, const void* w, const float* bias, void* y, int B,
                                   int Cin, int Cout, int H, int W, int n, int P, int dtype,
                                   int act, int path, void* stream)
{
    return run_checked(x, w, bias, act, y, B, Cin, Cout, H, W, n, P, dtype, path, nullptr, 0, stream);
}

int ukst_conv_transpose2d_ws(const void* x, const void* w, const float* bias, void* y, int B, int Cin,
                             int Cout, int H, int W, int n, int P, int dtype, int act, int path,
                             void* workspace, size_t workspace_bytes, void* stream)
{
    const int st = workspace_checked(workspace, workspace_bytes);
    if (st != UKST_OK) return st;
    return run_checked(x, w, bias, act, y, B, Cin, Cout, H, W, n, P, dtype, path, workspace,
                       workspace_bytes, stream);
}

size_t ukst_workspace_bytes(int op, int B, int Cin, int Cout, int H, int W, int n, int P, int dtype)
{
    if (validate_shape(B, Cin, Cout, H, W, n, P) != UKST_OK || n > UKST_MAX_N) return 0;
    if (dtype != UKST_F32 && dtype != UKST_BF16_F32 && dtype != UKST_BF16_BF16) return 0;
    ukst::Geom g = ukst::make_geom(B, Cin, Cout, H, W, n, P);
    ukst::Workspace ws;
    ws.query = true;
    hipError_t e = hipErrorInvalidValue;
    if (op == UKST_OP_FORWARD) {
        if (resolve_path(g, dtype, UKST_PATH_AUTO) != UKST_PATH_MFMA) return 0;
        e = ukst::launch_mfma(g, nullptr, nullptr, nullptr, dtype, ws, nullptr);
    } else if (dtype != UKST_BF16_BF16 && op == UKST_OP_GRAD_INPUT) {
        e = ukst::launch_grad_input(g, nullptr, nullptr, nullptr, dtype, ws, nullptr);
    } else if (dtype != UKST_BF16_BF16 && op == UKST_OP_GRAD_WEIGHT) {
        e = ukst::launch_grad_weight(g, nullptr, nullptr, nullptr, dtype, ws, nullptr);
    }
    return e == hipSuccess ? ws.need : 0;
}

int ukst_conv_transpose2d(const void* x, const void* w, void* y, int B, int Cin, int Cout, int H,
                          int W, int n, int P, int dtype, void* stream)
{
    return ukst_conv_transpose2d_path(x, w, y, B, Cin, Cout, H, W, n, P, dtype, UKST_PATH_AUTO,
                                      stream);
}

static int backward_checked(const void* p0, const void* p1, void* out, int B, int Cin, int Cout, int H,
                            int W, int n, int P, int dtype)
{
    if (!p0 || !p1 || !out) return UKST_ERR_NULL;
    const int st = validate_shape(B, Cin, Cout, H, W, n, P);
    if (st != UKST_OK) return st;
    if (dtype != UKST_F32 && dtype != UKST_BF16_F32 && dtype != UKST_BF16_BF16) return UKST_ERR_DTYPE;
    if (dtype == UKST_BF16_BF16 || n > UKST_MAX_N) return UKST_ERR_UNSUPPORTED;  // gradients are fp32
    const uintptr_t esz = dtype == UKST_F32 ? 4 : 2;
    if ((((uintptr_t)p0 | (uintptr_t)p1) & (esz - 1)) || ((uintptr_t)out & 3)) return UKST_ERR_UNSUPPORTED;
    // the kernels index every tensor with 64-bit offsets; nothing else to bound
    return UKST_OK;
}

int ukst_conv_transpose2d_grad_input(const void* dy, const void* w, void* dx, int B, int Cin, int Cout,
                                     int H, int W, int n, int P, int dtype, void* workspace,
                                     size_t workspace_bytes, void* stream)
{
    int st = backward_checked(dy, w, dx, B, Cin, Cout, H, W, n, P, dtype);
    if (st != UKST_OK) return st;
    if ((st = workspace_checked(workspace, workspace_bytes)) != UKST_OK) return st;
    const ukst::Geom g = ukst::make_geom(B, Cin, Cout, H, W, n, P);
    ukst::Workspace ws;
    ws.ptr = workspace;
    ws.bytes = workspace_bytes;
    return status_of(ukst::launch_grad_input(g, dy, w, (float*)dx, dtype, ws, (hipStream_t)stream));
}

int ukst_conv_transpose2d_grad_weight(const void* x, const void* dy, void* dw, int B, int Cin, int Cout,
                                      int H, int W, int n, int P, int dtype, void* workspace,
                                      size_t workspace_bytes, void* stream)
{
    int st = backward_checked(x, dy, dw, B, Cin, Cout, H, W, n, P, dtype);
    if (st != UKST_OK) return st;
    if ((st = workspace_checked(workspace, workspace_bytes)) != UKST_OK) return st;
    const ukst::Geom g = ukst::make_geom(B, Cin, Cout, H, W, n, P);
    ukst::Workspace ws;
    ws.ptr = workspace;
    ws.bytes = workspace_bytes;
    return status_of(ukst::launch_grad_weight(g, x, dy, (float*)dw, dtype, ws, (hipStream_t)stream));
}

size_t ukst_static_workspace_bytes(void) { return kStaticScratchBytes; }

int ukst_conv_transpose2d_grad_weight_static(const void* x, const void* dy, void* dw, int B, int Cin,
                                             int Cout, int H, int W, int n, int P, int dtype, void* stream)
{
    const int st = backward_checked(x, dy, dw, B, Cin, Cout, H, W, n, P, dtype);
    if (st != UKST_OK) return st;
    const ukst::Geom g = ukst::make_geom(B, Cin, Cout, H, W, n, P);
    ukst::Workspace q;
    q.query = true;
    if (ukst::launch_grad_weight(g, nullptr, nullptr, nullptr, dtype, q, nullptr) != hipSuccess)
        return UKST_ERR_LAUNCH;
    if (q.need > kStaticScratchBytes) return UKST_ERR_WORKSPACE;  // host arithmetic only so far
    hipError_t e = hipSuccess;
    ukst::Workspace ws;
    ws.ptr = static_scratch(&e);
    if (ws.ptr == nullptr) return UKST_ERR_LAUNCH;
    ws.bytes = kStaticScratchBytes;
    // every slice writes the whole of its copy before the sum kernel reads it: nothing in the
    // array has to start at zero, whatever the last call left there
    return status_of(ukst::launch_grad_weight(g, x, dy, (float*)dw, dtype, ws, (hipStream_t)stream));
}

int ukst_output_shape_strided(int H, int W, int n, int P, int s, int* OH, int* OW)
{
    if (!OH || !OW) return UKST_ERR_NULL;
    return general_shape(0, H, W, n, P, s, OH, OW) ? UKST_OK : UKST_ERR_SHAPE;
}

int ukst_output_shape_dilated(int H, int W, int n, int P, int d, int* OH, int* OW)
{
    if (!OH || !OW) return UKST_ERR_NULL;
    return general_shape(1, H, W, n, P, d, OH, OW) ? UKST_OK : UKST_ERR_SHAPE;
}

static unsigned long long general_macs(int dilated, int B, int Cin, int Cout, int H, int W, int n, int P,
                                       int k, int kind)
{
    int OH = 0, OW = 0;
    if (B < 1 || Cin < 1 || Cout < 1 || kind < 0 || kind > 2) return 0;
    if (!general_shape(dilated, H, W, n, P, k, &OH, &OW)) return 0;
    return (unsigned long long)B * Cin * Cout * general_line_taps(dilated, H, OH, n, P, k, kind) *
           general_line_taps(dilated, W, OW, n, P, k, kind);
}

unsigned long long ukst_mac_count_strided(int B, int Cin, int Cout, int H, int W, int n, int P, int s,
                                          int kind)
{
    return general_macs(0, B, Cin, Cout, H, W, n, P, s, kind);
}

unsigned long long ukst_mac_count_dilated(int B, int Cin, int Cout, int H, int W, int n, int P, int d,
                                          int kind)
{
    return general_macs(1, B, Cin, Cout, H, W, n, P, d, kind);
}

int ukst_conv_transpose2d_strided(const void* x, const void* w, void* y, int B, int Cin, int Cout, int H,
                                  int W, int n, int P, int s, int dtype, void* stream)
{
    return general_checked(0, x, w, y, B, Cin, Cout, H, W, n, P, s, dtype, stream);
}

int ukst_dilated_conv2d(const void* x, const void* w, void* y, int B, int Cin, int Cout, int H, int W,
                        int n, int P, int d, int dtype, void* stream)
{
    return general_checked(1, x, w, y, B, Cin, Cout, H, W, n, P, d, dtype, stream);
}

const char* ukst_grad_kernel_name(int which, int B, int Cin, int Cout, int H, int W, int n, int P,
                                  int dtype)
{
    if (which != 0 && which != 1) return "";
    if (validate_shape(B, Cin, Cout, H, W, n, P) != UKST_OK) return "";
    if ((dtype != UKST_F32 && dtype != UKST_BF16_F32) || n > UKST_MAX_N) return "";
    return ukst::grad_kernel_name(ukst::make_geom(B, Cin, Cout, H, W, n, P), which, dtype);
}

const char* ukst_kernel_name(int B, int Cin, int Cout, int H, int W, int n, int P, int dtype,
                             int path)
{
    if (validate_shape(B, Cin, Cout, H, W, n, P) != UKST_OK) return "";
    if ((dtype != UKST_F32 && dtype != UKST_BF16_F32 && dtype != UKST_BF16_BF16) || n > UKST_MAX_N) return "";
    const ukst::Geom g = ukst::make_geom(B, Cin, Cout, H, W, n, P);
    const int chosen = resolve_path(g, dtype, path);
    if (chosen < 0) return "";
    return chosen == UKST_PATH_MFMA ? ukst::mfma_kernel_name(g, dtype)
                                    : ukst::direct_kernel_name(g, dtype);
}

}  // extern "C"
