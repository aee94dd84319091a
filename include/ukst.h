/*
 * ukst -- unified kernel-segregated stride-2 2-D transpose convolution for AMD MI355X (gfx950).
 *
 * C ABI, stateless: nothing is cached or kept between calls (weights are re-read and re-gathered
 * by every call), no call synchronises, and no call allocates or frees memory.  Kernels that need
 * scratch memory for the duration of a call (partial sums of a split reduction, re-packed
 * weights) take it from a workspace the caller owns: ukst_workspace_bytes() gives its size from
 * the shape alone, the entry points that can use one have `workspace` / `workspace_bytes`
 * arguments.
 *
 * What is computed (Algorithm 1 of the paper is the definition, Algorithm 2 + Eqs. 1-4 + the
 * padding rule of Sec. 3.4 are how it is evaluated):
 *
 *   the input map is zero-inserted ("bed of nails") to (2H-1) x (2W-1), zero-padded by P on every
 *   side, and an n x n window slides over it with stride 1 and NO kernel flip:
 *
 *     y[b,co,oy,ox] = sum_ci sum_{a<n} sum_{c<n} U_P[b,ci,oy+a,ox+c] * w[co,ci,a,c]
 *     OH = 2H + 2P - n,  OW = 2W + 2P - n          (Sec. 1: (2N-n) x (2N-n) for P = 0)
 *
 *   The kernels never build U_P.  Each output pixel selects, from the parity of (oy+P, ox+P), one
 *   of the four sub-kernels k_rs[u][v] = w[r+2u][s+2v] (sizes ceil/floor(n/2), Sec. 3.1-3.2) and
 *   reads only the original input; the reduced padding floor(P/2) of Sec. 3.4 is a bounds
 *   predicate.  Odd output sizes are produced exactly: nothing is computed into, or stored to,
 *   elements outside [0,OH) x [0,OW) (Sec. 1, Sec. 3.4).
 *
 * Stride is 2, dilation 1, groups 1, no bias, no output padding: none of these appear in the paper.
 */
#ifndef UKST_H
#define UKST_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element types.  Accumulation is always fp32. */
typedef enum {
    UKST_F32 = 0,      /* x, w, y are IEEE fp32 */
    UKST_BF16_F32 = 1, /* x, w are bfloat16 (upper half of an fp32), y is fp32, stored unrounded */
    UKST_BF16_BF16 = 2 /* x, w, y are bfloat16: the fp32 sum (after the fused epilogue, if any) is
                          rounded once, to nearest even, at the store; halves the output traffic */
} ukst_dtype;

typedef enum {
    UKST_OK = 0,
    UKST_ERR_NULL = 1,        /* x, w, y (or an output pointer) is NULL */
    UKST_ERR_SHAPE = 2,       /* a dimension < 1, P < 0, or an empty output (2H+2P-n < 1 ...) */
    UKST_ERR_DTYPE = 3,       /* dtype is not a ukst_dtype */
    UKST_ERR_UNSUPPORTED = 4, /* n > UKST_MAX_N, unknown path id, or path cannot run this shape */
    UKST_ERR_LAUNCH = 5,      /* the HIP runtime reported an error at launch */
    UKST_ERR_WORKSPACE = 6    /* workspace NULL with a non-zero size, not 256-byte aligned, or smaller
                                 than ukst_workspace_bytes() for this call */
} ukst_status;

/* Kernel families ("paths").  UKST_PATH_AUTO picks by channel width. */
typedef enum {
    UKST_PATH_AUTO = 0,
    UKST_PATH_DIRECT = 1, /* vector-ALU kernels: a lane owns whole 2x2 output quads (all four parity
                             classes) and their shared input window; specialised for few channels
                             (narrow: Cin, Cout <= 4; thin: Cout <= 4), general otherwise; any
                             shape, either dtype */
    UKST_PATH_MFMA = 2    /* parity-class implicit GEMM on the matrix cores: wide channels, or <= 4 output channels (fp32) */
} ukst_path;

#define UKST_MAX_N 7    /* largest kernel side compiled in */
#define UKST_MAX_STEP 8 /* largest stride / dilation of the generalised operations */

/* Library version: major*10000 + minor*100 + patch. */
int ukst_version(void);

/* Static, NUL-terminated description of a ukst_status value (never NULL). */
const char* ukst_status_string(int status);

/*
 * Output size of Sec. 1 / Fig. 2: *OH = 2H+2P-n, *OW = 2W+2P-n.
 * Host arithmetic only.  Returns UKST_ERR_NULL, UKST_ERR_SHAPE (as above) or UKST_OK.
 */
int ukst_output_shape(int H, int W, int n, int P, int* OH, int* OW);

/*
 * Multiply-accumulate counts of one call (host arithmetic only; 0 on invalid shapes).
 *   kind 0: exact   -- products of an in-range input pixel with a kernel tap (no bed-of-nails
 *                      zero and no padding zero is counted); this is the "useful" work.
 *   kind 1: nominal -- what Algorithm 2 executes with its floor(P/2) padding: every tap of the
 *                      selected sub-kernel for every output pixel (25 per 2x2 outputs for n = 5,
 *                      Sec. 3.1).
 *   kind 2: naive   -- what Algorithm 1 executes: n*n per output pixel.
 */
unsigned long long ukst_mac_count(int B, int Cin, int Cout, int H, int W, int n, int P, int kind);

/*
 * The path UKST_PATH_AUTO resolves to for this problem (UKST_PATH_DIRECT or UKST_PATH_MFMA),
 * or a negative ukst_status on invalid arguments.  Host arithmetic only.
 */
int ukst_select_path(int B, int Cin, int Cout, int H, int W, int n, int P, int dtype);

/*
 * Stride-2 transpose convolution, Algorithm 2 (unified kernel segregation).
 *
 *   x       DEVICE pointer, [B][Cin][H][W] contiguous (NCHW), element type per dtype, read-only
 *   w       DEVICE pointer, [Cout][Cin][n][n] contiguous, same element type as x, read-only,
 *           used as printed in Eqs. 1-4 (no flip; note torch's ConvTranspose2d weight is
 *           [Cin][Cout][k][k] and flipped relative to this)
 *   y       DEVICE pointer, [B][Cout][OH][OW] contiguous fp32 (bf16 for UKST_BF16_BF16), every
 *           element overwritten,
 *           nothing outside it touched; must not overlap x or w
 *   B..P    sizes as above; 1 <= n <= UKST_MAX_N, P >= 0 (any P, also P > n-1: windows that
 *           meet no input give +0)
 *   dtype   a ukst_dtype
 *   stream  a hipStream_t (as void*), or NULL for the default stream
 *
 * Only element alignment is required (4 bytes fp32, 2 bytes bf16, for y too; UKST_ERR_UNSUPPORTED
 * otherwise).
 * The matrix-core kernels additionally want w (and x, for bf16 and for fp32 layers with at most 4
 * output channels) aligned to 16 bytes: when they are not, ukst_conv_transpose2d uses the vector-ALU kernels instead.  The caller owns all buffers;
 * the call enqueues work on `stream` and returns without synchronising.  Arguments are validated
 * on the host before anything touches the GPU; on a validation error nothing is launched.  A
 * failing launch is reported as UKST_ERR_LAUNCH.  This entry point (like the two below it) takes
 * no workspace and uses only kernels that need none; see ukst_conv_transpose2d_ws.
 * Returns a ukst_status.
 */
int ukst_conv_transpose2d(const void* x, const void* w, void* y, int B, int Cin, int Cout, int H,
                          int W, int n, int P, int dtype, void* stream);

/*
 * Same operation with the kernel family forced (tests and benchmarks compare the families on one
 * shape).  path = UKST_PATH_AUTO behaves exactly like ukst_conv_transpose2d.  Returns
 * UKST_ERR_UNSUPPORTED if that family cannot run the shape (or, for UKST_PATH_MFMA, buffers that
 * are not 16-byte aligned).
 */
int ukst_conv_transpose2d_path(const void* x, const void* w, void* y, int B, int Cin, int Cout,
                               int H, int W, int n, int P, int dtype, int path, void* stream);

typedef enum { UKST_ACT_NONE = 0, UKST_ACT_RELU = 1, UKST_ACT_TANH = 2 } ukst_activation;

/*
 * The same transpose convolution with the epilogue of a generator layer fused into the store:
 *     y[b][co] = act( (x (*) w)[b][co] + bias[co] )
 * so that the output is written once instead of being read and rewritten by an elementwise pass
 * (the unified kernel of Sec. 3 produces every output element exactly once, which is what makes
 * the fusion possible; bias and activation themselves are not part of the paper).
 *   bias  DEVICE pointer to Cout fp32 values, or NULL for none
 *   act   a ukst_activation (ReLU: max(v, 0); tanh: fp32, absolute error below 1e-6)
 *   path  as in ukst_conv_transpose2d_path
 * Everything else, including error behaviour, as ukst_conv_transpose2d; an unknown `act` gives
 * UKST_ERR_UNSUPPORTED.  With bias == NULL and act == UKST_ACT_NONE the result is bit-identical
 * to ukst_conv_transpose2d_path.
 */
int ukst_conv_transpose2d_bias_act(const void* x, const void* w, const float* bias, void* y, int B,
                                   int Cin, int Cout, int H, int W, int n, int P, int dtype,
                                   int act, int path, void* stream);

/* The operations that may want a workspace (argument `op` of ukst_workspace_bytes). */
typedef enum { UKST_OP_FORWARD = 0, UKST_OP_GRAD_INPUT = 1, UKST_OP_GRAD_WEIGHT = 2 } ukst_op;

/*
 * Bytes of scratch memory the given operation uses on this problem (host arithmetic only, a
 * function of the arguments alone; 0 if the operation needs none, or on invalid arguments).
 *   UKST_OP_FORWARD      layers with fewer output tiles than compute units on the fp32
 *                        matrix-core path divide the input channels of a tile among 2, 4 or 8
 *                        blocks; each slice writes its partial sums to its own copy of y in the
 *                        workspace and a second kernel adds the copies in slice order.
 *   UKST_OP_GRAD_INPUT   matrix-core kernels (Cin >= 32, Cout >= 16): the weights re-packed once
 *                        per call, plus, for layers with few pixels, one copy of dx per slice of
 *                        the sum over output channels (added in slice order).
 *   UKST_OP_GRAD_WEIGHT  one copy of dw per slice of the sum over batch and space (added in a
 *                        fixed order); every kernel of this operation needs it.
 * The workspace is caller-owned DEVICE memory, 256-byte aligned, needs no initialisation, holds
 * nothing of value after the call's work has finished on its stream, and must not be used by
 * another call that may run concurrently.
 */
size_t ukst_workspace_bytes(int op, int B, int Cin, int Cout, int H, int W, int n, int P, int dtype);

/*
 * ukst_conv_transpose2d_bias_act with a workspace (Algorithm 2, as above; bias == NULL and
 * act == UKST_ACT_NONE give the plain transpose convolution).
 *   workspace        DEVICE pointer as described at ukst_workspace_bytes, or NULL
 *   workspace_bytes  its size
 * With workspace == NULL (and workspace_bytes == 0) the call behaves like
 * ukst_conv_transpose2d_bias_act: layers that would split their input channels keep the whole sum
 * in one block per tile instead (same result up to fp32 summation order, fewer blocks).  With a
 * workspace smaller than ukst_workspace_bytes(UKST_OP_FORWARD, ...) for a layer that uses one the
 * call returns UKST_ERR_WORKSPACE and launches nothing.  Results are bit-reproducible either way.
 */
int ukst_conv_transpose2d_ws(const void* x, const void* w, const float* bias, void* y, int B, int Cin,
                             int Cout, int H, int W, int n, int P, int dtype, int act, int path,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward pass of the same layer: the gradients of  L = sum(dy * y)  for y = the transpose
 * convolution above (Algorithm 1 is the definition; these are its adjoints).  The paper measures
 * the forward layer only; the parity structure of Sec. 3.1 carries over: input pixel (i, j) meets
 * output pixel (oy, ox) through tap (2i+P-oy, 2j+P-ox), so both gradients run over a stride-2
 * lattice of dy and never touch an inserted zero:
 *
 *   dx[b,ci,i,j]  = sum_co sum_{a,c<n} dy[b,co,2i+P-a,2j+P-c] * w[co,ci,a,c]
 *   dw[co,ci,a,c] = sum_b  sum_{i,j}   x[b,ci,i,j] * dy[b,co,2i+P-a,2j+P-c]
 *
 * with terms whose output pixel lies outside [0,OH) x [0,OW) left out.
 *
 *   dy      DEVICE pointer, [B][Cout][OH][OW] contiguous, read-only
 *   w / x   DEVICE pointers with the layouts of ukst_conv_transpose2d, read-only
 *   dx      DEVICE pointer, [B][Cin][H][W] contiguous fp32, every element overwritten
 *   dw      DEVICE pointer, [Cout][Cin][n][n] contiguous fp32, every element overwritten
 *   dtype   UKST_F32 (all fp32) or UKST_BF16_F32 (the two operands bf16, the gradient fp32,
 *           fp32 accumulation); UKST_BF16_BF16 gives UKST_ERR_UNSUPPORTED
 *   workspace, workspace_bytes   caller-owned scratch of at least
 *           ukst_workspace_bytes(UKST_OP_GRAD_INPUT / UKST_OP_GRAD_WEIGHT, ...) bytes (NULL and 0
 *           where that is 0); UKST_ERR_WORKSPACE otherwise, with nothing launched
 *   B..P, stream, alignment (element alignment only), ownership, asynchrony and error behaviour
 *   as for ukst_conv_transpose2d; outputs must not overlap inputs.
 *
 * Partial results are added in a fixed order: both gradients are bit-reproducible.
 */
int ukst_conv_transpose2d_grad_input(const void* dy, const void* w, void* dx, int B, int Cin,
                                     int Cout, int H, int W, int n, int P, int dtype,
                                     void* workspace, size_t workspace_bytes, void* stream);
int ukst_conv_transpose2d_grad_weight(const void* x, const void* dy, void* dw, int B, int Cin,
                                      int Cout, int H, int W, int n, int P, int dtype,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * ukst_conv_transpose2d_grad_weight for callers that cannot allocate or carry a workspace (code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid allocation): the
 * partial sums live in a static device array that is part of the library, ukst_static_workspace_bytes()
 * = 64 MiB per GPU, held from the first use on that GPU until the process ends.  Same kernels,
 * same results (bit for bit) as ukst_conv_transpose2d_grad_weight; no hipMalloc, hipFree or other
 * allocating call is made.  Problems whose ukst_workspace_bytes(UKST_OP_GRAD_WEIGHT, ...) exceeds
 * that size return UKST_ERR_WORKSPACE with nothing launched (every benchmark configuration fits).
 * All calls on one GPU share the one array: calls that may overlap on a GPU (different streams,
 * different threads) race on it and must be serialised by the caller.  Everything else as
 * ukst_conv_transpose2d_grad_weight.
 */
int ukst_conv_transpose2d_grad_weight_static(const void* x, const void* dy, void* dw, int B, int Cin,
                                             int Cout, int H, int W, int n, int P, int dtype,
                                             void* stream);
size_t ukst_static_workspace_bytes(void);

/*
 * Name of the main device kernel a backward call launches for this problem (which = 0:
 * ukst_conv_transpose2d_grad_input, 1: ukst_conv_transpose2d_grad_weight), as it appears in a
 * profiler's kernel trace (substring match), or "" on invalid arguments.  Static storage.
 * Wide layers (Cin >= 32, Cout >= 16) run the input gradient on the matrix cores
 * ("ukst_grad_input_window_mfma_bf16_kernel": bf16 operands, 2 <= n <= 4, Cin > 64 and a multiple of 8,
 * Cout a multiple of 8, W >= 16 -- bf16 MFMA with an output channel's 16 taps as the contraction;
 * "ukst_grad_input_mfma_bf16_kernel": bf16 MFMA for other bf16 operands where its LDS tile fits,
 * i.e. kernel sides up to about 5;
 * "ukst_grad_input_mfma_kernel": fp32 MFMA otherwise; weights packed once per call into the
 * workspace, which also holds the copies of dx when the sum over output channels is split),
 * layers with Cin, Cout >= 32 run the kernel gradient there too
 * ("ukst_grad_weight_mfma_bf16_kernel": bf16 MFMA with the pixel axis as the contraction, for bf16
 * operands with kernel sides 2 to 4, W a multiple of 8 and at least 16;
 * "ukst_grad_weight_mfma_kernel": fp32 MFMA for everything else of that width, either dtype).
 * Layers with at most 4 output channels, Cout * n * n <= 64 and Cin >= 16 run the kernel gradient
 * as "ukst_grad_weight_thin_mfma_kernel" (fp32 MFMA whose rows are (channel, tap) pairs).
 * Narrow fp32 layers (Cin, Cout <= 4, 2 <= n <= 5, W >= 32) run both gradients as
 * "ukst_grad_input_narrow_kernel" / "ukst_grad_weight_narrow_kernel" (register-blocked strips on
 * the vector ALUs, no LDS).  Everything else runs on the general vector-ALU kernels.
 */
const char* ukst_grad_kernel_name(int which, int B, int Cin, int Cout, int H, int W, int n, int P,
                                  int dtype);

/*
 * The two generalisations the paper's discussion (Sec. 5) points to.  Both use the computation
 * pattern of Algorithm 2 -- every output pixel selects, from its own coordinates, the taps that
 * can meet data, and no inserted zero is ever multiplied -- in one general vector-ALU kernel.
 *
 * ukst_conv_transpose2d_strided: transpose convolution with stride s (Algorithm 1 with s-1 zeros
 * between neighbouring pixels; s = 2 is ukst_conv_transpose2d).  s*s parity classes: output row oy
 * has class r = (P - oy) mod s and uses taps r, r+s, ... on input rows (oy + r - P)/s + u.
 *     y[b,co,oy,ox] = sum_ci sum_{a,c<n} U_P[b,ci,oy+a,ox+c] * w[co,ci,a,c],  U[s*i][s*j] = x[i][j]
 *     OH = s(H-1) + 2P - n + 2,  OW = s(W-1) + 2P - n + 2
 *
 * ukst_dilated_conv2d: stride-1 convolution (correlation, no flip) with dilation d: the KERNEL is
 * the bed of nails (d-1 zeros between neighbouring taps), the input is zero-padded by P, and the
 * pattern is applied to the segregated input -- an output pixel only meets the sub-sampled input
 * map of its own residue modulo d, read in place.
 *     y[b,co,oy,ox] = sum_ci sum_{a,c<n} xpad[b,ci,oy+d*a,ox+d*c] * w[co,ci,a,c]
 *     OH = H + 2P - d(n-1),  OW = W + 2P - d(n-1)
 *
 * Pointers, layouts ([B][Cin][H][W], [Cout][Cin][n][n], [B][Cout][OH][OW] fp32), alignment,
 * ownership, asynchrony and error codes as for ukst_conv_transpose2d; dtype UKST_F32 or
 * UKST_BF16_F32 (UKST_BF16_BF16: UKST_ERR_UNSUPPORTED); 1 <= s, d <= UKST_MAX_STEP (larger:
 * UKST_ERR_UNSUPPORTED; < 1 or an empty output: UKST_ERR_SHAPE).  No workspace is used.
 * ukst_output_shape_* and ukst_mac_count_* are host arithmetic only (kinds as ukst_mac_count:
 * 0 exact in-range products, 1 what the segregated pattern executes, 2 what the definition with
 * its inserted zeros executes; 0 on invalid arguments).
 */
int ukst_output_shape_strided(int H, int W, int n, int P, int s, int* OH, int* OW);
int ukst_output_shape_dilated(int H, int W, int n, int P, int d, int* OH, int* OW);
int ukst_conv_transpose2d_strided(const void* x, const void* w, void* y, int B, int Cin, int Cout,
                                  int H, int W, int n, int P, int s, int dtype, void* stream);
int ukst_dilated_conv2d(const void* x, const void* w, void* y, int B, int Cin, int Cout, int H,
                        int W, int n, int P, int d, int dtype, void* stream);
unsigned long long ukst_mac_count_strided(int B, int Cin, int Cout, int H, int W, int n, int P,
                                          int s, int kind);
unsigned long long ukst_mac_count_dilated(int B, int Cin, int Cout, int H, int W, int n, int P,
                                          int d, int kind);

/*
 * Name of the device kernel the given path launches for this problem, as it appears in a
 * profiler's kernel trace (substring match), or "" on invalid arguments.  Static storage.
 */
const char* ukst_kernel_name(int B, int Cin, int Cout, int H, int W, int n, int P, int dtype,
                             int path);

#ifdef __cplusplus
}
#endif
#endif /* UKST_H */
