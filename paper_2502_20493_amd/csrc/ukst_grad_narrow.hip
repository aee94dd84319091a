// Backward pass of narrow fp32 layers (Cin, Cout <= 4, 2 <= n <= 5, maps at least 32 wide): the
// image layers, where both gradients are bound by memory traffic and not by arithmetic.
//
// Input pixel (i,j) meets output pixel (2i+P-k, 2j+P-l) through tap (k,l) (Eqs. 1-4 read
// backwards), so four consecutive input columns j0..j0+3 meet the n+6 dy columns that start at
// 2 j0 + P - (n-1), in the rows 2i + P - k.  A lane owns such a strip of four columns, a wave 256
// consecutive columns of one row, and every index of the arithmetic is a
// compile-time constant: the dy window of a row sits in n+6 registers.  No LDS staging.
//
// Edges are left to the buffer addressing hardware, as in the narrow forward kernel: a row is
// described by a scalar offset (its start) and a size (its end; zero for a row that does not
// exist), dwords past the end come back as zeros one by one and stores past the end are dropped.
// A window may begin up to n-1 columns left of the row; an offset there would lie inside the row
// before, so such a lane (the first of a row) gets an offset that is out of range for every row and
// fetches its in-row columns one by one.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef const float __attribute__((address_space(4)))* scalar_fptr;  // read through the scalar cache
constexpr int kRsrcFlags = 0x00020000;      // raw 32-bit buffer, gfx9 family
constexpr unsigned kLeftOfRow = 0x7FFF0000u;  // plus any row start below 2^31: beyond every row end

constexpr int PXL = 4;  // input columns per lane: a wave covers 64 * PXL columns of a row (2 was no faster)
constexpr int OWN = 2 * PXL;  // dy columns a lane fetches itself
constexpr int window_regs(int n) { return OWN + 4; }  // + n - 2 <= 3 columns of the next lane

// The n+6 dy columns that start at column c0 = 8 * lane + const (may be negative in lane 0) of the
// row described by (rs, row_off).  Neighbouring lanes' windows overlap in n-2 columns: a lane
// fetches its own eight columns with two 16-byte loads (consecutive lanes, consecutive 32-byte
// runs: every cache line is asked for once per load) and takes the rest from the lane above with
// a wave shift; the last lane fetches them itself.  A 16-byte load that begins left of the row
// returns nothing, so a lane whose window does fetches those columns one by one.
template <int N>
__device__ __forceinline__ void load_window(__amdgpu_buffer_rsrc_t rs, int c0, unsigned row_off, int lane,
                                            float (&v)[window_regs(N)])
{
    {
        const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rs, c0 < 0 ? kLeftOfRow : (unsigned)(4 * c0), row_off, 0);
        const unsigned t[4] = {q.x, q.y, q.z, q.w};  // by value: a bit cast of a vector element reads element 0
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(t[e]);
    }
#pragma unroll
    for (int m = 4; m < OWN; m += 4) {  // c0 + 4 >= 0: a window begins at most four columns left of its row
        const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rs, (unsigned)(4 * (c0 + m)), row_off, 0);
        const unsigned t[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) v[m + e] = __uint_as_float(t[e]);
    }
    if (c0 < 0) {
#pragma unroll
        for (int m = 1; m < 4; ++m)
            if (c0 + m >= 0) v[m] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, (unsigned)(4 * (c0 + m)), row_off, 0));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)  // lane i takes lane i + 1's (wave_shl:1), zeros into lane 63
        v[OWN + e] = e < N - 2 ? __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v[e]), 0x130, 0xF, 0xF, true)) : 0.f;
    if (N > 2 && lane == 63) {
        const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rs, (unsigned)(4 * (c0 + OWN)), row_off, 0);
        const unsigned t[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) v[OWN + e] = __uint_as_float(t[e]);
    }
}

// sum over the 64 lanes, valid in lane 63: an inclusive scan over each row of 16 lanes (row shifts
// by 1, 2, 4, 8, zeros moving in), then the row totals passed on to the rows above
__device__ __forceinline__ float wave_sum_to_last(float v)
{
#define UKST_DPP_ADD(ctrl, rmask)                                                                   \
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rmask, 0xF, true))
    UKST_DPP_ADD(0x111, 0xF);  // row_shr:1
    UKST_DPP_ADD(0x112, 0xF);  // row_shr:2
    UKST_DPP_ADD(0x114, 0xF);  // row_shr:4
    UKST_DPP_ADD(0x118, 0xF);  // row_shr:8
    UKST_DPP_ADD(0x142, 0xA);  // row_bcast:15 into rows 1 and 3
    UKST_DPP_ADD(0x143, 0xC);  // row_bcast:31 into rows 2 and 3
#undef UKST_DPP_ADD
    return v;
}

struct NarrowGradArgs {
    GeomBase g;
    int chunks;         // 256-column chunks per row
    int nUnits;         // wave work items: (image, row, chunk)
    int unitsPerWave;   // kernel gradient: consecutive items a wave adds up
};

// Kernel gradient.  grid = (blocks, Cout): a block's eight waves each add up unitsPerWave
// (image, row, chunk) items of one output channel in CI * n * n registers per lane, the lanes are
// summed with row shifts, the waves through LDS in wave order, and the block writes its copy of
// dw[co]; the copies are added in a fixed order afterwards.
constexpr int GW_WAVES = 8;  // waves per block of the kernel gradient: one copy of dw per 8 waves

template <int N, int CI>
__global__ __launch_bounds__(64 * GW_WAVES) void ukst_grad_weight_narrow_kernel(const float* __restrict__ x,
                                                                     const float* __restrict__ dy,
                                                                     float* __restrict__ part, NarrowGradArgs a)
{
    constexpr int NWP = window_regs(N), NN = N * N;
    __shared__ float red[GW_WAVES][CI * NN];
    const GeomBase& g = a.g;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int co = blockIdx.y;
    const int wid = blockIdx.x * GW_WAVES + wave;
    const size_t xplane = (size_t)g.H * g.W, yplane = (size_t)g.OH * g.OW;
    const unsigned xrow = (unsigned)g.W * 4u, yrow = (unsigned)g.OW * 4u;

    float acc[CI][N][N];
#pragma unroll
    for (int c = 0; c < CI; ++c)
#pragma unroll
        for (int k = 0; k < N; ++k)
#pragma unroll
            for (int l = 0; l < N; ++l) acc[c][k][l] = 0.f;

    const int u_end = (wid + 1) * a.unitsPerWave < a.nUnits ? (wid + 1) * a.unitsPerWave : a.nUnits;
    for (int u = wid * a.unitsPerWave; u < u_end; ++u) {  // uniform
        const int chunk = u % a.chunks, r = u / a.chunks;
        const int i = r % g.H, b = r / g.H;
        const int j0 = chunk * (64 * PXL) + PXL * lane;
        float xv[CI][PXL];
#pragma unroll
        for (int c = 0; c < CI; ++c) {
            // row i of plane (b, c): dwords past its end are zeros
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(x + ((size_t)b * g.Cin + c) * xplane), 0, (int)((unsigned)(i + 1) * xrow), kRsrcFlags);
            if constexpr (PXL == 4) {
                const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rs, (unsigned)(4 * j0), (unsigned)i * xrow, 0);
                const unsigned t[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int e = 0; e < PXL; ++e) xv[c][e] = __uint_as_float(t[e]);
            } else {
                const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rs, (unsigned)(4 * j0), (unsigned)i * xrow, 0);
                const unsigned t[2] = {q.x, q.y};
#pragma unroll
                for (int e = 0; e < PXL; ++e) xv[c][e] = __uint_as_float(t[e]);
            }
        }
        float row[N][NWP];
        const float* plane = dy + ((size_t)b * g.Cout + co) * yplane;
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const int oy = 2 * i + g.P - k;
            const bool have = oy >= 0 && oy < g.OH;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)plane, 0, have ? (int)((unsigned)(oy + 1) * yrow) : 0, kRsrcFlags);
            load_window<N>(rs, 2 * j0 + g.P - (N - 1), have ? (unsigned)oy * yrow : 0u, lane, row[k]);
        }
        // pixel p of the strip meets dy column 2 (j0 + p) + P - l = window column 2 p + (N - 1 - l)
#pragma unroll
        for (int c = 0; c < CI; ++c)
#pragma unroll
            for (int k = 0; k < N; ++k)
#pragma unroll
                for (int l = 0; l < N; ++l)
#pragma unroll
                    for (int p = 0; p < PXL; ++p) acc[c][k][l] = fmaf(row[k][2 * p + (N - 1 - l)], xv[c][p], acc[c][k][l]);
    }

#pragma unroll
    for (int c = 0; c < CI; ++c)
#pragma unroll
        for (int k = 0; k < N; ++k)
#pragma unroll
            for (int l = 0; l < N; ++l) {
                const float s = wave_sum_to_last(acc[c][k][l]);
                if (lane == 63) red[wave][(c * N + k) * N + l] = s;
            }
    __syncthreads();
    if (threadIdx.x < CI * NN) {
        const int t = threadIdx.x;
        float s = red[0][t];
#pragma unroll
        for (int wv = 1; wv < GW_WAVES; ++wv) s += red[wv][t];
        part[((size_t)blockIdx.x * g.Cout + co) * (CI * NN) + t] = s;
    }
}

// dw[e] = sum of the copies in the order 0, 1, 2, ...: 64 lanes per element take every 64th copy,
// their sums are added with the same row shifts
__global__ __launch_bounds__(256) void ukst_sum_copies_narrow_kernel(const float* __restrict__ part,
                                                                    float* __restrict__ dw, int elems, int copies)
{
    const int lane = threadIdx.x & 63;
    const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (e >= elems) return;  // whole waves
    float s = 0.f;
    for (int c = lane; c < copies; c += 64) s += part[(size_t)c * elems + e];
    s = wave_sum_to_last(s);
    if (lane == 63) dw[e] = s;
}

// Input gradient.  A wave owns 256 columns of one row of one image (two rows per wave share a dy
// row but halve the waves: 16.8 us instead of 14.7 on the 224 x 224 image layer, four rows 24.3), a
// lane four of the columns for every input channel; per output channel the n dy rows the row meets
// are fetched (n+6 dwords each) and multiplied with the channel's weights, which come through the
// scalar cache.  One 16-byte store per lane and channel.
template <int N, int CI>
__global__ __launch_bounds__(256) void ukst_grad_input_narrow_kernel(const float* __restrict__ dy,
                                                                    const float* __restrict__ w,
                                                                    float* __restrict__ dx, NarrowGradArgs a)
{
    constexpr int NWP = window_regs(N), NN = N * N;
    const GeomBase& g = a.g;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int u = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + wave;
    if (u >= a.nUnits) return;  // whole waves, no barrier below
    const int chunk = u % a.chunks, r = u / a.chunks;
    constexpr int RH = 1;  // input rows per wave
    const int hp = (g.H + RH - 1) / RH;
    const int i0 = RH * (r % hp), b = r / hp;
    const int j0 = chunk * (64 * PXL) + PXL * lane;
    const size_t xplane = (size_t)g.H * g.W, yplane = (size_t)g.OH * g.OW;
    const unsigned xrow = (unsigned)g.W * 4u, yrow = (unsigned)g.OW * 4u;
    const scalar_fptr ws = (scalar_fptr)(unsigned long long)w;

    float acc[RH][CI][PXL];
#pragma unroll
    for (int h = 0; h < RH; ++h)
#pragma unroll
        for (int c = 0; c < CI; ++c)
#pragma unroll
            for (int p = 0; p < PXL; ++p) acc[h][c][p] = 0.f;

    const int oy0 = 2 * i0 + g.P - (N - 1);  // first dy row the row pair meets
    // output channels per group whose dy rows are all requested before the first is used.  One at a
    // time is fastest (cfg2a 16.8 us; two 18.0, all three 18.9): the 64 registers of that form let
    // every wave of the grid be resident at once, and that, not a wave's own round trips, is what
    // covers the memory latency here
    constexpr int CG = 1;
    for (int cg = 0; cg < g.Cout; cg += CG) {
        float row[CG][N + 2 * RH - 2][NWP];
#pragma unroll
        for (int q = 0; q < CG; ++q) {
            const bool chan = cg + q < g.Cout;  // uniform
            const float* plane = dy + ((size_t)b * g.Cout + (chan ? cg + q : 0)) * yplane;
#pragma unroll
            for (int rr = 0; rr < N + 2 * RH - 2; ++rr) {
                const int oy = oy0 + rr;
                const bool have = chan && oy >= 0 && oy < g.OH;
                const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                    (void*)plane, 0, have ? (int)((unsigned)(oy + 1) * yrow) : 0, kRsrcFlags);
                load_window<N>(rs, 2 * j0 + g.P - (N - 1), have ? (unsigned)oy * yrow : 0u, lane, row[q][rr]);
            }
        }
        // input row i0 + h meets dy row 2 (i0 + h) + P - k = oy0 + 2 h + (N - 1 - k)
#pragma unroll
        for (int q = 0; q < CG; ++q) {
            if (cg + q >= g.Cout) break;  // uniform
#pragma unroll
            for (int c = 0; c < CI; ++c)
#pragma unroll
                for (int k = 0; k < N; ++k)
#pragma unroll
                    for (int l = 0; l < N; ++l) {
                        const float wv = ws[((size_t)(cg + q) * g.Cin + c) * NN + k * N + l];
#pragma unroll
                        for (int h = 0; h < RH; ++h)
#pragma unroll
                            for (int p = 0; p < PXL; ++p)
                                acc[h][c][p] = fmaf(row[q][2 * h + (N - 1 - k)][2 * p + (N - 1 - l)], wv, acc[h][c][p]);
                    }
        }
    }
#pragma unroll
    for (int h = 0; h < RH; ++h) {
        const int i = i0 + h;
        const bool have = i < g.H;
#pragma unroll
        for (int c = 0; c < CI; ++c) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(dx + ((size_t)b * g.Cin + c) * xplane), 0, have ? (int)((unsigned)(i + 1) * xrow) : 0, kRsrcFlags);
            // the whole offset in the vector offset, scalar offset a literal 0: the form of a 16-byte
            // store whose data registers the compiler keeps apart from the next write to them
            const unsigned off = (unsigned)(4 * j0) + (have ? (unsigned)i * xrow : 0u);
            if constexpr (PXL == 4) {
                u32x4 q;
                q.x = __float_as_uint(acc[h][c][0]); q.y = __float_as_uint(acc[h][c][1]);
                q.z = __float_as_uint(acc[h][c][2]); q.w = __float_as_uint(acc[h][c][3]);
                __builtin_amdgcn_raw_buffer_store_b128(q, rs, off, 0, 0);
            } else {
                u32x2 q;
                q.x = __float_as_uint(acc[h][c][0]); q.y = __float_as_uint(acc[h][c][1]);
                __builtin_amdgcn_raw_buffer_store_b64(q, rs, off, 0, 0);
            }
        }
    }
}

bool narrow_args(const Geom& g, int dtype, NarrowGradArgs& a)
{
    if (dtype != 0 || g.Cin > 4 || g.Cout > 4 || g.n < 2 || g.n > 5 || g.W < 32) return false;
    // rows are addressed with 32-bit byte offsets inside their plane
    if ((size_t)g.H * g.W * 4 >= 0x7FFF0000u || (size_t)g.OH * g.OW * 4 >= 0x7FFF0000u) return false;
    a.g = g;
    a.chunks = (g.W + 64 * PXL - 1) / (64 * PXL);
    if ((long long)g.B * g.H * a.chunks > 0x3fffffffLL) return false;  // work items are counted in an int
    return true;
}

template <int N, int CI>
hipError_t launch_gw_narrow(NarrowGradArgs a, const void* x, const void* dy, float* dw, Workspace& ws,
                            hipStream_t stream)
{
    const GeomBase& g = a.g;
    const long long units = (long long)g.B * g.H * a.chunks;
    if (units > 0x3fffffffLL) return hipErrorInvalidConfiguration;
    a.nUnits = (int)units;
    // about 8192 waves over the whole grid (one or two work items each: what hides the memory
    // latency is the number of waves in flight); a figure of the shape alone, so that the workspace
    // size is host arithmetic
    hipError_t e;
    long long waves = 8192 / g.Cout;
    if (waves < GW_WAVES) waves = GW_WAVES;
    if (waves > units) waves = units;
    a.unitsPerWave = (int)((units + waves - 1) / waves);
    const int nwaves = (int)((units + a.unitsPerWave - 1) / a.unitsPerWave);
    const int blocks = (nwaves + GW_WAVES - 1) / GW_WAVES;
    const int elems = g.Cout * CI * N * N;
    const size_t need = (size_t)blocks * elems * sizeof(float);
    if (ws.query) { ws.need = need; return hipSuccess; }
    if (ws.bytes < need) return kWorkspaceTooSmall;
    float* part = (float*)ws.ptr;
    hipLaunchKernelGGL((ukst_grad_weight_narrow_kernel<N, CI>), dim3((unsigned)blocks, (unsigned)g.Cout), dim3(64 * GW_WAVES), 0,
                       stream, (const float*)x, (const float*)dy, part, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(ukst_sum_copies_narrow_kernel, dim3((unsigned)((elems + 3) / 4)), dim3(256), 0, stream,
                       (const float*)part, dw, elems, blocks);
    return hipGetLastError();
}

template <int N, int CI>
hipError_t launch_gi_narrow(NarrowGradArgs a, const void* dy, const void* w, float* dx, hipStream_t stream)
{
    const GeomBase& g = a.g;
    const long long units = (long long)g.B * ((g.H + 1 - 1) / 1) * a.chunks;
    if (units > 0x3fffffffLL) return hipErrorInvalidConfiguration;
    a.nUnits = (int)units;
    a.unitsPerWave = 1;
    hipLaunchKernelGGL((ukst_grad_input_narrow_kernel<N, CI>), dim3((unsigned)((units + 3) / 4)), dim3(256), 0, stream,
                       (const float*)dy, (const float*)w, dx, a);
    return hipGetLastError();
}

template <int N>
hipError_t launch_narrow_n(int which, const NarrowGradArgs& a, const void* p0, const void* p1, float* out,
                           Workspace& ws, hipStream_t stream)
{
    switch (a.g.Cin) {
        case 1: return which ? launch_gw_narrow<N, 1>(a, p0, p1, out, ws, stream) : launch_gi_narrow<N, 1>(a, p0, p1, out, stream);
        case 2: return which ? launch_gw_narrow<N, 2>(a, p0, p1, out, ws, stream) : launch_gi_narrow<N, 2>(a, p0, p1, out, stream);
        case 3: return which ? launch_gw_narrow<N, 3>(a, p0, p1, out, ws, stream) : launch_gi_narrow<N, 3>(a, p0, p1, out, stream);
        default: return which ? launch_gw_narrow<N, 4>(a, p0, p1, out, ws, stream) : launch_gi_narrow<N, 4>(a, p0, p1, out, stream);
    }
}

}  // namespace

bool grad_narrow_supported(const Geom& g, int dtype)
{
    NarrowGradArgs a;
    return narrow_args(g, dtype, a);
}

// which 0: (p0, p1) = (dy, w) -> dx (no scratch); which 1: (p0, p1) = (x, dy) -> dw (one copy of dw per block)
hipError_t launch_grad_narrow(int which, const Geom& g, const void* p0, const void* p1, float* out, Workspace& ws,
                              hipStream_t stream)
{
    NarrowGradArgs a;
    if (!narrow_args(g, 0, a)) return hipErrorInvalidValue;
    if (which == 0 && ws.query) return hipSuccess;
    switch (g.n) {
        case 2: return launch_narrow_n<2>(which, a, p0, p1, out, ws, stream);
        case 3: return launch_narrow_n<3>(which, a, p0, p1, out, ws, stream);
        case 4: return launch_narrow_n<4>(which, a, p0, p1, out, ws, stream);
        default: return launch_narrow_n<5>(which, a, p0, p1, out, ws, stream);
    }
}

}  // namespace ukst
