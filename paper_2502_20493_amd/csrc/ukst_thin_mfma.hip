// Thin-output layers on the matrix cores (fp32, Cout <= 4, n = 3 or 4, Cin a multiple of 16): the
// last layer of a generator, e.g. 64 -> 3 channels.
//
// With so few output channels the channel axis cannot fill an MFMA tile, but the four parity
// classes of Algorithm 2 can: all classes of a quad read the same 2 x 2 input window (see
// ukst_internal.h), so with
//
//     A[quad][(ci, u, v)]        = x[ci][k - P + u][m - P + v]            (0 outside the map)
//     B[(ci, u, v)][(co, r, s)]  = w[co][ci][r + 2u][s + 2v]              (0 if the tap does not exist)
//
// the whole layer is ONE dense product D = A * B with M = quads (flattened over image, quad row
// and quad column), K = 4 Cin and N = 4 Cout <= 16 columns: column (co, r, s) of D is parity
// class (r, s) of output channel co (Eqs. 1-4), and no column of B multiplies a bed-of-nails zero
// (for n = 3 the classes with fewer taps carry zeros in B instead: 9 of 16 entries are real).
// v_mfma_f32_16x16x4_f32 fits exactly: one instruction takes 16 quads, one input channel (its
// four window positions are the four K values) and all 16 columns.
//
// Block = 4 waves, 64*MT consecutive quads; a wave owns MT tiles of 16 quads.  Input channels
// advance 16 per stage: the rows of x that the block's quads touch go to LDS as [ci][row][col]
// with 16-byte loads and stores (zero columns on both sides stand for the floor(P/2) padding of
// Sec. 3.4, rows that do not exist are loaded through an out-of-range offset and arrive as
// zeros), the stage's slice of B goes next to them.  The layer is bound by how fast x arrives,
// so every block keeps the loads of the next DEPTH stages in flight in a ring of register sets
// (two sets leave room for four blocks per compute unit, which measured faster than a deeper ring
// with three); the first stage is requested before anything else is set up, the second only
// after the set-up, so that the first requests of all waves reach memory ahead of any second.
// Per MFMA a lane reads one float of A (its quad, its window position) and per channel one float
// of B from LDS.
//
// Epilogue: an accumulator lane holds one column (co, r, s) for 4 consecutive quads.  Lanes s = 1
// and s = 0 are neighbours, so one DPP swap gives each lane both column classes of two quads,
// which it stores as 8-byte pairs: the classes are interleaved in place.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));

constexpr int kRsrcFlags = 0x00020000;   // raw 32-bit buffer, gfx9 family
constexpr unsigned kDrop = 0x80000000u;  // byte offset beyond any buffer this kernel accepts
constexpr int KCH = 16;                  // input channels per stage
constexpr int LPAD = 4;                  // zero columns left of input column 0 in LDS
constexpr int RPAD = 4;                  // and right of the last one
constexpr int NU = 4;                    // 16-byte activation pieces per thread and stage, at most
constexpr int DEPTH = 2;                 // stages in flight ahead of the multiplication (register ring)
constexpr int LDS_LIMIT = 64 * 1024;

struct ThinMfmaArgs {
    GeomBase g;
    int Q;      // total quads = B * KH * KW
    int EH;     // input rows one image's quad rows touch = KH + 1
    int ROWS;   // input rows a stage holds
    int LW;     // floats per staged row = LPAD + W + RPAD
    int XP;     // floats per channel plane of a stage = ROWS * LW
    int W4;     // 16-byte pieces per input row
    int units;  // pieces per stage = KCH * ROWS * W4
    int nqt;    // blocks
    FastDiv dKHW, dKW, dEH, dW4, dROWS;
};

// EPI: the fused epilogue (bias, activation) is compiled into the drain.
template <int N, int MT, bool EPI>
__global__ __launch_bounds__(256) void ukst_thin_mfma_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ w,
                                                            float* __restrict__ y, ThinMfmaArgs a,
                                                            Epilogue ep)
{
    static_assert(N == 3 || N == 4, "2 x 2 window: the four K values of one MFMA");
    constexpr int NN = N * N;
    constexpr int TN = 64 * MT;
    extern __shared__ __align__(16) float lds[];
    float* const xl = lds;               // activations [KCH][ROWS][LW]
    float* const wl = lds + KCH * a.XP;  // B slice [KCH][window position][column (co, r, s)]

    const GeomBase& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KHW = g.KH * g.KW;
    const int q0 = xcd_contiguous(blockIdx.x, gridDim.x) * TN;
    const int q_last = (q0 + TN - 1 < a.Q ? q0 + TN - 1 : a.Q - 1);
    // quad row rho = b*KH + kk uses input rows e = b*EH + kk + u (u < 2)
    const int bf0 = fdiv(q0, a.dKHW), kf0 = fdiv(q0 - bf0 * KHW, a.dKW);
    const int e_first = bf0 * a.EH + kf0;

    // ---- staging units of this thread: piece c4 of row `row` of channel ci_l, c4 fastest so that
    // lanes walk contiguous memory
    unsigned goff[NU];
    int loff[NU];
#pragma unroll
    for (int s = 0; s < NU; ++s) {
        const int un = tid + 256 * s;
        goff[s] = kDrop;
        loff[s] = 0;
        if (un < a.units) {
            const int t2 = fdiv(un, a.dW4), c4 = un - t2 * a.W4;
            const int ci_l = fdiv(t2, a.dROWS), row = t2 - ci_l * a.ROWS;
            const int e = e_first + row;
            const int b = fdiv(e, a.dEH), ii = e - b * a.EH;
            const int i = g.k_min - g.P + ii;
            if (b < g.B && i >= 0 && i < g.H)
                goff[s] = (unsigned)((((b * g.Cin + ci_l) * g.H + i) * g.W + 4 * c4) * 4);
            loff[s] = (ci_l * a.ROWS + row) * a.LW + LPAD + 4 * c4;
        }
    }
    // weights: thread = (output channel, channel of the stage, tap row): the n taps of that row
    const int w_co = tid >> 6, w_ci = (tid >> 2) & 15, w_ta = tid & 3;
    const bool w_active = w_co < g.Cout && w_ta < N;
    const unsigned w_off = w_active ? (unsigned)(((w_co * g.Cin + w_ci) * NN + w_ta * N) * 4) : kDrop;

    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * 4), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)w, 0, (int)((size_t)g.Cout * g.Cin * NN * 4), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        (void*)y, 0, (int)((size_t)g.B * g.Cout * g.OH * g.OW * 4), kRsrcFlags);
    const unsigned x_cstride = (unsigned)(g.H * g.W * 4);  // bytes between input channels

    u4v xr[DEPTH][NU];
    float wr[DEPTH][N];
    auto load_stage = [&](int ci0, u4v (&xs)[NU], float (&ws)[N]) {
#pragma unroll
        for (int s = 0; s < NU; ++s)
            if (256 * s < a.units)  // uniform
                xs[s] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, goff[s], (unsigned)ci0 * x_cstride, 0);
        if constexpr (N == 4) {
            const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rs_w, w_off, (unsigned)(ci0 * NN * 4), 0);
            const unsigned e0 = t.x, e1 = t.y, e2 = t.z, e3 = t.w;  // by value, then bits
            ws[0] = __uint_as_float(e0);
            ws[1] = __uint_as_float(e1);
            ws[2] = __uint_as_float(e2);
            ws[3] = __uint_as_float(e3);
        } else {
#pragma unroll
            for (int p = 0; p < N; ++p)
                ws[p] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                    rs_w, w_off + 4u * p, (unsigned)(ci0 * NN * 4), 0));
        }
    };
    auto store_stage = [&](const u4v (&xs)[NU], const float (&ws)[N]) {
#pragma unroll
        for (int s = 0; s < NU; ++s)
            if (tid + 256 * s < a.units) *reinterpret_cast<u4v*>(xl + loff[s]) = xs[s];
        if (w_active) {
#pragma unroll
            for (int tc = 0; tc < N; ++tc) {
                const int pos = (w_ta >> 1) * 2 + (tc >> 1);  // window position (u, v)
                const int col = (w_ta & 1) * 2 + (tc & 1);    // class (r, s)
                wl[w_ci * 64 + pos * 16 + w_co * 4 + col] = ws[tc];
            }
        }
    };

    const int nstages = g.Cin / KCH;
    load_stage(0, xr[0], wr[0]);

    // ---- zero LDS once: the pad columns and the B entries of taps / channels that do not exist
    // are never written again
    {
        const int n4 = (KCH * a.XP + KCH * 64) / 4;
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        for (int i = tid; i < n4; i += 256) reinterpret_cast<f32x4*>(lds)[i] = z;
    }

    // ---- A operand: lane = (quad i16 of the tile, window position kk = (u, v))
    const int i16 = lane & 15, kk = lane >> 4;
    int aoff[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int q = q0 + (wave * MT + t) * 16 + i16;
        if (q > q_last) q = q_last;
        const int b = fdiv(q, a.dKHW);
        const int rem = q - b * KHW;
        const int kq = fdiv(rem, a.dKW), mm = rem - kq * g.KW;
        const int row = b * a.EH + kq - e_first + (kk >> 1);
        const int col = mm + g.m_min - g.P + (kk & 1) + LPAD;
        aoff[t] = row * a.LW + col;
    }

#pragma unroll
    for (int d = 1; d < DEPTH; ++d)
        if (d < nstages) load_stage(d * KCH, xr[d], wr[d]);

    f32x4 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int base = 0; base < nstages; base += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int st = base + d;
            if (st < nstages) {   // uniform
                __syncthreads();  // zero fill done / previous stage consumed
                store_stage(xr[d], wr[d]);
                if (st + DEPTH < nstages) load_stage((st + DEPTH) * KCH, xr[d], wr[d]);
                __syncthreads();
                const float* xp = xl;
#pragma unroll
                for (int ci = 0; ci < KCH; ++ci) {
                    const float bw = wl[ci * 64 + lane];
#pragma unroll
                    for (int t = 0; t < MT; ++t)
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(xp[aoff[t]], bw, acc[t], 0, 0, 0);
                    xp += a.XP;
                }
            }
        }
    }

    // ---- drain: lane holds column j = (co, r, s) for quads 4*(lane/16) .. +3 of each tile
    const int co = i16 >> 2, r = (i16 >> 1) & 1;
    const bool s1 = (i16 & 1) != 0;  // class s = 1 is the left column of the pair
    float bv = 0.f;
    if constexpr (EPI)
        if (ep.bias && co < g.Cout) bv = ep.bias[co];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        float own[4], par[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            own[e] = acc[t][e];
            // neighbour lane (s flipped): quad_perm [1, 0, 3, 2]
            par[e] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(own[e]), 0xB1, 0xF,
                                                                0xF, true));
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // an s = 1 lane writes quads 0, 1 of its four, its s = 0 neighbour quads 2, 3
            float left = s1 ? own[h] : par[2 + h];
            float right = s1 ? par[h] : own[2 + h];
            if constexpr (EPI) {
                left = epilogue(left, bv, ep.act);
                right = epilogue(right, bv, ep.act);
            }
            const int q = q0 + (wave * MT + t) * 16 + 4 * kk + (s1 ? h : 2 + h);
            const bool ok = q < a.Q && co < g.Cout;
            const int qq = q < a.Q ? q : q_last;
            const int b = fdiv(qq, a.dKHW);
            const int rem = qq - b * KHW;
            const int kq = fdiv(rem, a.dKW), mm = rem - kq * g.KW;
            const int oy = 2 * (g.k_min + kq) - r - g.P;
            const int ox1 = 2 * (g.m_min + mm) - 1 - g.P;  // column of class s = 1; s = 0 is ox1 + 1
            const bool vrow = ok && oy >= 0 && oy < g.OH;
            const bool vl = ox1 >= 0 && ox1 < g.OW, vr = ox1 + 1 < g.OW;
            const unsigned base = (unsigned)((((b * g.Cout + co) * g.OH + oy) * g.OW + ox1) * 4);
            u2v d;
            d.x = __float_as_uint(left);
            d.y = __float_as_uint(right);
            __builtin_amdgcn_raw_buffer_store_b64(d, rs_y, (vrow && vl && vr) ? base : kDrop, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(d.x, rs_y, (vrow && vl && !vr) ? base : kDrop, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(d.y, rs_y, (vrow && !vl && vr) ? base + 4u : kDrop, 0, 0);
        }
    }
}

template <int MT>
bool make_args(const Geom& g, ThinMfmaArgs& a)
{
    constexpr int TN = 64 * MT;
    if (g.n != 3 && g.n != 4) return false;
    if (g.Cout > 4 || g.Cin < KCH || g.Cin % KCH != 0) return false;
    if (g.W % 4 != 0) return false;  // 16-byte row pieces
    // 32-bit byte offsets with room for the out-of-range marker and a channel offset on top
    const long long xbytes = 4LL * g.B * g.Cin * g.H * g.W, ybytes = 4LL * g.B * g.Cout * g.OH * g.OW;
    if (xbytes >= (1LL << 30) || ybytes >= (1LL << 31)) return false;
    // window columns: first = -(P/2), last = m_min + KW - 1 - P + 1; both inside the zero pads
    if ((g.P >> 1) > LPAD) return false;
    if (g.m_min + g.KW - g.P > g.W - 1 + RPAD) return false;
    a.g = g;
    const long long Q = (long long)g.B * g.KH * g.KW;
    if (Q > 0x3FFFFFFFLL) return false;
    a.Q = (int)Q;
    a.EH = g.KH + 1;
    // TN consecutive flattened quads touch at most this many quad rows / images
    const int nrho = (TN - 2) / g.KW + 2;
    const int nimg = (TN - 2) / (g.KH * g.KW) + 2;
    a.ROWS = nrho + nimg;
    a.LW = LPAD + g.W + RPAD;
    a.XP = a.ROWS * a.LW;
    a.W4 = g.W / 4;
    const long long units = (long long)KCH * a.ROWS * a.W4;
    if (units > 256 * NU) return false;
    a.units = (int)units;
    if ((KCH * a.XP + KCH * 64) * 4 > LDS_LIMIT) return false;
    a.nqt = (int)((Q + TN - 1) / TN);
    a.dKHW = make_fastdiv((unsigned)(g.KH * g.KW));
    a.dKW = make_fastdiv((unsigned)g.KW);
    a.dEH = make_fastdiv((unsigned)a.EH);
    a.dW4 = make_fastdiv((unsigned)a.W4);
    a.dROWS = make_fastdiv((unsigned)a.ROWS);
    return true;
}

// Quads per block: as many as possible while the grid still covers the chip about twice.
int pick_mt(const Geom& g, ThinMfmaArgs& a)
{
    ThinMfmaArgs t;
    int best = 0;
    for (int mt : {4, 2, 1}) {
        const bool ok = mt == 4 ? make_args<4>(g, t) : mt == 2 ? make_args<2>(g, t) : make_args<1>(g, t);
        if (!ok) continue;
        best = mt;
        a = t;
        if (t.nqt >= 512) break;
    }
    return best;
}

template <int N, int MT>
hipError_t launch_t(const ThinMfmaArgs& a, const Epilogue& ep, const float* x, const float* w, float* y,
                    hipStream_t stream)
{
    const size_t lds = (size_t)(KCH * a.XP + KCH * 64) * 4;
    if (has_epilogue(ep))
        hipLaunchKernelGGL((ukst_thin_mfma_kernel<N, MT, true>), dim3((unsigned)a.nqt), dim3(256), lds,
                           stream, x, w, y, a, ep);
    else
        hipLaunchKernelGGL((ukst_thin_mfma_kernel<N, MT, false>), dim3((unsigned)a.nqt), dim3(256), lds,
                           stream, x, w, y, a, ep);
    return hipGetLastError();
}

template <int N>
hipError_t launch_n(int mt, const ThinMfmaArgs& a, const Epilogue& ep, const float* x, const float* w,
                    float* y, hipStream_t stream)
{
    switch (mt) {
        case 4: return launch_t<N, 4>(a, ep, x, w, y, stream);
        case 2: return launch_t<N, 2>(a, ep, x, w, y, stream);
        case 1: return launch_t<N, 1>(a, ep, x, w, y, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool thin_mfma_supported(const Geom& g, int dtype)
{
    ThinMfmaArgs a;
    return dtype == 0 && pick_mt(g, a) != 0;
}

hipError_t launch_thin_mfma(const Geom& g, const void* x, const void* w, float* y, hipStream_t stream)
{
    ThinMfmaArgs a;
    const int mt = pick_mt(g, a);
    if (!mt) return hipErrorInvalidValue;
    // both operands move in 16-byte pieces
    if ((((uintptr_t)x | (uintptr_t)w) & 15) != 0) return hipErrorInvalidValue;
    return g.n == 4 ? launch_n<4>(mt, a, g.ep, (const float*)x, (const float*)w, y, stream)
                    : launch_n<3>(mt, a, g.ep, (const float*)x, (const float*)w, y, stream);
}

}  // namespace ukst
