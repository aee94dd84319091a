// MFMA path for fp32 operands: the same parity-class implicit GEMM as the bf16 kernel
// (ukst_mfma.hip), on v_mfma_f32_32x32x2_f32.
//
// Per quad the four parity classes of Algorithm 2 share one ceil(n/2) x ceil(n/2) input window,
// so one B fragment (activations at window position (u, v), two input channels) feeds one MFMA
// per class that owns a tap there, with that class's tap w[co][ci][r+2u][s+2v] as A fragment
// (Eqs. 1-4): n*n MFMA columns per quad tile and channel pair, none spent on a bed-of-nails zero.
// M = output channels, N = quads flattened over (image, quad row, quad column), K = input
// channels.  An fp32 MFMA lane holds ONE K value per operand, so NCHW data needs no transposition:
// activations go to LDS as [k][row][col], weights as [k][tap][channel], with plain 4-byte loads
// (any W, any n <= 5, no alignment requirement).  The matrix pipe needs 16 passes per
// instruction, so staging is cheap next to it: global loads for the next stage are issued before
// the current stage is multiplied and written to the other LDS buffer afterwards.
//
// Even kernel sides with even padding (the generator layers: n = 4, P = 2) take quads that are
// aligned to the OUTPUT instead (template flag AL): rows {2ky, 2ky+1} x cols {2kx, 2kx+1}, all inside
// the even-sized output, where the shifted quads carry an extra row and column of half-empty quads
// (25 instead of 16 quads on a 4x4 map).  Output row 2ky + rr then has row class rr and a window
// starting at input row ky - P/2 + rr (Algorithm 2, Sec. 3.4), so a quad reads a
// (ceil(n/2)+1)^2 window and class (rr, cc) multiplies position (a, b) by tap
// w[rr + 2(a-rr)][cc + 2(b-cc)] where it has one: the same n*n MFMAs per quad tile and channel
// pair, on fewer quads, and a drain without edge cases.
//
// Tiny maps with many channels (the first generator layers: 4x4 and 8x8 maps, 512 and 256 input
// channels) have far fewer 64 x 64 tiles than the chip has compute units.  They take NW = 0: block
// tile 32 channels x 32 quads, all four waves on the SAME tile, each multiplying every fourth K
// pair of a stage; at the end the waves park their accumulators in LDS and add them in wave order
// (bit-reproducible) on their way to memory.  No partial sums leave the compute unit: no
// workspace, no second kernel.  On such layers the weights are the traffic, and a wave is the only
// reader of its K pairs' weights, so they skip LDS: a lane's A operands of one K pair -- all n*n
// taps of its (channel, input channel) -- are n*n consecutive floats in memory, fetched with
// 16-byte loads a stage ahead, straight into the registers the MFMAs read.
//
// Block = 4 waves; tile = 64 channels x (64*NW) quads x 4 classes; wave = 32 channels x 32*NW
// quads (NW = 4, 2 or 1 so that small layers still fill the chip).  The epilogue stores the two
// column classes of a quad as one 8-byte element, classes interleaved in place.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));

constexpr int kRsrcFlags = 0x00020000;      // raw 32-bit buffer, gfx9 family
constexpr unsigned kInvalid = 0xFFFFFF00u;  // byte offset that is out of range for any buffer
constexpr int TM = 64;      // output channels per block
// input channels per K stage: small kernels get longer stages so that the fixed cost of a stage
// (loads, LDS writes, barrier) is spread over enough MFMAs
constexpr int kc_for(int n) { return n <= 3 ? 16 : 8; }
// ... of the small-tile variant (NW = 0), whose waves each take a quarter of a stage's K pairs: long
// stages, so that one stage of arithmetic covers the latency of the next one's loads
constexpr int kc_small(int n) { return n <= 3 ? 64 : 32; }
constexpr int PW = 65;      // floats per (k, tap) weight row in LDS: 64 channels + 1, so that the
                            // staging lanes (consecutive rows, one channel) hit consecutive banks
// activation elements one thread stages per K stage, at most (register arrays of that size)
constexpr int nxl_max_for(int n) { return n <= 3 ? 32 : 24; }
// ... of the small-tile variant: every one of these slots is issued in every stage (a slot without an
// element reads nothing and writes a zero to a spare word), one per multiplication step
constexpr int NXS_SMALL = 8;
constexpr int LDS_LIMIT = 160 * 1024;

struct F32Args {
    GeomBase g;
    int aligned; // 1: quads aligned to the output (even n, even P), 0: shifted quads
    int KHq, KWq; // quad rows / columns
    int cb_major; // tile order: 1 = consecutive blocks share the channel block (big weights)
    int Q;       // total quads = B * KHq * KWq
    int EH;      // input rows one image's quad rows touch = KH + ceil(n/2) - 1
    int ROWS;    // input rows an activation stage holds
    int LWX;     // floats per staged row: left halo + W + right halo
    int XP;      // floats per k plane of the activation stage
    int SH;      // LDS column of input column 0 = floor(P/2)
    int nxl;     // activation elements per thread and stage
    int nco, nqt;
    int xs_stage_bytes;
    int ksplit;  // the K loop of a tile is cut into this many slices, one block each (see below)
    int kstages; // stages per slice
    FastDiv dKHW, dKW, dEH, dRW, dW;
};

// Narrow tiles (NW < 4) keep few accumulators, so two blocks may share a compute unit and cover
// each other's staging latency; the widest tile needs the whole register file.
// EPI: the fused epilogue (bias, activation) is compiled into the drain; the plain instance keeps
// the register allocation and schedule of its drain to itself.
// tap of class c = 2*rr + cc (aligned) / 2*r + s (shifted) at window position (pa, pb), or -1
template <int N, bool AL>
constexpr int tap_at(int pa, int pb, int c)
{
    const int r = c >> 1, sc = c & 1;
    const int u = AL ? pa - r : pa, v = AL ? pb - sc : pb;
    if (u < 0 || v < 0 || r + 2 * u >= N || sc + 2 * v >= N) return -1;
    return (r + 2 * u) * N + (sc + 2 * v);
}

// TIn = float, or uint16_t for bf16 operands: they are widened to fp32 on their way into LDS
// (exact) and multiplied on the fp32 matrix pipe -- the path of bf16 layers whose kernel side the
// bf16 kernels do not take (n = 2, 3, 5).
template <int N, int NW, int KC, bool EPI, bool AL, typename TIn>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, NW == 4 ? 1 : 2)))
void ukst_mfma_f32_kernel(const TIn* __restrict__ x, const TIn* __restrict__ w,
                          float* __restrict__ y, F32Args a, Epilogue ep)
{
    constexpr bool B16 = sizeof(TIn) == 2;
    constexpr int ES = (int)sizeof(TIn);
    constexpr int HI = (N + 1) / 2;
    constexpr int NN = N * N;
    constexpr bool SK = NW == 0;                // the four waves split the K pairs of one small tile
    constexpr int NWA = SK ? 1 : NW;            // groups of 32 quads per wave
    constexpr int TMk = SK ? 32 : TM;           // output channels per block
    constexpr int PWk = TMk + 1;                // floats per (k, tap) weight row in LDS
    constexpr int TN = SK ? 32 : 64 * NW;       // quads per block
    constexpr int WS_STAGE = SK ? 0 : NN * KC * PWk * 4; // bytes of one weight stage (NW = 0: none)
    constexpr int NXL_MAX = SK ? NXS_SMALL : nxl_max_for(N);
    constexpr int NWL = (TMk * KC * NN / 4 + 255) / 256;  // 16-byte weight pieces per thread and stage
    static_assert(!SK || AL, "the split-K-in-block tile is built for the output-aligned quads");
    static_assert(!SK || (sizeof(TIn) == 4 && NN % 4 == 0), "NW = 0: fp32 operands, 16-byte tap rows");
    extern __shared__ __align__(16) unsigned char lds[];
    float* const ldsf = reinterpret_cast<float*>(lds);
    // layout: weights stage 0 | weights stage 1 | activations stage 0 | activations stage 1
    constexpr int XS_OFF = 2 * WS_STAGE;

    const GeomBase& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = SK ? 0 : wave & 1;   // which 32-channel half of the block tile
    const int qh = SK ? 0 : wave >> 1;  // which half of the block's quads
    const int kw = SK ? wave : 0;       // which K pairs of a stage (every fourth, starting here)
    const int l32 = lane & 31, gk = lane >> 5;
    const int KHW = a.KHq * a.KWq;

    // Split K: when a layer has too few tiles to fill the chip (small maps, many channels), the
    // input channels of a tile are divided among `ksplit` blocks; slice ks writes its partial
    // sums to the ks-th copy of the output in scratch memory and a second kernel adds the copies
    // in a fixed order.
    const int bid_all = xcd_contiguous(blockIdx.x, gridDim.x);
    const int ks = bid_all % a.ksplit, bid = bid_all / a.ksplit;
    // tile order: blocks of one XCD (consecutive numbers) share what is bigger, the weights of a
    // channel block or the activations of a quad tile
    const int cb = a.cb_major ? bid / a.nqt : bid % a.nco;
    const int qt = a.cb_major ? bid % a.nqt : bid / a.nco;
    const int co0 = cb * TMk;
    const int q0 = qt * TN;
    const int q_last = (q0 + TN - 1 < a.Q ? q0 + TN - 1 : a.Q - 1);
    // quad row rho = b*KH + kk uses input rows e = b*EH + kk + u (u < HI)
    const int bf0 = fdiv(q0, a.dKHW), kf0 = fdiv(q0 - bf0 * KHW, a.dKW);
    const int e_first = bf0 * a.EH + kf0;

    // ---- zero both activation buffers once: halo columns are never written again
    {
        const int nf = 2 * a.xs_stage_bytes / 4;
        for (int i = tid; i < nf; i += 256) ldsf[XS_OFF / 4 + i] = 0.f;
    }

    // ---- activation staging: element e = tid + 256*j -> (k, row, col) of the stage
    unsigned x_goff[NXL_MAX];  // global byte offset (for ci0 = 0), kInvalid for rows that do not exist
    int x_loff[NXL_MAX];       // LDS float index inside an activation stage (padding where there is no element)
#pragma unroll
    for (int j = 0; j < NXL_MAX; ++j) {
        x_goff[j] = kInvalid;
        x_loff[j] = a.XP - 1;  // (the last word of a k plane is padding: never read)
        if (j < a.nxl) {
            const int e = tid + 256 * j;
            const int k = fdiv(e, a.dRW);
            const int rem = e - k * (a.ROWS * g.W);
            const int row = fdiv(rem, a.dW), col = rem - row * g.W;
            if (k < KC) {
                const int er = e_first + row;
                const int b = fdiv(er, a.dEH), ii = er - b * a.EH;
                const int i = ii - (g.P >> 1);  // = k_min - P + ii for the shifted quads
                if (b < g.B && i >= 0 && i < g.H)
                    x_goff[j] = (unsigned)((((b * g.Cin + k) * g.H + i) * g.W + col) * ES);
                x_loff[j] = k * a.XP + row * a.LWX + a.SH + col;
            }
        }
    }
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * ES), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)w, 0, (int)((size_t)g.Cout * g.Cin * NN * ES), kRsrcFlags);
    const unsigned x_cstride = (unsigned)(g.H * g.W * ES);  // bytes between input channels

    // ---- per-lane operand positions
    // A (weights): lane = channel cw*32 + l32, k parity gk
    const int a_base = (gk + 2 * kw) * NN * PWk + cw * 32 + l32;  // + (2*ks*NN + tap) * PWk
    // B (activations): lane = quad q0 + (qh*NW + nt)*32 + l32, k parity gk
    int b_base[NWA];
#pragma unroll
    for (int nt = 0; nt < NWA; ++nt) {
        int q = q0 + (qh * NWA + nt) * 32 + l32;
        if (q > q_last) q = q_last;
        const int b = fdiv(q, a.dKHW);
        const int rem = q - b * KHW;
        const int kk = fdiv(rem, a.dKW), mm = rem - kk * a.KWq;
        const int r = b * a.EH + kk - e_first;
        // window column v of quad column mm is input column mm - floor(P/2) + v in either quad
        // system (shifted: m_min + mm - P + v), i.e. LDS column mm + v
        b_base[nt] = XS_OFF / 4 + (gk + 2 * kw) * a.XP + r * a.LWX + mm;
    }

    f32x16 acc[NWA][2][2];
#pragma unroll
    for (int nt = 0; nt < NWA; ++nt)
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int sc = 0; sc < 2; ++sc)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[nt][r][sc][i] = 0.f;

    u4v wreg[NWL];
    float xreg[NXL_MAX];
    // The staging work of a stage is cut into items: item i < NWL is weight piece e = tid + 256*i
    // (four consecutive floats of channel co = 4e / (KC*NN); the (k, tap) pairs of a channel are
    // contiguous in memory and a stage's chunk of a channel starts on a 16-byte boundary, so lanes
    // read consecutive 16-byte pieces), item NWL + j is activation element j.  Slots without an
    // element read nothing (zeros) and write to padding: no lane-divergent branches.
    constexpr int NITEMS = NWL + NXL_MAX;
    auto load_item = [&](int i, int ci0) {  // (i: a constant once unrolled)
        if (i < NWL) {
            const int e = (tid + 256 * i) * 4;
            const int co = e / (KC * NN), rem = e - co * (KC * NN);
            const unsigned voff = (co < TMk) ? (unsigned)(((co0 + co) * g.Cin * NN + rem) * ES) : kInvalid;
            if constexpr (B16) {  // (kept as loaded: widening here would wait for the load on the spot)
                const u2v t = __builtin_amdgcn_raw_buffer_load_b64(rs_w, voff, (unsigned)(ci0 * NN * ES), 0);
                wreg[i] = u4v{t.x, t.y, 0u, 0u};
            } else {
                wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, voff, (unsigned)(ci0 * NN * ES), 0);
            }
        } else if (i - NWL < a.nxl) {
            const int j = i - NWL;
            if constexpr (B16)
                xreg[j] = __uint_as_float((unsigned)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(
                    rs_x, x_goff[j], (unsigned)ci0 * x_cstride, 0));
            else
                xreg[j] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, x_goff[j], (unsigned)ci0 * x_cstride, 0));
        }
    };
    auto store_item = [&](int i, int buf) {
        if (i < NWL) {
            const int e = (tid + 256 * i) * 4;
            const int co = e / (KC * NN), rem = e - co * (KC * NN);  // rem = k*NN + tap, multiple of 4
            // (a piece past the last channel lands in the padding column of its rows)
            float* dst = ldsf + buf * (WS_STAGE / 4) + rem * PWk + (co < TMk ? co : TMk);
            u4v v = wreg[i];
            if constexpr (B16) v = u4v{v.x << 16, v.x & 0xFFFF0000u, v.y << 16, v.y & 0xFFFF0000u};
#pragma unroll
            for (int t = 0; t < 4; ++t) dst[t * PWk] = __uint_as_float(v[t]);
        } else if (i - NWL < a.nxl) {
            const int j = i - NWL;
            float v = xreg[j];
            if constexpr (B16) v = __uint_as_float(__float_as_uint(v) << 16);
            ldsf[XS_OFF / 4 + buf * (a.xs_stage_bytes / 4) + x_loff[j]] = v;
        }
    };
    // One step = one window position (u, v) at one K pair.  The fragments of step t+1 are
    // requested before the MFMAs of step t are issued, so LDS latency hides under the matrix pipe.
    // A wave is alone on its SIMD: whatever is not an MFMA and does not sit between two MFMAs is
    // time the matrix pipe idles.  So the staging items are dealt out over the steps: an item's
    // registers (fetched a stage ago, for the NEXT stage) go to the other LDS buffer and are
    // refilled at once for the stage after next.
    constexpr int NP1 = AL ? HI + 1 : HI;  // window positions per axis
    // K pairs of a stage this wave multiplies: all KC/2, or (NW = 0) every fourth one
    constexpr int KSTEP = SK ? 4 : 1;
    constexpr int NP = NP1 * NP1, NSTEP = (KC / 2 / KSTEP) * NP;
    constexpr int IPS = (NITEMS + NSTEP - 1) / NSTEP;  // items per step
    auto compute = [&](int buf, int sidx, int last) {
        // (the last two stages fetch the last stage again rather than branch: in bounds, unused)
        const int ci_next = (sidx + 2 < last ? sidx + 2 : last - 1) * KC;
        const float* ws = ldsf + buf * (WS_STAGE / 4) + a_base;
        const int xb = buf * (a.xs_stage_bytes / 4);
        auto load_step = [&](int t, float (&bfr)[NWA], float (&afr)[4]) {
            const int ks = (t / NP) * KSTEP, p = t % NP, pa = p / NP1, pb = p % NP1;
            const int xo = xb + 2 * ks * a.XP + pa * a.LWX + pb;
#pragma unroll
            for (int nt = 0; nt < NWA; ++nt) bfr[nt] = ldsf[b_base[nt] + xo];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int tap = tap_at<N, AL>(pa, pb, c);
                if (tap < 0) continue;  // class has no tap here
                afr[c] = ws[(2 * ks * NN + tap) * PWk];
            }
        };
        float bfr[2][NWA], afr[2][4];
        load_step(0, bfr[0], afr[0]);
#pragma unroll
        for (int t = 0; t < NSTEP; ++t) {
            const int p = t % NP, pa = p / NP1, pb = p % NP1;
            if (t + 1 < NSTEP) load_step(t + 1, bfr[(t + 1) & 1], afr[(t + 1) & 1]);
#pragma unroll
            for (int r = 0; r < IPS; ++r) {
                const int i = t * IPS + r;
                if (i < NITEMS) {
                    store_item(i, buf ^ 1);
                    load_item(i, ci_next);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (tap_at<N, AL>(pa, pb, c) < 0) continue;
#pragma unroll
                for (int nt = 0; nt < NWA; ++nt)
                    acc[nt][c >> 1][c & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                        afr[t & 1][c], bfr[t & 1][nt], acc[nt][c >> 1][c & 1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int s0 = ks * a.kstages;              // this block's slice of the K stages
    const int stages = s0 + a.kstages;          // (ksplit * kstages covers Cin exactly)
    if constexpr (SK) {
        // One wave per SIMD: whatever is not an MFMA and does not sit between two MFMAs is time
        // the matrix pipe idles.  So the whole stage pipeline is dealt out over the steps of the
        // multiplication: step t < NXS hands activation element t of the NEXT stage (fetched a
        // stage ago) to the other LDS buffer and requests its successor; the last step of a K pair
        // requests that pair's weights of the stage after next into the registers just freed.
        constexpr int PPS = KC / 8;   // K pairs per stage and wave
        constexpr int NS = PPS * NP;  // steps per stage
        static_assert(NS >= NXS_SMALL, "one activation element per step");
        float areg[2][PPS][NN];
        float xs[NXS_SMALL];
        const unsigned a_voff = (co0 + l32 < g.Cout) ? (unsigned)((((co0 + l32) * g.Cin + gk) * NN) * 4) : kInvalid;
        auto load_pair = [&](auto c_tag, int jj, int stage) {  // (jj: a constant once unrolled)
            constexpr int C = decltype(c_tag)::value;
            const unsigned soff = (unsigned)(((stage * KC + 2 * (kw + 4 * jj)) * NN) * 4);
#pragma unroll
            for (int q4 = 0; q4 < NN / 4; ++q4) {
                const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rs_w, a_voff + 16u * q4, soff, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) areg[C][jj][4 * q4 + e] = __uint_as_float(t[e]);
            }
        };
        auto load_x = [&](int j, int stage) {
            xs[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                  rs_x, x_goff[j], (unsigned)(stage * KC) * x_cstride, 0));
        };
        auto store_x = [&](int j, int buf) {
            ldsf[XS_OFF / 4 + buf * (a.xs_stage_bytes / 4) + x_loff[j]] = xs[j];
        };
        auto stage_sk = [&](int buf, auto c_tag, int sidx) {
            constexpr int C = decltype(c_tag)::value;
            const bool more1 = sidx + 1 < stages, more2 = sidx + 2 < stages;  // uniform
            const int xb = buf * (a.xs_stage_bytes / 4);
            auto b_at = [&](int t) {
                const int jj = t / NP, p = t % NP;
                return ldsf[b_base[0] + xb + 8 * jj * a.XP + (p / NP1) * a.LWX + (p % NP1)];
            };
            float bfr[3];
            bfr[0] = b_at(0);
            bfr[1] = b_at(1);
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                const int jj = t / NP, p = t % NP, pa = p / NP1, pb = p % NP1;
                if (t + 2 < NS) bfr[(t + 2) % 3] = b_at(t + 2);
                if (t < NXS_SMALL) {
                    if (more1) store_x(t, buf ^ 1);
                    if (more2) load_x(t, sidx + 2);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int tap = tap_at<N, AL>(pa, pb, c);
                    if (tap < 0) continue;
                    acc[0][c >> 1][c & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                        areg[C][jj][tap], bfr[t % 3], acc[0][c >> 1][c & 1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                // this pair's registers are free: its weights of the stage after next
                if (p == NP - 1 && more2) load_pair(c_tag, jj, sidx + 2);
            }
            __syncthreads();
        };
        const std::integral_constant<int, 0> i0;
        const std::integral_constant<int, 1> i1;
#pragma unroll
        for (int jj = 0; jj < PPS; ++jj) load_pair(i0, jj, 0);
#pragma unroll
        for (int j = 0; j < NXS_SMALL; ++j) load_x(j, 0);
        __syncthreads();  // zero fill done before the first activation writes
#pragma unroll
        for (int j = 0; j < NXS_SMALL; ++j) store_x(j, 0);
#pragma unroll
        for (int j = 0; j < NXS_SMALL; ++j) load_x(j, 1);  // (the stage count is even: stage 1 exists)
#pragma unroll
        for (int jj = 0; jj < PPS; ++jj) load_pair(i1, jj, 1);
        __syncthreads();
        for (int s = 0; s < stages; s += 2) {
            stage_sk(0, i0, s);
            stage_sk(1, i1, s + 1);
        }
    }
    if constexpr (!SK) {
#pragma unroll
        for (int i = 0; i < NITEMS; ++i) load_item(i, s0 * KC);
        __syncthreads();  // zero fill done before the first activation writes
#pragma unroll
        for (int i = 0; i < NITEMS; ++i) store_item(i, 0);
#pragma unroll
        for (int i = 0; i < NITEMS; ++i) load_item(i, (s0 + 1 < stages ? s0 + 1 : s0) * KC);
        __syncthreads();
        int buf = 0;
        for (int s = s0; s < stages; ++s) {
            compute(buf, s, stages);
            __syncthreads();
            buf ^= 1;
        }
    }

    // ---- epilogue: accumulator register i of a tile holds channel 8*(i/4) + 4*gk + (i%4) of the
    // wave's 32, for the lane's quad; column classes s = 1, 0 are neighbours in memory
    const size_t ybytes = (size_t)g.B * g.Cout * g.OH * g.OW * 4;
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((unsigned char*)y + (size_t)ks * ybytes), 0, (int)ybytes, kRsrcFlags);
    const unsigned plane = (unsigned)(g.OH * g.OW * 4);
    // Cout is a multiple of 8, so a group of 8 channels (4 per k parity) exists or not as a whole
    const int co_w = co0 + cw * 32;  // first channel of this wave
    // fused epilogue (whole sums only: with a split K loop the slice sum applies it instead)
    float bias_i[16];
    if constexpr (EPI) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ch = co_w + 8 * (i / 4) + 4 * gk + (i % 4);
            bias_i[i] = (ep.bias && ch < g.Cout) ? ep.bias[ch] : 0.f;
        }
    }
    if constexpr (SK) {
        // The four waves hold partial sums of the same 32 x 32 x 4 tile.  Park them in LDS as
        // [wave][row class][column class][register][lane]; wave w then finishes output row class
        // w & 1 for registers 8*(w/2) .. +7, adding the four copies in wave order.
        __syncthreads();  // every wave is done with the stage buffers
#pragma unroll
        for (int rr = 0; rr < 2; ++rr)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    ldsf[(((wave * 2 + rr) * 2 + cc) * 16 + i) * 64 + lane] = acc[0][rr][cc][i];
        __syncthreads();
        const int rr = wave & 1, ih = wave >> 1;
        const int q = q0 + l32;
        const bool qv = q <= q_last;
        const int qq = qv ? q : q_last;
        const int b = fdiv(qq, a.dKHW);
        const int rem = qq - b * KHW;
        const int kk = fdiv(rem, a.dKW), mm = rem - kk * a.KWq;
        const unsigned off = qv ? (unsigned)((((b * g.Cout + co0 + 4 * gk) * g.OH + 2 * kk + rr) * g.OW + 2 * mm) * 4)
                                : kInvalid;
        auto finish = [&](auto act_tag) {
            constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
            for (int ii = 0; ii < 8; ++ii) {
                const int i = 8 * ih + ii;
                if (co0 + 8 * (i / 4) >= g.Cout) continue;  // uniform: ragged last channel block
                float v0 = 0.f, v1 = 0.f;
#pragma unroll
                for (int wv = 0; wv < 4; ++wv) {
                    v0 += ldsf[(((wv * 2 + rr) * 2 + 0) * 16 + i) * 64 + lane];
                    v1 += ldsf[(((wv * 2 + rr) * 2 + 1) * 16 + i) * 64 + lane];
                }
                if constexpr (ACT >= 0) {
                    const int ch = co0 + 8 * (i / 4) + 4 * gk + (i % 4);
                    const float bv = (ep.bias && ch < g.Cout) ? ep.bias[ch] : 0.f;
                    v0 = epilogue_t<ACT>(v0, bv);
                    v1 = epilogue_t<ACT>(v1, bv);
                }
                u2v d;
                d.x = __float_as_uint(v0);
                d.y = __float_as_uint(v1);
                __builtin_amdgcn_raw_buffer_store_b64(d, rs_y, off, (unsigned)(8 * (i / 4) + (i % 4)) * plane, 0);
            }
        };
        if constexpr (EPI) with_activation(ep.act, finish);
        else finish(std::integral_constant<int, -1>{});
        return;
    }
    auto drain = [&](auto act_tag) {
        constexpr int ACT = decltype(act_tag)::value;  // -1: no epilogue at all
#pragma unroll
        for (int nt = 0; nt < NWA; ++nt) {
            const int q = q0 + (qh * NWA + nt) * 32 + l32;
            const bool qv = q <= q_last;
            const int qq = qv ? q : q_last;
            const int b = fdiv(qq, a.dKHW);
            const int rem = qq - b * KHW;
            const int kk = fdiv(rem, a.dKW), mm = rem - kk * a.KWq;
            if constexpr (AL) {
                // quad (kk, mm) = output rows 2kk, 2kk+1 x columns 2mm, 2mm+1, all inside the
                // output: one 8-byte store per row and channel, no edges
                const unsigned y_off = qv ? (unsigned)((((b * g.Cout + co_w + 4 * gk) * g.OH + 2 * kk) * g.OW +
                                                       2 * mm) * 4) : kInvalid;
#pragma unroll
                for (int rr = 0; rr < 2; ++rr) {
                    const unsigned off = qv ? y_off + (unsigned)(rr * g.OW * 4) : kInvalid;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        if (co_w + 8 * (i / 4) >= g.Cout) continue;  // uniform: ragged last channel block
                        const unsigned soff = (unsigned)(8 * (i / 4) + (i % 4)) * plane;
                        float v0 = acc[nt][rr][0][i], v1 = acc[nt][rr][1][i];
                        if constexpr (ACT >= 0) {
                            v0 = epilogue_t<ACT>(v0, bias_i[i]);
                            v1 = epilogue_t<ACT>(v1, bias_i[i]);
                        }
                        u2v d;
                        d.x = __float_as_uint(v0);
                        d.y = __float_as_uint(v1);
                        __builtin_amdgcn_raw_buffer_store_b64(d, rs_y, off, soff, 0);
                    }
                }
                continue;
            }
            const int k = g.k_min + kk, m = g.m_min + mm;
            const int oy1 = 2 * k - 1 - g.P, ox1 = 2 * m - 1 - g.P;  // row / column of class 1
            const bool vcol1 = ox1 >= 0 && ox1 < g.OW, vcol0 = ox1 + 1 < g.OW;
            // byte offset of (channel co_w + 4*gk, row oy1, column ox1); unsigned wrap-around keeps
            // the arithmetic right when oy1 or ox1 is -1 and only the other class exists
            const unsigned y_off =
                (unsigned)((((b * g.Cout + co_w + 4 * gk) * g.OH + oy1) * g.OW + ox1) * 4);
#pragma unroll
            for (int r = 1; r >= 0; --r) {
                const bool vrow = qv && (r ? (oy1 >= 0 && oy1 < g.OH) : (oy1 + 1 < g.OH));
                const unsigned base = y_off + (r ? 0u : (unsigned)(g.OW * 4));
                // interior quads store both column classes as one 8-byte element; a quad on the left
                // or right edge of an odd-sized output has one class only and stores 4 bytes
                const unsigned off_pair = (vrow && vcol1 && vcol0) ? base : kInvalid;
                const bool only1 = vrow && vcol1 && !vcol0, only0 = vrow && !vcol1 && vcol0;
                const unsigned off_edge = only1 ? base : (only0 ? base + 4u : kInvalid);
                const bool any_edge = __builtin_amdgcn_ballot_w64(only1 || only0) != 0;  // uniform
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (co_w + 8 * (i / 4) >= g.Cout) continue;  // uniform: ragged last channel block
                    const unsigned soff = (unsigned)(8 * (i / 4) + (i % 4)) * plane;
                    float v1 = acc[nt][r][1][i], v0 = acc[nt][r][0][i];  // by value, then bits
                    if constexpr (ACT >= 0) {
                        v1 = epilogue_t<ACT>(v1, bias_i[i]);
                        v0 = epilogue_t<ACT>(v0, bias_i[i]);
                    }
                    u2v d;
                    d.x = __float_as_uint(v1);
                    d.y = __float_as_uint(v0);
                    __builtin_amdgcn_raw_buffer_store_b64(d, rs_y, off_pair, soff, 0);
                    if (any_edge)
                        __builtin_amdgcn_raw_buffer_store_b32(only1 ? d.x : d.y, rs_y, off_edge, soff, 0);
                }
            }
        }
    };
    if constexpr (EPI) with_activation(ep.act, drain);  // one uniform branch per block
    else drain(std::integral_constant<int, -1>{});
}

// y[i] = part[0][i] + part[1][i] + ... in this order, four floats per thread; the fused epilogue
// (bias of the element's channel, activation) is applied to the finished sums
__global__ __launch_bounds__(256) void ukst_sum_slices_kernel(const float4* __restrict__ part,
                                                              float4* __restrict__ y, int n4,
                                                              int ksplit, const float* __restrict__ bias,
                                                              int act, unsigned plane, unsigned cout)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float4 s = part[i];
    for (int k = 1; k < ksplit; ++k) {
        const float4 p = part[(size_t)k * n4 + i];
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    if (bias != nullptr || act != 0) {  // uniform
        float v[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned idx = 4u * (unsigned)i + e;  // element of y[B][Cout][plane]
            const float bv = bias ? bias[(idx / plane) % cout] : 0.f;
            v[e] = epilogue(v[e], bv, act);
        }
        s = make_float4(v[0], v[1], v[2], v[3]);
    }
    y[i] = s;
}

template <int NW>
bool make_args(const Geom& g, F32Args& a, int es = 4)
{
    constexpr int TN = NW == 0 ? 32 : 64 * NW;
    constexpr int TMk = NW == 0 ? 32 : TM, PWk = TMk + 1;
    const int KC = NW == 0 ? kc_small(g.n) : kc_for(g.n);
    if (g.n < 2 || g.n > 5) return false;
    if (g.Cin % KC != 0) return false;  // a stage never straddles the channel count
    if (g.Cout % 8 != 0) return false;  // channel groups of the accumulator layout stay whole
    const size_t xbytes = (size_t)g.B * g.Cin * g.H * g.W * es;
    const size_t wbytes = (size_t)g.Cout * g.Cin * g.n * g.n * es;
    const size_t ybytes = (size_t)g.B * g.Cout * g.OH * g.OW * 4;
    const size_t lim = 0x7FFFFFF0u;  // single buffer descriptors, 32-bit byte offsets
    if (xbytes > lim || wbytes > lim || ybytes > lim) return false;
    const int HI = (g.n + 1) / 2;
    a.g = g;
    // even kernel side and even padding: quads aligned to the (even-sized) output
    a.aligned = (g.n % 2 == 0 && g.P % 2 == 0) ? 1 : 0;
    // the small-tile variant: aligned quads, fp32 operands, an even number of stages (its A operands
    // come from memory a stage at a time into one of two register sets)
    if (NW == 0 && (!a.aligned || es != 4 || (g.Cin / KC) % 2 != 0)) return false;
    a.KHq = a.aligned ? g.OH / 2 : g.KH;
    a.KWq = a.aligned ? g.OW / 2 : g.KW;
    const int wrows = a.aligned ? HI + 1 : HI;  // window rows / columns of a quad
    const long long khw = (long long)a.KHq * a.KWq;
    const long long Q = (long long)g.B * khw;
    if (Q > 0x3FFFFFFFLL) return false;
    a.Q = (int)Q;
    a.EH = a.KHq + wrows - 1;
    // TN consecutive flattened quads touch at most this many quad rows / images (exactly TN/KWq
    // rows / one image where tiles start on row / image boundaries)
    const int nrho = (TN % a.KWq == 0) ? TN / a.KWq : (TN - 2) / a.KWq + 2;
    const int nimg = (khw % TN == 0) ? 1 : (TN % khw == 0) ? (int)(TN / khw) : (int)((TN - 2) / khw) + 2;
    a.ROWS = nrho + (wrows - 1) * nimg;
    a.SH = g.P >> 1;
    a.LWX = a.SH + g.W + HI;
    const int need = a.KWq + wrows - 1;  // largest LDS column read: KWq-1 + wrows-1
    if (a.LWX < need + 1) a.LWX = need + 1;
    int xp = a.ROWS * a.LWX;
    xp = ((xp + 63) / 64) * 64 + 32;  // k planes 32 banks apart: the two k parities do not collide
    a.XP = xp;
    a.xs_stage_bytes = KC * xp * 4;
    const long long elems = (long long)KC * a.ROWS * g.W;
    a.nxl = (int)((elems + 255) / 256);
    if (a.nxl > (NW == 0 ? NXS_SMALL : nxl_max_for(g.n))) return false;
    const int ws_stage = NW == 0 ? 0 : g.n * g.n * KC * PWk * 4;
    if (2 * (ws_stage + a.xs_stage_bytes) > LDS_LIMIT) return false;
    a.nco = (g.Cout + TMk - 1) / TMk;
    a.nqt = (int)((Q + TN - 1) / TN);
    if ((long long)a.nco * a.nqt > 0x3FFFFFFFLL) return false;
    a.cb_major = wbytes > xbytes ? 1 : 0;
    a.dKHW = make_fastdiv((unsigned)khw);
    a.dKW = make_fastdiv((unsigned)a.KWq);
    a.dEH = make_fastdiv((unsigned)a.EH);
    a.dRW = make_fastdiv((unsigned)(a.ROWS * g.W));
    a.dW = make_fastdiv((unsigned)g.W);
    // K slices: only for layers with fewer tiles than compute units.  Two blocks share a compute
    // unit, so about 512 blocks fill the chip once: take the power of two that brings the block
    // count closest to that (in ratio), as long as it divides the stage count, leaves at least
    // two stages per slice and the outputs are 16-byte sized (the slice sum moves such pieces).
    a.ksplit = 1;
    const int stages = g.Cin / KC;
    const long long tiles = (long long)a.nco * a.nqt;
    if (NW != 0 && ybytes % 16 == 0 && tiles < 256) {
        auto distance = [&](int ks) {
            const double r = (double)(tiles * ks) / 512.0;
            return r >= 1.0 ? r : 1.0 / r;
        };
        for (int ks = 2; ks <= 8; ks *= 2) {
            if (stages % ks != 0 || stages / ks < 2 || (size_t)ks * ybytes > ((size_t)1 << 30)) break;
            if (distance(ks) < distance(a.ksplit)) a.ksplit = ks;
        }
    }
    a.kstages = stages / a.ksplit;
    return true;
}

template <int N, int NW, bool AL, typename TIn>
hipError_t launch_a(const F32Args& a, const Epilogue& ep, const TIn* x, const TIn* w, float* y,
                    void* part, hipStream_t stream)
{
    constexpr int KC = NW == 0 ? kc_small(N) : kc_for(N);
    constexpr int PWk = (NW == 0 ? 32 : TM) + 1;
    size_t lds = 2 * (size_t)((NW == 0 ? 0 : N * N * KC * PWk * 4) + a.xs_stage_bytes);
    if (NW == 0 && lds < 65536) lds = 65536;  // the four waves' accumulators meet in LDS at the end
    // more than 64 KiB of dynamic LDS has to be allowed per device (a property of the loaded
    // kernel, not library state); cheap enough to repeat on every call
    // the epilogue belongs to whole sums: with a split K loop the slice sum applies it
    const bool epi = a.ksplit == 1 && has_epilogue(ep);
    typedef void (*kernel_t)(const TIn*, const TIn*, float*, F32Args, Epilogue);
    const kernel_t kfn = epi ? ukst_mfma_f32_kernel<N, NW, KC, true, AL, TIn>
                             : ukst_mfma_f32_kernel<N, NW, KC, false, AL, TIn>;
    hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const unsigned nblocks = (unsigned)(a.nco * a.nqt * a.ksplit);
    if (a.ksplit == 1) {
        hipLaunchKernelGGL(kfn, dim3(nblocks), dim3(256), lds, stream, x, w, y, a, ep);
        return hipGetLastError();
    }
    // partial outputs live in the caller's workspace for the duration of this call
    const GeomBase& g = a.g;
    const size_t ybytes = (size_t)g.B * g.Cout * g.OH * g.OW * 4;
    hipLaunchKernelGGL(kfn, dim3(nblocks), dim3(256), lds, stream, x, w, (float*)part, a, ep);
    const int n4 = (int)(ybytes / 16);
    hipLaunchKernelGGL(ukst_sum_slices_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                       stream, (const float4*)part, (float4*)y, n4, a.ksplit, ep.bias, ep.act,
                       (unsigned)(g.OH * g.OW), (unsigned)g.Cout);
    return hipGetLastError();
}

template <int N, int NW, typename TIn>
hipError_t launch_t(const F32Args& a, const Epilogue& ep, const TIn* x, const TIn* w, float* y,
                    void* part, hipStream_t stream)
{
    if constexpr (N % 2 == 0) {
        if (a.aligned) return launch_a<N, NW, true, TIn>(a, ep, x, w, y, part, stream);
    }
    if constexpr (NW == 0) return hipErrorInvalidValue;  // only the aligned quads have that tile
    else return launch_a<N, NW, false, TIn>(a, ep, x, w, y, part, stream);
}

template <int NW, typename TIn>
hipError_t launch_n(const F32Args& a, const Epilogue& ep, const TIn* x, const TIn* w, float* y,
                    void* part, hipStream_t st)
{
    switch (a.g.n) {
        case 2: return launch_t<2, NW, TIn>(a, ep, x, w, y, part, st);
        case 3: return launch_t<3, NW, TIn>(a, ep, x, w, y, part, st);
        case 4: return launch_t<4, NW, TIn>(a, ep, x, w, y, part, st);
        case 5: return launch_t<5, NW, TIn>(a, ep, x, w, y, part, st);
        default: return hipErrorInvalidValue;
    }
}

// Quads per wave: as wide as possible while the grid still covers the chip about twice.
int pick_nw(const Geom& g, F32Args& a, int es)
{
    const long long want = 512;
    F32Args t;
    int best = 0;
    for (int nw : {4, 2, 1}) {
        bool ok = nw == 4 ? make_args<4>(g, t, es) : nw == 2 ? make_args<2>(g, t, es) : make_args<1>(g, t, es);
        if (!ok) continue;
        best = nw;
        a = t;
        if ((long long)t.nco * t.nqt >= want) break;
    }
    // layers that cannot give every compute unit a 64 x 64 tile: 32 x 32 tiles whose K loop the
    // four waves of a block share (no workspace, no slice sum)
    if (best != 0 && (long long)a.nco * a.nqt < 256 && make_args<0>(g, t, es)) {
        a = t;
        return -1;
    }
    return best;
}

}  // namespace

// dtype 0: fp32 operands; 1: bf16 operands (fp32 output); a bf16 output is not produced here
bool mfma_f32_supported(const Geom& g, int dtype)
{
    F32Args a;
    return (dtype == 0 || dtype == 1) && pick_nw(g, a, dtype == 0 ? 4 : 2) != 0;  // (-1: the split-K-in-block tile)
}

hipError_t launch_mfma_f32(const Geom& g, const void* x, const void* w, float* y, int dtype, Workspace& ws,
                           hipStream_t stream)
{
    F32Args a;
    const int nw = pick_nw(g, a, dtype == 0 ? 4 : 2);
    const size_t ybytes = (size_t)g.B * g.Cout * g.OH * g.OW * 4;
    const size_t need = a.ksplit > 1 ? ybytes * (size_t)a.ksplit : 0;
    if (ws.query) {
        ws.need = need;
        return hipSuccess;
    }
    // without a workspace, and for outputs the slice sum cannot move in 16-byte pieces, the K loop
    // stays in one block per tile
    if (a.ksplit > 1 && (ws.ptr == nullptr || ((uintptr_t)y & 15) != 0)) {
        a.kstages *= a.ksplit;
        a.ksplit = 1;
    }
    if (a.ksplit > 1 && ws.bytes < need) return kWorkspaceTooSmall;
    if (dtype == 1) {
        const uint16_t* xh = (const uint16_t*)x;
        const uint16_t* wh = (const uint16_t*)w;
        switch (nw) {
            case 4: return launch_n<4, uint16_t>(a, g.ep, xh, wh, y, ws.ptr, stream);
            case 2: return launch_n<2, uint16_t>(a, g.ep, xh, wh, y, ws.ptr, stream);
            case 1: return launch_n<1, uint16_t>(a, g.ep, xh, wh, y, ws.ptr, stream);
            default: return hipErrorInvalidValue;
        }
    }
    const float* xf = (const float*)x;
    const float* wf = (const float*)w;
    switch (nw) {
        case 4: return launch_n<4, float>(a, g.ep, xf, wf, y, ws.ptr, stream);
        case 2: return launch_n<2, float>(a, g.ep, xf, wf, y, ws.ptr, stream);
        case 1: return launch_n<1, float>(a, g.ep, xf, wf, y, ws.ptr, stream);
        case -1: return launch_n<0, float>(a, g.ep, xf, wf, y, ws.ptr, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ukst
