// bf16 MFMA path for even padding (n = 4): the parity-class implicit GEMM of ukst_mfma.hip on quads
// that are aligned to the OUTPUT.
//
// A quad here is the 2x2 group of output pixels rows {2ky, 2ky+1} x cols {2kx, 2kx+1}.  With n = 4
// the output size 2H+2P-4 is even, so every quad lies inside the output: there are no edge quads,
// no store predicates and no matrix work on pixels that do not exist (the shifted quads of
// ukst_mfma.hip have one extra row and column of half-empty quads when P is even: 13 % more
// MFMAs on a 16x16 map).  Output row 2ky + rr has row class r = rr (P even, Sec. 3.4) and its
// window starts at input row ky - P/2 + rr (Algorithm 2); likewise for columns.  The four classes
// of a quad therefore read a 3x3 input window: class (rr, cc) multiplies window position (a, b),
// a - rr and b - cc in {0, 1}, by tap w[2a - rr][2b - cc] (Eqs. 1-4).  One B fragment (activations
// at window position (a, b), 16 channels) feeds 1, 2 or 4 classes: 16 MFMA groups per K step as
// before, 9 window positions instead of 4 -- but column-neighbouring quads share window columns,
// and a lane holds two such quads, so a K step reads 24 B fragments for its 4 accumulator tiles.
//
// Lanes of two neighbouring accumulator tiles hold column-neighbouring quads, so the drain writes
// four consecutive output floats (both column classes of two quads) as one aligned 16-byte store:
// a quarter of the store instructions of the 8-byte class-pair drain.  Tile counts divide evenly
// (256 quads per tile, maps with W % 8 == 0), which removes the ragged last round of the
// persistent blocks.
//
// Block = 4 waves; block tile = 64 output channels x 256 quads x 4 classes; wave tile = 32
// channels x 128 quads x 4 classes = 16 accumulator tiles of 32x32.  K advances 16 input channels
// per stage, stages double-buffered in LDS; both operands are transposed in registers (8x8 b16
// transposes out of v_perm_b32) on their way into LDS; loads are requested two stages ahead.
#include "ukst_internal.h"

namespace ukst {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef const float __attribute__((address_space(4)))* bias_cptr;

constexpr int kRsrcFlags = 0x00020000;      // raw 32-bit buffer, gfx9 family
constexpr unsigned kInvalid = 0xFFFFFF00u;  // byte offset that is out of range for any buffer

constexpr int TM = 64;    // output channels per block
constexpr int TN = 256;   // quads per block
constexpr int KC = 16;    // input channels per stage (one MFMA K step)
constexpr int W_PLANE = (TM + 1) * 16;     // bytes of one tap plane of a k-half (64 channels + 1 pad slot)
constexpr int W_HALF = 16 * W_PLANE + 64;  // bytes of one k-half (16 tap planes), skewed by 4 slots
constexpr int WS_STAGE = 2 * W_HALF;       // [k-half][tap][channel][8 ci]
constexpr int XS_STAGE_MAX = 48384;        // bytes reserved per activation stage buffer
constexpr int XS_OFF = 2 * WS_STAGE;       // weights stage 0 | weights stage 1 | activations 0 | 1

struct AArgs {
    GeomBase g;
    int KHa, KWa;  // quad rows / columns = OH/2, OW/2
    int HP;        // P/2: the reduced padding of Sec. 3.4
    int Q;         // total quads = B * KHa * KWa
    int EH;        // input rows one image's quad rows touch = KHa + 2
    int ROWS;      // input rows an activation stage buffer holds
    int HS;        // 16-byte slots per column-parity region of a staged row
    int LWS;       // slots per staged row = 2 * HS
    int OFFS;      // staged column of input column 0 (multiple of 8, >= P/2)
    int C8;        // 8-column groups per input row
    int nco, nqt, ntiles, cb_major;
    FastDiv dKHW, dKW, dEH, dC8, dROWS, dNCO, dNQT;
};

// 8x8 transpose of 16-bit elements held as 8 rows of 4 dwords: row k of the result collects
// element k of every input row.
__device__ __forceinline__ u4v transposed_row(const u4v (&in)[8], int k)
{
    u4v t;
    const int q = k >> 1;
    const unsigned sel = (k & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
    for (int pp = 0; pp < 4; ++pp) t[pp] = __builtin_amdgcn_perm(in[2 * pp + 1][q], in[2 * pp][q], sel);
    return t;
}

// The 16 MFMA groups of a K step, ordered by window position (a, b) so that a B fragment is
// fetched once: group = window position x one class (rr, cc) that has a tap there.
struct Grp { int a, b, rr, cc; };
constexpr Grp kGrp[16] = {{0, 0, 0, 0}, {0, 1, 0, 0}, {0, 1, 0, 1}, {0, 2, 0, 1},
                          {1, 0, 0, 0}, {1, 0, 1, 0}, {1, 1, 0, 0}, {1, 1, 0, 1},
                          {1, 1, 1, 0}, {1, 1, 1, 1}, {1, 2, 0, 1}, {1, 2, 1, 1},
                          {2, 0, 1, 0}, {2, 1, 1, 0}, {2, 1, 1, 1}, {2, 2, 1, 1}};
constexpr int grp_tap(int g) { return (2 * kGrp[g].a - kGrp[g].rr) * 4 + (2 * kGrp[g].b - kGrp[g].cc); }
// EPI: the fused epilogue (bias, activation) is compiled into the drain.  OUT16: y is bf16, each
// sum rounded once (to nearest even) at the store.
template <bool EPI, bool OUT16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void ukst_mfma_bf16_aligned_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                   void* __restrict__ y, AArgs a, Epilogue ep)
{
    constexpr int NN = 16;
    extern __shared__ __align__(16) unsigned char lds[];

    const GeomBase& g = a.g;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cw = wave & 1;   // which 32-channel half of the block tile
    const int qh = wave >> 1;  // which 128-quad half of the block tile
    const int l32 = lane & 31, gk = lane >> 5;
    const int KHW = a.KHa * a.KWa;
    const int G = gridDim.x;

    // Tile walked in round rho by this block.  Blocks are spread over the 8 XCDs round-robin, so
    // within a round the blocks of one XCD get consecutive tile numbers: the tiles that share
    // weights or activations meet in the same L2 at the same time.
    const int xcd_rank = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);  // G is a multiple of 8
    auto tile_of = [&](int rho, int& cb, int& qt) -> bool {
        const int t = rho * G + xcd_rank;
        if (t >= a.ntiles) return false;
        // (both orders through the same assignments: a store to "cb or qt" picked by the flag
        // would put the two in scratch memory, and every later read behind all loads in flight)
        const int major = a.cb_major ? fdiv(t, a.dNQT) : fdiv(t, a.dNCO);
        const int minor = t - major * (a.cb_major ? a.nqt : a.nco);
        cb = a.cb_major ? major : minor;
        qt = a.cb_major ? minor : major;
        return true;
    };

    // ---- zero the activation buffers once: halo columns and pad slots are never written again
    {
        const int n16 = 2 * XS_STAGE_MAX / 16;
        u4v z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < n16; i += 256) *reinterpret_cast<u4v*>(lds + XS_OFF + i * 16) = z;
    }

    // ---- per-thread staging units
    // weights: thread = (channel co_l, k-half g, tap-half h), h fastest; planes skewed so that the
    // 16 lanes of a write phase hit distinct bank groups
    const int w_co = tid >> 2, w_g = (tid >> 1) & 1, w_h = tid & 1;
    const int w_lds = w_g * W_HALF + (8 * w_h) * W_PLANE + w_co * 16;  // + t * W_PLANE
    // activations: thread = (8-column group c8, row r, k-half g), c8 fastest; threads beyond the
    // unit count repeat a unit.  A staged row keeps even and odd columns in two regions (lanes of
    // a fragment read hold every second column), column c in slot (c & 1) * HS + c/2.
    int x_r, x_g, x_c8;
    {
        const int units = a.ROWS * 2 * a.C8;
        const int un = tid % units;
        const int t2 = fdiv(un, a.dC8);
        x_c8 = un - t2 * a.C8;
        x_g = fdiv(t2, a.dROWS);
        x_r = t2 - x_g * a.ROWS;
    }
    const int x_lds0 = XS_OFF + ((x_g * a.ROWS + x_r) * a.LWS + 4 * (x_c8 + (a.OFFS >> 3))) * 16;
    const int x_lds1 = x_lds0 + a.HS * 16;  // odd columns of the group

    // global offsets of this thread's staging units for tile (cb, qt)
    auto staging_offsets = [&](int cb, int qt, unsigned& wv, unsigned& xv) {
        wv = cb * TM + w_co < g.Cout ? (unsigned)(((cb * TM + w_co) * g.Cin + 8 * w_g) * (NN * 2) + w_h * 16)
                                     : kInvalid;  // channels past the last one: zeros
        const int q0 = qt * TN;
        const int bf = fdiv(q0, a.dKHW), kf = fdiv(q0 - bf * KHW, a.dKW);
        const int e = bf * a.EH + kf + x_r;  // input row index over the whole batch
        const int b = fdiv(e, a.dEH), ii = e - b * a.EH;
        const int i = ii - a.HP;
        xv = kInvalid;
        if (b < g.B && i >= 0 && i < g.H)
            xv = (unsigned)((((b * g.Cin + 8 * x_g) * g.H + i) * g.W + 8 * x_c8) * 2);
    };

    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((size_t)g.B * g.Cin * g.H * g.W * 2), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)w, 0, (int)((size_t)g.Cout * g.Cin * NN * 2), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(
        y, 0, (int)((size_t)g.B * g.Cout * g.OH * g.OW * (OUT16 ? 2 : 4)), kRsrcFlags);
    const unsigned x_cstride = (unsigned)(g.H * g.W * 2);  // bytes between input channels
    constexpr unsigned ES = OUT16 ? 2u : 4u;  // bytes per output element
    const unsigned plane = (unsigned)(g.OH * g.OW) * ES;
    const unsigned yrow = (unsigned)g.OW * ES;
    const int xrow_lds = a.LWS * 16;  // bytes between staged rows

    // A (weights): lane = channel cw*32 + l32 of the block tile, k-half gk
    const int a_lds = gk * W_HALF + (cw * 32 + l32) * 16;

    // ---- software pipeline: stage s lives in LDS buffer s&1 and passes through register set s&1
    const int stages = g.Cin / KC;              // real stages per tile
    const int stages_even = (stages + 1) & ~1;  // an odd count is padded with a stage of zeros
    u4v wreg[2][8], xreg[2][8];
    f32x16 acc[4][2][2];
    int b_lds[2][4];  // per pair of accumulator tiles (2h, 2h+1) and column j of their joint window: LDS byte address at window row 0

    auto load_one = [&](int ci0, unsigned wv, unsigned xv, int j, u4v (&wr)[8], u4v (&xr)[8]) {
        if (j < 8)
            wr[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, wv,
                                                          (unsigned)((ci0 + j) * (NN * 2)), 0);
        else
            xr[j - 8] = __builtin_amdgcn_raw_buffer_load_b128(
                rs_x, xv, (unsigned)(ci0 + j - 8) * x_cstride, 0);
    };
    auto store_one = [&](int buf, int j, const u4v (&wr)[8], const u4v (&xr)[8]) {
        if (j < 8)
            *reinterpret_cast<u4v*>(lds + buf * WS_STAGE + w_lds + j * W_PLANE) = transposed_row(wr, j);
        else
            *reinterpret_cast<u4v*>(lds + buf * XS_STAGE_MAX + (((j - 8) & 1) ? x_lds1 : x_lds0) +
                                    ((j - 8) >> 1) * 16) = transposed_row(xr, j - 8);
    };
    auto a_frag = [&](int buf, int grp) {
        return *reinterpret_cast<const bf16x8*>(lds + buf * WS_STAGE + a_lds + grp_tap(grp) * W_PLANE);
    };
    // B fragment: window row a, tile pair h, column j of the pair's joint window
    auto b_frag = [&](int buf, int a_row, int h, int j) {
        return *reinterpret_cast<const bf16x8*>(lds + b_lds[h][j] + a_row * xrow_lds + buf * XS_STAGE_MAX);
    };
    // one K stage; `set` is a literal at every call site so that all indices fold.  (ci_next, wv,
    // xv) describe the stage requested from memory during this one.
    // Tiles 2h and 2h+1 hold column-neighbouring quads, so window column b of the odd tile is window
    // column b + 1 of the even one: a tile pair reads 4 distinct columns per window row instead of
    // 2 x 3, 24 B fragments per K step instead of 36 (the fragment reads, not the MFMAs, were what
    // filled LDS: 68 KiB per wave and stage against 128 B/clk).  Position (a, b) of tile nt uses
    // column j = b + (nt & 1) of pair nt >> 1.  The 8 fragments of a window row sit in one of two
    // register sets; the next row's are read while this row's groups multiply.
    auto stage = [&](int set, int ci_next, unsigned wv, unsigned xv) {
        bf16x8 fr[2][2][4], af[3];
#pragma unroll
        for (int i = 0; i < 8; ++i) fr[0][i >> 2][i & 3] = b_frag(set, 0, i >> 2, i & 3);
        af[0] = a_frag(set, 0);
        af[1] = a_frag(set, 1);
#pragma unroll
        for (int grp = 0; grp < 16; ++grp) {
            const int wa = kGrp[grp].a, wb = kGrp[grp].b, rr = kGrp[grp].rr, cc = kGrp[grp].cc;
            // A wave issues in order and waits for the matrix pipe at every MFMA, so the other
            // instructions are spread one by one into the shadows of the four MFMAs of a group:
            // one global load | fragment reads | v_perm | LDS write.  (All 16 loads in the first
            // groups of a stage, for a longer flight time, was measured slower: several memory
            // instructions in one MFMA shadow hold up the next MFMA.)
            auto mfma = [&](int nt) {
                __builtin_amdgcn_sched_barrier(0);
                acc[nt][rr][cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    af[grp % 3], fr[wa & 1][nt >> 1][wb + (nt & 1)], acc[nt][rr][cc], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            // fragments of the next window row: row 0's four groups read two each, row 1's eight
            // groups one each, into the set the row before this one has left
            auto next_row = [&](int i) {
                fr[(wa + 1) & 1][i >> 2][i & 3] = b_frag(set, wa + 1, i >> 2, i & 3);
            };
            mfma(0);
            load_one(ci_next, wv, xv, grp, wreg[set], xreg[set]);
            if (wa == 0) next_row(2 * grp);
            if (wa == 1) next_row(grp - 4);
            mfma(1);
            if (wa == 0) next_row(2 * grp + 1);
            if (grp + 2 < 16) af[(grp + 2) % 3] = a_frag(set, grp + 2);
            mfma(2);
            const u4v t = grp < 8 ? transposed_row(wreg[set ^ 1], grp)
                                  : transposed_row(xreg[set ^ 1], grp - 8);
            mfma(3);
            if (grp < 8)
                *reinterpret_cast<u4v*>(lds + (set ^ 1) * WS_STAGE + w_lds + grp * W_PLANE) = t;
            else
                *reinterpret_cast<u4v*>(lds + (set ^ 1) * XS_STAGE_MAX + ((grp & 1) ? x_lds1 : x_lds0) +
                                        ((grp - 8) >> 1) * 16) = t;
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- first tile of this block: fill the pipeline
    int cb = 0, qt = 0;
    bool have = tile_of(0, cb, qt);
    unsigned wv_c = kInvalid, xv_c = kInvalid;
    if (have) staging_offsets(cb, qt, wv_c, xv_c);
#pragma unroll
    for (int j = 0; j < 16; ++j) load_one(0, wv_c, xv_c, j, wreg[0], xreg[0]);
    {
        const bool real = stages > 1;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            load_one(real ? KC : 0, real ? wv_c : kInvalid, real ? xv_c : kInvalid, j, wreg[1], xreg[1]);
    }
    __syncthreads();  // zero fill done before the first activation writes
#pragma unroll
    for (int j = 0; j < 16; ++j) store_one(0, j, wreg[0], xreg[0]);
    __syncthreads();

    for (int rho = 0; have; ++rho) {
        // next tile of this block (its first two stages are fetched during this tile's last two)
        int cb_n = 0, qt_n = 0;
        const bool have_n = tile_of(rho + 1, cb_n, qt_n);
        unsigned wv_n = kInvalid, xv_n = kInvalid;
        if (have_n) staging_offsets(cb_n, qt_n, wv_n, xv_n);

        // B (activations): accumulator tile nt, lane l32 holds quad
        //   q0 + qh*128 + 64*(nt/2) + 2*l32 + (nt & 1)
        // of this tile, i.e. tiles 2h and 2h+1 hold the even and odd quads of a 64-quad span: a
        // lane owns two column-neighbouring quads (KWa is even), four consecutive output columns
        const int q0 = qt * TN;
        const int q_last = (q0 + TN - 1 < a.Q ? q0 + TN - 1 : a.Q - 1);
        const int bf0 = fdiv(q0, a.dKHW), kf0 = fdiv(q0 - bf0 * KHW, a.dKW);
        const int e_first = bf0 * a.EH + kf0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int q = q0 + qh * 128 + 64 * h + 2 * l32;  // the even quad of the lane's pair
            if (q > q_last) q = q_last;                 // (past the end of the batch: results dropped)
            const int b = fdiv(q, a.dKHW);
            const int rem = q - b * KHW;
            const int ky = fdiv(rem, a.dKW), kx = rem - ky * a.KWa;
            const int r = b * a.EH + ky - e_first;  // staged row of window row 0
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = kx - a.HP + a.OFFS + j;  // staged column of joint window column j
                const int slot = (c & 1) * a.HS + (c >> 1);
                b_lds[h][j] = XS_OFF + ((gk * a.ROWS + r) * a.LWS + slot) * 16;
            }
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int sc = 0; sc < 2; ++sc)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[nt][r][sc][i] = 0.f;

        // In iteration s the loads of stage s+2 go into register set 0 and those of s+3 into set 1
        // (their previous contents are already in LDS), while sets 1 / 0 are transposed into the
        // other LDS buffer.  The last iteration requests stages 0 and 1 of the next tile instead.
        for (int s = 0; s < stages_even; s += 2) {
            const bool last = s + 2 >= stages_even;
            {
                const int t = last ? 0 : s + 2;
                stage(0, t * KC, last ? wv_n : wv_c, last ? xv_n : xv_c);
            }
            __syncthreads();
            {
                const int t = last ? 1 : s + 3;
                const bool real = t < stages;
                stage(1, real ? t * KC : 0, real ? (last ? wv_n : wv_c) : kInvalid,
                      real ? (last ? xv_n : xv_c) : kInvalid);
            }
            __syncthreads();
        }

        // ---- drain: accumulator register i of a tile holds channel 8*(i/4) + 4*gk + (i%4) of the
        // wave's 32, for the lane's quad.  Per output row the lane's two quads give four
        // consecutive columns: one 16-byte store (8 bytes for bf16 output), aligned because
        // OW % 4 == 0 and the first column is a multiple of 4.
        const int co0 = cb * TM;
        unsigned y_off[2];
        bool qv[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int q = q0 + qh * 128 + 64 * h + 2 * l32;
            qv[h] = q < a.Q;
            const int qq = qv[h] ? q : 0;
            const int b = fdiv(qq, a.dKHW);
            const int rem = qq - b * KHW;
            const int ky = fdiv(rem, a.dKW), kx = rem - ky * a.KWa;
            y_off[h] = (unsigned)(((b * g.Cout + co0 + cw * 32 + 4 * gk) * g.OH + 2 * ky) * g.OW + 2 * kx) * ES;
        }
        auto drain = [&](auto act_tag) {
            constexpr int ACT = decltype(act_tag)::value;  // -1: no epilogue at all
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (!qv[h]) continue;  // quads past the end of the batch (last tile only)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    // (a partial last channel block: groups of 8 channels exist or not as a whole)
                    if (co0 + cw * 32 + 8 * (i / 4) >= g.Cout) continue;
                    // The channel offset goes into the vector offset: a store of more than 8 bytes
                    // whose data registers are rewritten by the next instruction needs a wait state
                    // that the compiler only inserts for stores without a scalar offset register.
                    const unsigned voff = y_off[h] + (unsigned)(8 * (i / 4) + (i % 4)) * plane;
                    float bv = 0.f;
                    if constexpr (ACT >= 0)
                        if (ep.bias) {
                            // both candidates through wave-uniform indices of a constant-address-space
                            // view (the bias is never written here): scalar loads, which do not queue
                            // behind the drain's stores the way a per-lane vector load would
                            const int ch = co0 + cw * 32 + 8 * (i / 4) + (i % 4);
                            const bias_cptr bp = (bias_cptr)(unsigned long long)ep.bias;
                            const float b_lo = bp[ch], b_hi = bp[ch + 4];
                            bv = gk ? b_hi : b_lo;
                        }
#pragma unroll
                    for (int rr = 0; rr < 2; ++rr) {
                        float v[4] = {acc[2 * h][rr][0][i], acc[2 * h][rr][1][i],
                                      acc[2 * h + 1][rr][0][i], acc[2 * h + 1][rr][1][i]};
                        if constexpr (ACT >= 0) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = epilogue_t<ACT>(v[e], bv);
                        }
                        if constexpr (OUT16) {
                            const bf16x2 p0 = {(__bf16)v[0], (__bf16)v[1]}, p1 = {(__bf16)v[2], (__bf16)v[3]};
                            u2v d;
                            d.x = __builtin_bit_cast(unsigned, p0);
                            d.y = __builtin_bit_cast(unsigned, p1);
                            __builtin_amdgcn_raw_buffer_store_b64(d, rs_y, voff + rr * yrow, 0, 0);
                        } else {
                            u4v d;
                            d.x = __float_as_uint(v[0]); d.y = __float_as_uint(v[1]);
                            d.z = __float_as_uint(v[2]); d.w = __float_as_uint(v[3]);
                            __builtin_amdgcn_raw_buffer_store_b128(d, rs_y, voff + rr * yrow, 0, 0);
                        }
                    }
                }
            }
        };
        if constexpr (EPI) with_activation(ep.act, drain);  // one uniform branch per tile
        else drain(std::integral_constant<int, -1>{});
        have = have_n; cb = cb_n; qt = qt_n; wv_c = wv_n; xv_c = xv_n;
    }
}

bool make_args(const Geom& g, int dtype, AArgs& a)
{
    if (dtype != 1 && dtype != 2) return false;
    if (g.n != 4 || (g.P & 1)) return false;     // odd P: the shifted quads are the aligned ones
    // (whole groups of 8 output channels: a partial last channel block skips the missing groups)
    if (g.Cin % KC != 0 || g.Cout % 8 != 0) return false;
    if (g.W % 8 != 0) return false;              // 16-byte row chunks; makes OW a multiple of 4
    const size_t xbytes = (size_t)g.B * g.Cin * g.H * g.W * 2;
    const size_t wbytes = (size_t)g.Cout * g.Cin * g.n * g.n * 2;
    const size_t ybytes = (size_t)g.B * g.Cout * g.OH * g.OW * 4;
    const size_t lim = 0x7FFFFFF0u;              // single buffer descriptors, 32-bit byte offsets
    if (xbytes > lim || wbytes > lim || ybytes > lim) return false;
    a.g = g;
    a.KHa = g.OH / 2;
    a.KWa = g.OW / 2;
    a.HP = g.P / 2;
    const long long Q = (long long)g.B * a.KHa * a.KWa;
    if (Q > 0x7FFFFFFFLL - TN) return false;
    a.Q = (int)Q;
    a.EH = a.KHa + 2;
    // TN consecutive flattened quads touch at most this many quad rows / images; tiles that start
    // on row (image) boundaries touch exactly TN/KWa rows (one image)
    const long long khw = (long long)a.KHa * a.KWa;
    const int nrho = (TN % a.KWa == 0) ? TN / a.KWa : (TN - 2) / a.KWa + 2;
    const int nimg = (khw % TN == 0) ? 1 : (int)((TN - 2) / khw) + 2;
    a.ROWS = nrho + 2 * nimg;
    a.OFFS = (a.HP + 7) & ~7;
    // staged columns: input columns -P/2 .. W + P/2 - 1, shifted by OFFS, rounded to groups of 8
    const int cw = (a.OFFS + g.W + a.HP + 7) & ~7;
    a.HS = cw / 2 + 1;
    a.LWS = 2 * a.HS;
    // The 16 lanes of a fragment-read pass hold 32 consecutive quads, i.e. 32/KWa rows of KWa/2
    // consecutive slots each: a row pitch of KWa/2 slots modulo the 16 slots the banks span lays
    // them side by side (measured on 16x16 maps: 234 -> 224 us; padding inside the rows, which
    // would spread the staging writes instead, was slower).
    if (a.KWa < 32)
        while (a.LWS % 16 != (a.KWa / 2) % 16) ++a.LWS;
    a.C8 = g.W / 8;
    if (2 * a.ROWS * a.LWS * 16 > XS_STAGE_MAX) return false;
    if (a.ROWS * 2 * a.C8 > 256) return false;   // one staging unit per thread
    a.nco = (g.Cout + TM - 1) / TM;
    a.nqt = (int)((Q + TN - 1) / TN);
    if ((long long)a.nco * a.nqt > 0x3FFFFFFFLL) return false;
    a.ntiles = a.nco * a.nqt;
    // keep in one L2 what is bigger: the weights of a channel block or a tile's activations
    a.cb_major = ((size_t)TM * g.Cin * g.n * g.n * 2 > (size_t)(1 << 20)) ? 1 : 0;
    a.dKHW = make_fastdiv((unsigned)khw);
    a.dKW = make_fastdiv((unsigned)a.KWa);
    a.dEH = make_fastdiv((unsigned)a.EH);
    a.dC8 = make_fastdiv((unsigned)a.C8);
    a.dROWS = make_fastdiv((unsigned)a.ROWS);
    a.dNCO = make_fastdiv((unsigned)a.nco);
    a.dNQT = make_fastdiv((unsigned)a.nqt);
    return true;
}

}  // namespace

bool mfma_aligned_supported(const Geom& g, int dtype)
{
    AArgs a;
    return make_args(g, dtype, a);
}

hipError_t launch_mfma_aligned(const Geom& g, const void* x, const void* w, float* y, int dtype,
                               hipStream_t stream)
{
    AArgs a;
    if (!make_args(g, dtype, a)) return hipErrorInvalidValue;
    const size_t lds = 2 * (size_t)WS_STAGE + 2 * (size_t)XS_STAGE_MAX;
    const bool epi = has_epilogue(g.ep), out16 = dtype == 2;
    typedef void (*kernel_t)(const uint16_t*, const uint16_t*, void*, AArgs, Epilogue);
    const kernel_t kfn = out16 ? (epi ? ukst_mfma_bf16_aligned_kernel<true, true> : ukst_mfma_bf16_aligned_kernel<false, true>)
                               : (epi ? ukst_mfma_bf16_aligned_kernel<true, false> : ukst_mfma_bf16_aligned_kernel<false, false>);
    // more than 64 KiB of dynamic LDS has to be allowed per device (a property of the loaded
    // kernel, not library state); cheap enough to repeat on every call
    hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // persistent blocks: one per compute unit (a multiple of the 8 XCDs), never more than tiles,
    // and only as many as the round count needs (idle compute units leave power for the clock of
    // the busy ones)
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess)
        return e;
    int grid = (cus / 8) * 8;
    if (grid < 8) grid = 8;
    const int need = ((a.ntiles + 7) / 8) * 8;
    if (grid > need) grid = need;
    {
        const int rounds = (a.ntiles + grid - 1) / grid;
        const int fewer = (((a.ntiles + rounds - 1) / rounds + 7) / 8) * 8;
        if (fewer < grid) grid = fewer;
    }
    hipLaunchKernelGGL(kfn, dim3((unsigned)grid), dim3(256), lds, stream, (const uint16_t*)x,
                       (const uint16_t*)w, (void*)y, a, g.ep);
    return hipGetLastError();
}

}  // namespace ukst
