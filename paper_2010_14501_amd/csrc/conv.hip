// Convolution forward, input-gradient and weight-gradient as implicit GEMMs on the fp32
// matrix cores of gfx950 (v_mfma_f32_32x32x2_f32), NHWC activations, KRSC filters.
//
//   forward : Y[m, k]   = sum_{r,s,c} X[n, p*st+r-pad, q*st+s-pad, c] * W[k, r, s, c]     m = (n,p,q)
//   dgrad   : dX[m, c]  = sum_{r,s,k} dY[n, (h+pad-r)/st, (w+pad-s)/st, k] * W[k, r, s, c] m = (n,h,w)
//   wgrad   : dW[k, j]  = sum_{m}     dY[m, k] * X[n, p*st+r-pad, q*st+s-pad, c]           j = (r,s,c)
//
// These are the convolution operator and the two backward operators it is split into in the
// paper's Appendix D (parameter-gradient, then input-gradient).  wgrad with splits > 1 writes
// one partial result per split into a workspace and sums them in split order: the workspace /
// time trade-off the schedule chooses between (Section 4, "Forward/Backward Operator
// Optimization").
//
// One workgroup computes a (64*WM) x (64*WN) tile with WM*WN waves, each wave a 64x64 sub-tile
// as 2x2 MFMA blocks.  The reduction runs in steps of 16, double-buffered through LDS: global
// loads for step t+1 are issued into registers before step t's MFMAs and written to the other
// LDS buffer afterwards.  An operand whose reduction index is contiguous in memory is kept
// [row][16+4] in LDS and read as one 128-bit load per lane (lane group g = lane/32 takes
// reduction indices 8h+4g..8h+4g+3); the MFMA pairs index 8h+4g+j of both operands, so the
// order of the sum inside a step is permuted but complete.  An operand contiguous along its
// row/column index is kept [16][cols+4] and read with 32-bit loads under the same pairing.
//
// The position of a reduction step -- (r, s, c0) forward, (tap, k0) dgrad, (n, p, q) of each
// staged row for wgrad -- is carried from step to step by increments; no integer division is
// executed inside the main loop of the aligned ("fast") variants.
//
// dgrad with stride st > 1 runs one GEMM per residue class (h mod st, w mod st) of the input
// position: within a class only the filter taps r = r0 + st*i, s = s0 + st*j contribute, so no
// multiply-by-zero work is issued (a 3x3 stride-2 layer does 9 taps in total, not 36).
//
// Workgroup ids are remapped so that consecutive work items (same activation rows, neighbouring
// filter columns) run on the same XCD and share its L2: hardware deals workgroups to the 8 XCDs
// round-robin, so logical item = (id mod 8) * (grid/8) + id / 8.  A work item is (tile, reduction
// split) with the tile index fastest, so a launch with few tiles and many splits (weight
// gradients) still spreads over all XCDs and the tiles of one split share their operand rows.
#include <type_traits>

#include "bn_affine.hpp"
#include "buffer_addr.hpp"
#include "kernels.hpp"
#include "tile_stats.hpp"

namespace monet {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BK = 16;        // reduction step
constexpr int KC_LD = BK + 4; // row stride of a reduction-contiguous operand in LDS (floats)
constexpr int NUM_XCD = 8;

enum ConvMode { FWD = 0, DGRAD = 1, WGRAD = 2 };

struct TileArgs {
    const float *a;   // FWD: x, DGRAD: dy, WGRAD: dy
    const float *b;   // FWD: w, DGRAD: w,  WGRAD: x
    float *out;       // FWD: y, DGRAD: dx, WGRAD: dw or workspace
    ConvShape cs;
    int64_t Mg;       // GEMM rows (DGRAD: of residue class 0, the largest)
    int Ng;           // GEMM columns
    int64_t Kg;       // reduction length (DGRAD: recomputed per class)
    int tiles_n;
    int64_t total_tiles;
    int splits;                // reduction splits (>= 1); split z writes partial result z
    int64_t out_elems;         // elements of one (partial) result
    int accumulate;            // FWD/DGRAD, whole result only: add into the output
    // Split tiles that meet inside the kernel (FWD/DGRAD): tiles [main_tiles, total_tiles) are cut into
    // meet_splits reduction ranges, each workgroup leaves its partial tile in `part`, and the one that
    // arrives last adds the parts in range order and writes the result.  Tiles below main_tiles are whole.
    int64_t main_tiles;        // multiple of 8
    int meet_splits;           // <= 1: off
    float *part;               // (class, tile - main_tiles, range) x 64 x threads floats, register order
    float *stats_part;         // FWD, whole results only: BatchNorm partial statistics of the output (tile_stats.hpp), or null
    BnAffine affine;           // FWD, whole results only: BatchNorm apply step of the output in the epilogue (gamma == null: off)
    int64_t batch_a, batch_b, batch_out;   // FWD / WGRAD with gridDim.z > 1: z-th GEMM of a batch, operands and result this many floats apart
    // decoding a row index into (image, row, column) without a division: floor(n / Q) = umulhi(n, q_mul) >> q_shift for
    // n < 2^31 (Q >= 2), likewise P (forward rows, the filter gradient's reduction rows) and W, H (input-gradient rows at
    // stride 1); set by launch_tile
    unsigned q_mul, q_shift, p_mul, p_shift, w_mul, w_shift, h_mul, h_shift;
};

// arrivals per split tile; zero whenever no convolution kernel is running (the last arrival puts its entry back)
constexpr int MEET_SLOTS = 1 << 16;
__device__ unsigned g_meet_arrivals[MEET_SLOTS];

// puts every entry back to zero (a step that ended in an error may have left counts behind)
__global__ __launch_bounds__(256) void meet_reset_kernel() { g_meet_arrivals[blockIdx.x * 256 + threadIdx.x] = 0; }

__device__ inline float4 ld4(const float *p) { return *(const float4 *)p; }

// TAG only names the use in profiles: 0 a convolution, 1 / 2 / 3 the batched GEMMs of a Winograd forward / input gradient /
// filter gradient
// FAST: 0 element-wise loaders, 1 aligned loaders, 2 aligned loaders of a 1x1 layer whose last reduction step is partly
// empty (a kernel of its own: the two tests per step would cost the other layers 2 %, measured on ResNet-50)
template <int MODE, int WM, int WN, int FAST, int TAG = 0>
__global__ __launch_bounds__(64 * WM * WN, (WM == 2 && WN == 2 ? 4 : (WM * WN == 4 ? 3 : 2))) void conv_tile_kernel(TileArgs ta) {
    // The square four-wave tile runs four workgroups per CU (4 x 40 KiB of LDS, 128 registers per lane) and
    // prefetches one reduction step; the other tiles keep two register stages (loads two steps ahead) at three
    // (256x64, 64x256: 50 KiB of LDS) or two waves per SIMD.  Measured on the ResNet-50 layer set: 4 waves /
    // 1 stage beats 3 waves / 2 stages by 2-3 % for the square tile.
    constexpr int STAGES = (WM == 2 && WN == 2) ? 1 : 2;
    constexpr int BM = 64 * WM, BN = 64 * WN, NT = 64 * WM * WN;
    constexpr bool A_KC = (MODE != WGRAD);          // A operand reduction-contiguous?
    constexpr bool B_KC = (MODE == FWD);
    constexpr int A_LD = A_KC ? KC_LD : BM + 4;
    constexpr int B_LD = B_KC ? KC_LD : BN + 4;
    constexpr int A_SZ = A_KC ? BM * KC_LD : BK * (BM + 4);
    constexpr int B_SZ = B_KC ? BN * KC_LD : BK * (BN + 4);
    constexpr int LA = BM * 4 / NT;                 // float4 slots per thread, A tile
    constexpr int LB = BN * 4 / NT;
    __shared__ float As[2][A_SZ];
    __shared__ float Bs[2][B_SZ];
    // First layers (3 input channels): the element-wise forward loader looks the (r, s, c) of a reduction index up
    // instead of dividing (measured 925 -> 815 us on the ResNet-50 stem).  Only the four-wave non-square tiles have
    // the LDS to spare (2 KiB), and those are the ones results up to 64 channels wide, i.e. every first layer, use.
    constexpr bool HAS_KTAB = !FAST && MODE == FWD && WM * WN == 4 && !(WM == 2 && WN == 2);
    constexpr int KTAB = 256;
    __shared__ int2 ktab[HAS_KTAB ? KTAB : 1];   // x = ((r*W + s)*C + c), y = r | s << 8, or y < 0 beyond the reduction
    // Aligned filter gradient: the BK output positions a reduction step covers, decoded once per step by 16 lanes for
    // the whole workgroup: x = byte offset of the position's window in the (shifted) input tensor, y = bit per filter
    // tap that falls inside the image.  Two entries: the table of step j + 1 is written while step j is loaded.
    constexpr bool ROWTAB = FAST && MODE == WGRAD;
    __shared__ uint2 rowtab[ROWTAB ? 2 : 1][ROWTAB ? BK : 1];

    if (MODE != DGRAD) {   // batched GEMMs (the 16 products of a Winograd convolution) share one launch
        ta.a += (int64_t)blockIdx.z * ta.batch_a;
        ta.b += (int64_t)blockIdx.z * ta.batch_b;
        ta.out += (int64_t)blockIdx.z * ta.batch_out;
    }
    const ConvShape &cs = ta.cs;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g = lane >> 5;

    // XCD-aware order of the (tile, split) work items
    int nsplit = ta.splits, split;
    int64_t logical;
    bool meet = false;
    if (MODE != WGRAD && ta.meet_splits > 1) {
        // every XCD takes its share of the whole tiles first, then its share of the split ones, so the short
        // items come last everywhere and fill the ragged end of the launch
        const int64_t xcd = blockIdx.x % NUM_XCD, idx = blockIdx.x / NUM_XCD;
        const int64_t pm = ta.main_tiles / NUM_XCD;
        if (idx < pm) {
            logical = xcd * pm + idx;
            split = 0;
            nsplit = 1;
        } else {
            const int64_t nt = (ta.total_tiles - ta.main_tiles) * ta.meet_splits;
            const int64_t pt = (nt + NUM_XCD - 1) / NUM_XCD;
            const int64_t j = xcd * pt + (idx - pm);
            if (idx - pm >= pt || j >= nt) return;
            logical = ta.main_tiles + j / ta.meet_splits;
            split = (int)(j % ta.meet_splits);
            nsplit = ta.meet_splits;
            meet = true;
        }
    } else {
        const int64_t per_xcd = gridDim.x / NUM_XCD;
        const int64_t item = (int64_t)(blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
        if (item >= ta.total_tiles * nsplit) return;
        split = (int)(item / ta.total_tiles);
        logical = item - (int64_t)split * ta.total_tiles;
    }
    const int tile_n = (int)((unsigned)logical % (unsigned)ta.tiles_n);      // the host bounds the tile count below 2^31
    const int64_t tile_m = (unsigned)logical / (unsigned)ta.tiles_n;
    const int64_t row0 = tile_m * BM;
    const int col0 = tile_n * BN;
    const int RSC = (int)cs.RSC();

    // ---------------- DGRAD: residue class of this launch slice
    int64_t Mg = ta.Mg, Kg = ta.Kg;
    int ph = 0, pw = 0, r0 = 0, s0 = 0, nr = cs.R, ns = cs.S, bh = cs.pad, bw = cs.pad, Hc = cs.H, Wc = cs.W;
    // blockIdx.z = residue class (DGRAD only)
    if (MODE == DGRAD) {
        const int st = cs.stride;
        const int cls = blockIdx.z;
        ph = cls / st;
        pw = cls % st;
        Hc = (cs.H - ph + st - 1) / st;
        Wc = (cs.W - pw + st - 1) / st;
        r0 = (ph + cs.pad) % st;
        s0 = (pw + cs.pad) % st;
        nr = r0 < cs.R ? (cs.R - r0 + st - 1) / st : 0;
        ns = s0 < cs.S ? (cs.S - s0 + st - 1) / st : 0;
        bh = (ph + cs.pad - r0) / st;
        bw = (pw + cs.pad - s0) / st;
        Mg = (int64_t)cs.N * Hc * Wc;
        Kg = (int64_t)nr * ns * cs.K;
        if (row0 >= Mg) return;
        if (Kg == 0 && ta.accumulate && nsplit == 1) return;       // this class receives no contribution
    }

    // reduction range of this workgroup: split z takes steps [z*sps, (z+1)*sps) (possibly none: it
    // then contributes zeros to its partial result)
    int64_t kt0 = 0, kt1 = (Kg + BK - 1) / BK;
    if (nsplit > 1) {
        const int64_t sps = (kt1 + nsplit - 1) / nsplit;
        kt0 = split * sps;
        int64_t e = kt0 + sps;
        kt1 = e < kt1 ? e : kt1;
    }

    // ---------------- per-slot constants of the A loader
    // reduction-contiguous A (FWD / DGRAD): slot = (row, float4 j): idx = tid + s*NT, row = idx/4, j = idx%4
    // row-contiguous A (WGRAD)            : slot = (red row, float4 along k): red = idx/(BM/4), k4 = idx%(BM/4)
    int64_t a_base[LA];   // FWD/DGRAD: image base + j4; WGRAD: unused
    int a_h0[LA], a_w0[LA];
    bool a_ok[LA];
#pragma unroll
    for (int s = 0; s < LA; ++s) {
        int idx = tid + s * NT;
        if (A_KC) {
            int64_t m = row0 + idx / 4;
            a_ok[s] = m < Mg;
            int64_t mm = a_ok[s] ? m : 0;
            if (MODE == FWD) {
                const unsigned m32 = (unsigned)mm;                                 // rows are bounded below 2^31 by the host
                const unsigned t = cs.Q == 1 ? m32 : __umulhi(m32, ta.q_mul) >> ta.q_shift;
                const unsigned nn = cs.P == 1 ? t : __umulhi(t, ta.p_mul) >> ta.p_shift;
                int q = (int)(m32 - t * (unsigned)cs.Q);
                int p = (int)(t - nn * (unsigned)cs.P);
                int n = (int)nn;
                a_h0[s] = p * cs.stride - cs.pad;
                a_w0[s] = q * cs.stride - cs.pad;
                a_base[s] = (int64_t)n * cs.H * cs.W * cs.C + (idx % 4) * 4;
            } else {   // DGRAD: m = (n, hc, wc) within the residue class
                const unsigned m32 = (unsigned)mm;
                unsigned t, nn;
                if (cs.stride == 1) {      // the one class is the tensor itself: Wc = W, Hc = H
                    t = cs.W == 1 ? m32 : __umulhi(m32, ta.w_mul) >> ta.w_shift;
                    nn = cs.H == 1 ? t : __umulhi(t, ta.h_mul) >> ta.h_shift;
                } else {
                    t = m32 / (unsigned)Wc;
                    nn = t / (unsigned)Hc;
                }
                int wc = (int)(m32 - t * (unsigned)Wc);
                int hc = (int)(t - nn * (unsigned)Hc);
                int n = (int)nn;
                a_h0[s] = hc + bh;      // p = a_h0 - tap row
                a_w0[s] = wc + bw;
                a_base[s] = (int64_t)n * cs.P * cs.Q * cs.K + (idx % 4) * 4;
            }
        } else {
            int k4 = idx % (BM / 4);
            a_h0[s] = idx / (BM / 4);                       // red row within the step
            a_w0[s] = (int)(row0 + k4 * 4);                 // first out-channel of the float4
            a_ok[s] = a_w0[s] < cs.K;
            a_base[s] = 0;
        }
    }
    // ---------------- per-slot constants of the B loader
    int b_i0[LB], b_i1[LB], b_i2[LB];
    bool b_ok[LB];
    // WGRAD: (n, p, q) of the row each slot stages in the next step
    int w_n[LB], w_p[LB], w_q[LB];
#pragma unroll
    for (int s = 0; s < LB; ++s) {
        int idx = tid + s * NT;
        w_n[s] = w_p[s] = w_q[s] = 0;
        if (B_KC) {          // FWD: slot = (filter k, float4 j)
            b_i0[s] = col0 + idx / 4;
            b_ok[s] = b_i0[s] < cs.K;
            b_i1[s] = (idx % 4) * 4;
            b_i2[s] = 0;
        } else {             // slot = (red row, float4 along the column index)
            int c4 = idx % (BN / 4);
            int col = col0 + c4 * 4;
            b_i0[s] = idx / (BN / 4);                       // red row within the step
            if (MODE == DGRAD) {
                b_i1[s] = col;                              // input channel c
                b_ok[s] = col < cs.C;
                b_i2[s] = 0;
            } else {         // WGRAD: column = (r,s,c)
                b_ok[s] = col < RSC;
                int cc = b_ok[s] ? col : 0;
                int rs = cc / cs.C;
                b_i1[s] = (rs / cs.S) * cs.W + (rs % cs.S);   // r*W + s: pixel offset of the tap
                b_i2[s] = cc % cs.C;                          // c
                // tap (r, s) packed for the bounds test
                b_i1[s] |= (rs / cs.S) << 24;
                b_i2[s] |= (rs % cs.S) << 24;
                if (!FAST) {
                    int64_t m = kt0 * BK + b_i0[s];
                    int64_t mm = m < Kg ? m : 0;
                    const unsigned m32 = (unsigned)mm, t = m32 / (unsigned)cs.Q;
                    w_q[s] = (int)(m32 % (unsigned)cs.Q);
                    w_p[s] = (int)(t % (unsigned)cs.P);
                    w_n[s] = (int)(t / (unsigned)cs.P);
                }
            }
        }
    }

    // ---------------- aligned forward / input-gradient loaders: buffer addressing
    // Every vector instruction takes its cycles from the matrix pipe of the same SIMD, so an address is split into what
    // differs between lanes and never changes (a 32-bit byte offset per slot, computed once) and what changes from step
    // to step and is the same for every lane (the filter tap and the channel block: a scalar offset).  The descriptor of
    // the activation operand starts `a_shift` floats before the tensor, enough for the most negative tap offset and for
    // the offset that sends an absent element (padding, rows beyond the tensor) to the tensor's first floats instead;
    // bit t of a_taps says whether tap t of the slot exists.  The host takes this path only for tensors the 32-bit
    // offsets can span and for filters of at most 32 taps.
    unsigned a_voff[LA], a_taps[LA], b_voff[LB];
    int64_t a_shift = 0;
    if (FAST && MODE != WGRAD) {
        const int row = MODE == FWD ? cs.W : cs.Q, inner = MODE == FWD ? cs.C : cs.K;
        const int tr = MODE == FWD ? cs.R : nr, ts = MODE == FWD ? cs.S : ns;
        const int64_t back = MODE == FWD ? ((int64_t)cs.pad * row + cs.pad) * inner : 0;                    // most negative slot offset
        const int64_t reach = ((int64_t)(tr > 0 ? tr - 1 : 0) * row + (ts > 0 ? ts - 1 : 0)) * inner;       // largest tap offset
        a_shift = MODE == FWD ? (back > reach ? back : reach) : reach;
#pragma unroll
        for (int s = 0; s < LA; ++s) {
            a_voff[s] = (unsigned)((a_base[s] + ((int64_t)a_h0[s] * row + a_w0[s]) * inner + (MODE == FWD ? a_shift : 0)) * 4);
            unsigned rows = 0, cols = 0, taps = 0;
            for (int r = 0; r < tr; ++r)
                if (MODE == FWD ? (unsigned)(a_h0[s] + r) < (unsigned)cs.H : (unsigned)(a_h0[s] - r) < (unsigned)cs.P) rows |= 1u << r;
            for (int c = 0; c < ts; ++c)
                if (MODE == FWD ? (unsigned)(a_w0[s] + c) < (unsigned)cs.W : (unsigned)(a_w0[s] - c) < (unsigned)cs.Q) cols |= 1u << c;
            for (int r = 0; r < tr; ++r)
                if ((rows >> r) & 1) taps |= cols << (r * ts);
            a_taps[s] = a_ok[s] ? taps : 0u;
        }
#pragma unroll
        for (int s = 0; s < LB; ++s)
            b_voff[s] = b_ok[s] ? (unsigned)(((int64_t)b_i0[s] * RSC + b_i1[s]) * 4) : 0u;      // an absent filter row reads the tensor's start
    }
    // Aligned filter gradient: dy rows advance by a scalar offset; the window of an output position comes from the
    // row table, the slot adds its tap and channel and tests its tap's bit.  The input descriptor starts b_shift floats
    // early (a window begins up to `pad` rows and columns before the image).
    unsigned w_tapbit[LB];
    int64_t b_shift = 0;
    if (FAST && MODE == WGRAD) {
        b_shift = ((int64_t)cs.pad * cs.W + cs.pad) * cs.C;
#pragma unroll
        for (int s = 0; s < LA; ++s) a_voff[s] = a_ok[s] ? (unsigned)(((int64_t)a_h0[s] * cs.K + a_w0[s]) * 4) : 0u;
#pragma unroll
        for (int s = 0; s < LB; ++s) {
            const int r = b_i1[s] >> 24, ss = b_i2[s] >> 24;
            b_voff[s] = (unsigned)(((int64_t)(b_i1[s] & 0xffffff) * cs.C + (b_i2[s] & 0xffffff)) * 4);
            w_tapbit[s] = b_ok[s] ? 1u << (r * cs.S + ss) : 0u;
        }
    }
    const __amdgpu_buffer_rsrc_t ra = buffer_of(ta.a - a_shift), rb = buffer_of(ta.b - b_shift);
    int w_slot = 0;   // row table entry the next load_tiles reads
    // Decodes the output positions of reduction step `step`: the last wave alone, every lane the entry lane % BK (four
    // lanes write the same value), and no lane switched off on the way (the branch is uniform over the wave, the
    // rest are selects).  Measured: a version in which only 16 lanes ran this code, under a narrowed execution mask
    // while the step's loads were still in flight, now and then lost one row of a step on the two-wave tile shapes
    // when several workgroups shared a compute unit; this version does not (kernel test with many short ranges).
    auto fill_rows = [&](int64_t step, int slot) {
        if (ROWTAB && __builtin_amdgcn_readfirstlane(tid >> 6) == NT / 64 - 1) {
            const int e = tid & (BK - 1);
            const int64_t m = step * BK + e;
            const bool in = m < Kg;
            const unsigned m32 = in ? (unsigned)m : 0u;
            const unsigned t = cs.Q == 1 ? m32 : __umulhi(m32, ta.q_mul) >> ta.q_shift;
            const unsigned q = m32 - t * (unsigned)cs.Q;
            const unsigned n = cs.P == 1 ? t : __umulhi(t, ta.p_mul) >> ta.p_shift;
            const unsigned pp = t - n * (unsigned)cs.P;
            const int h0 = (int)pp * cs.stride - cs.pad, w0 = (int)q * cs.stride - cs.pad;
            const int rlo = max(0, -h0), rhi = min(cs.R, cs.H - h0), clo = max(0, -w0), chi = min(cs.S, cs.W - w0);
            const unsigned rows = rhi > rlo ? (unsigned)((1ull << rhi) - (1ull << rlo)) : 0u;
            const unsigned cols = chi > clo ? (unsigned)((1ull << chi) - (1ull << clo)) : 0u;
            unsigned taps = 0;
            for (int r = 0; r < cs.R; ++r) taps |= ((rows >> r) & 1u) ? cols << (r * cs.S) : 0u;
            const unsigned pix = (unsigned)((((int64_t)n * cs.H + h0) * cs.W + w0) * cs.C + b_shift) * 4u;
            rowtab[slot][e] = make_uint2(in ? pix : 0u, in ? taps : 0u);
        }
    };

    // ---------------- position of the next step to load (uniform over the workgroup)
    int64_t kk0 = kt0 * BK;
    int u_r = 0, u_s = 0, u_c = 0;   // FWD: (r, s, c0); DGRAD: (tap row, tap column, k0)
    if (MODE != WGRAD && kt0 > 0) {  // a later reduction split starts in the middle: locate it once
        const int inner = MODE == FWD ? cs.C : cs.K, cols = MODE == FWD ? cs.S : ns;
        int tap = (int)(kk0 / inner);
        u_c = (int)(kk0 % inner);
        u_r = tap / cols;
        u_s = tap % cols;
    }

    const bool use_ktab = HAS_KTAB && (ta.Kg + BK - 1) / BK * BK <= KTAB;
    if (HAS_KTAB && use_ktab) {
        for (int kk = tid; kk < KTAB; kk += NT) {
            int2 e = make_int2(0, -1);
            if (kk < Kg) {
                const int rs = kk / cs.C, c = kk % cs.C;
                const int r = rs / cs.S, ss = rs % cs.S;
                e = make_int2((r * cs.W + ss) * cs.C + c, r | (ss << 8));
            }
            ktab[kk] = e;
        }
        __syncthreads();
    }

    float4 a_set0[LA], b_set0[LB], a_set1[LA], b_set1[LB];   // two register stages: loads run two steps ahead

    // In the aligned variants every load is issued unconditionally (an out-of-range slot reads the
    // tensor's first 16 bytes instead) and zeroed when it is written to LDS: without branches around
    // the loads the compiler can count outstanding loads exactly and wait only for the older stage.
    // pm: which slots hold data (lane masks, kept in scalar registers).
    struct Present { bool a[LA], b[LB]; };
    auto load_tiles = [&](float4 (&a_reg)[LA], float4 (&b_reg)[LB], Present &pm, int &full) {
        bool every = FAST;      // every slot of this lane holds data
        // 1x1 layers whose reduction length is a multiple of 4 only: the last step holds `left` < 16 reduction indices
        // (uniform over the workgroup; every other step, and every step of the other layers, is whole)
        const int left = (int)(Kg - kk0 < BK ? Kg - kk0 : BK);
        const bool part_step = FAST == 2 && MODE != WGRAD && left < BK;
        // aligned filter gradient: the table entries of this lane's B slots, read before anything else is issued
        unsigned long long w_row[LB];
        if (ROWTAB) {
#pragma unroll
            for (int s = 0; s < LB; ++s) w_row[s] = *(const unsigned long long *)&rowtab[w_slot][b_i0[s]];
        }
        // ======== A
#pragma unroll
        for (int s = 0; s < LA; ++s) {
            int idx = tid + s * NT;
            float4 v = make_float4(0, 0, 0, 0);
            bool ok = !FAST;    // the element-wise variants zero what they do not load
            if (MODE == FWD) {
                if (FAST) {
                    // scalar: tap number and offset; an absent element reads float u_c of the tensor instead
                    const unsigned tapoff = (unsigned)(((int64_t)u_r * cs.W + u_s) * cs.C);
                    ok = (a_taps[s] >> (u_r * cs.S + u_s)) & 1u;
                    if (part_step) ok = ok && (idx % 4) * 4 < left;
                    const bf4 q = buffer_load4(ra, ok ? a_voff[s] : ((unsigned)a_shift - tapoff) * 4u, (tapoff + (unsigned)u_c) * 4u);
                    v = make_float4(q.x, q.y, q.z, q.w);
                } else if (HAS_KTAB && use_ktab) {
                    // branch-free: an element outside the image or the reduction reads the tensor's first word and is zeroed
                    float e[4];
                    const float *pix = ta.a + (a_base[s] - (idx % 4) * 4 + ((int64_t)a_h0[s] * cs.W + a_w0[s]) * cs.C);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int2 t = ktab[(int)kk0 + (idx % 4) * 4 + u];
                        const int h = a_h0[s] + (t.y & 0xff), w = a_w0[s] + ((t.y >> 8) & 0xff);
                        const bool in = a_ok[s] && t.y >= 0 && (unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W;
                        const float got = *(in ? pix + t.x : ta.a);
                        e[u] = in ? got : 0.0f;
                    }
                    v = make_float4(e[0], e[1], e[2], e[3]);
                } else {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        int kk = (int)kk0 + (idx % 4) * 4 + u;
                        if (a_ok[s] && kk < Kg) {
                            int rs = kk / cs.C, c = kk % cs.C;
                            int r = rs / cs.S, ss = rs % cs.S;
                            int h = a_h0[s] + r, w = a_w0[s] + ss;
                            if ((unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                                e[u] = ta.a[a_base[s] - (idx % 4) * 4 + ((int64_t)h * cs.W + w) * cs.C + c];
                        }
                    }
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else if (MODE == DGRAD) {
                // reduction index = (tap row, tap column, k); FAST: K % 16 == 0 so a step stays inside one tap
                if (FAST) {
                    // the descriptor starts a_shift floats early: tap (u_r, u_s) lies tapoff floats before the slot's offset
                    const unsigned tapoff = (unsigned)(((int64_t)u_r * cs.Q + u_s) * cs.K);
                    ok = (a_taps[s] >> (u_r * ns + u_s)) & 1u;
                    if (part_step) ok = ok && (idx % 4) * 4 < left;
                    const bf4 q = buffer_load4(ra, ok ? a_voff[s] : tapoff * 4u, ((unsigned)a_shift - tapoff + (unsigned)u_c) * 4u);
                    v = make_float4(q.x, q.y, q.z, q.w);
                } else {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        int kk = (int)kk0 + (idx % 4) * 4 + u;
                        if (a_ok[s] && kk < Kg) {
                            int tap = kk / cs.K, k = kk % cs.K;
                            int p = a_h0[s] - tap / ns, q = a_w0[s] - tap % ns;
                            if ((unsigned)p < (unsigned)cs.P && (unsigned)q < (unsigned)cs.Q)
                                e[u] = ta.a[a_base[s] - (idx % 4) * 4 + ((int64_t)p * cs.Q + q) * cs.K + k];
                        }
                    }
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else {   // WGRAD: A[red = m][row = k] = dy[m][k]
                int64_t m = kk0 + a_h0[s];
                if (FAST) {
                    // an absent element (row beyond the reduction, column beyond K) reads the step's first row instead
                    const int left = (int)(Kg - kk0 < BK ? Kg - kk0 : BK);
                    ok = a_ok[s] && a_h0[s] < left;
                    const bf4 q = buffer_load4(ra, ok ? a_voff[s] : 0u, (unsigned)(kk0 * cs.K) * 4u);
                    v = make_float4(q.x, q.y, q.z, q.w);
                } else if (m < Kg) {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (a_w0[s] + u < cs.K) e[u] = ta.a[m * cs.K + a_w0[s] + u];
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            }
            a_reg[s] = v;
            pm.a[s] = ok;
            every = every && ok;
        }
        // ======== B
#pragma unroll
        for (int s = 0; s < LB; ++s) {
            int idx = tid + s * NT;
            float4 v = make_float4(0, 0, 0, 0);
            bool ok = !FAST;
            if (MODE == FWD) {
                if (FAST) {
                    ok = b_ok[s];
                    unsigned vo = b_voff[s];
                    // beyond the filter row's end: the row's floats kk0 .. kk0 + 3 instead (in bounds), zeroed below
                    if (part_step && b_i1[s] >= left) { vo = ok ? vo - (unsigned)b_i1[s] * 4u : 0u; ok = false; }
                    const bf4 q = buffer_load4(rb, vo, (unsigned)kk0 * 4u);
                    v = make_float4(q.x, q.y, q.z, q.w);
                } else {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (b_ok[s] && kk0 + b_i1[s] + u < Kg) e[u] = ta.b[(int64_t)b_i0[s] * RSC + kk0 + b_i1[s] + u];
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else if (MODE == DGRAD) {
                // B[red = (tap, k)][col = c] = W[k][r0 + st*tr][s0 + st*ts][c]
                int64_t kk = kk0 + b_i0[s];
                if (FAST) {
                    // a step reaches beyond the reduction only in the last step of a 1x1 layer with K % 16 != 0 (part_step)
                    const int r = r0 + cs.stride * u_r, ss = s0 + cs.stride * u_s;
                    ok = b_ok[s];
                    unsigned vo = b_voff[s];
                    // a filter beyond the last one: the step's first filter instead (in bounds), zeroed below
                    if (part_step && b_i0[s] >= left) { vo = ok ? vo - (unsigned)b_i0[s] * (unsigned)RSC * 4u : 0u; ok = false; }
                    const bf4 q = buffer_load4(rb, vo, (unsigned)(((int64_t)u_c * RSC + (r * cs.S + ss) * cs.C) * 4));
                    v = make_float4(q.x, q.y, q.z, q.w);
                } else if (kk < Kg) {
                    int tap = (int)kk / cs.K, k = (int)kk % cs.K;
                    int r = r0 + cs.stride * (tap / ns), ss = s0 + cs.stride * (tap % ns);
                    const float *src = ta.b + (int64_t)k * RSC + (r * cs.S + ss) * cs.C + b_i1[s];
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (b_i1[s] + u < cs.C) e[u] = src[u];
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else {   // WGRAD: B[red = m][col = (r,s,c)] = x[n, p*st+r-pad, q*st+s-pad, c]
                int64_t m = kk0 + b_i0[s];
                if (FAST) {
                    const unsigned pix = (unsigned)w_row[s], taps = (unsigned)(w_row[s] >> 32);
                    ok = (taps & w_tapbit[s]) != 0u;
                    const bf4 q = buffer_load4(rb, ok ? pix + b_voff[s] : (unsigned)b_shift * 4u, 0u);
                    v = make_float4(q.x, q.y, q.z, q.w);
                } else if (m < Kg) {
                    int h0 = w_p[s] * cs.stride - cs.pad, w0 = w_q[s] * cs.stride - cs.pad;
                    const float *img = ta.b + (int64_t)w_n[s] * cs.H * cs.W * cs.C;
                    {
                        float e[4] = {0, 0, 0, 0};
                        int col = col0 + (idx % (BN / 4)) * 4;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            int cc = col + u;
                            if (cc < RSC) {
                                int rs = cc / cs.C, c = cc % cs.C;
                                int r = rs / cs.S, ss = rs % cs.S;
                                int h = h0 + r, w = w0 + ss;
                                if ((unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                                    e[u] = img[((int64_t)h * cs.W + w) * cs.C + c];
                            }
                        }
                        v = make_float4(e[0], e[1], e[2], e[3]);
                    }
                }
            }
            b_reg[s] = v;
            pm.b[s] = ok;
            every = every && ok;
        }
        // uniform over the wave: when nothing is absent the LDS write below needs no selects (vector instructions that
        // would take their cycles from the matrix pipe)
        full = __all(every) ? 1 : 0;
        // ======== advance to the next step
        kk0 += BK;
        if (MODE == FWD) {
            u_c += BK;
            if (u_c >= cs.C) { u_c = 0; if (++u_s == cs.S) { u_s = 0; ++u_r; } }
        } else if (MODE == DGRAD) {
            u_c += BK;
            if (u_c >= cs.K) { u_c = 0; if (++u_s == ns) { u_s = 0; ++u_r; } }
        } else if (FAST) {
            // kk0 now names the step after the one just loaded: its table goes into the entry that step's loads will
            // read; every wave finished reading that entry before the barrier that ended the previous step
            fill_rows(kk0 / BK, w_slot ^ 1);
            w_slot ^= 1;
        } else {
#pragma unroll
            for (int s = 0; s < LB; ++s) {
                w_q[s] += BK;
                while (w_q[s] >= cs.Q) {
                    w_q[s] -= cs.Q;
                    if (++w_p[s] == cs.P) { w_p[s] = 0; ++w_n[s]; }
                }
            }
        }
    };

    auto store_tiles = [&](int buf, const float4 (&a_reg)[LA], const float4 (&b_reg)[LB], const Present &pm, int full) {
        const float4 zero = make_float4(0, 0, 0, 0);
        auto put = [&](auto whole) {
#pragma unroll
            for (int s = 0; s < LA; ++s) {
                int idx = tid + s * NT;
                float4 v = decltype(whole)::value || pm.a[s] ? a_reg[s] : zero;
                if (A_KC) *(float4 *)&As[buf][(idx / 4) * KC_LD + (idx % 4) * 4] = v;
                else *(float4 *)&As[buf][(idx / (BM / 4)) * A_LD + (idx % (BM / 4)) * 4] = v;
            }
#pragma unroll
            for (int s = 0; s < LB; ++s) {
                int idx = tid + s * NT;
                float4 v = decltype(whole)::value || pm.b[s] ? b_reg[s] : zero;
                if (B_KC) *(float4 *)&Bs[buf][(idx / 4) * KC_LD + (idx % 4) * 4] = v;
                else *(float4 *)&Bs[buf][(idx / (BN / 4)) * B_LD + (idx % (BN / 4)) * 4] = v;
            }
        };
        // uniform over the wave: a step in which no lane misses anything is written without the selects
        if (full) put(std::true_type{});
        else put(std::false_type{});
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto compute = [&](int buf) {
        const float *A = As[buf], *B = Bs[buf];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float af[2][4], bf[2][4];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                int r = wm * 64 + mi * 32 + l32;
                if (A_KC) {
                    float4 v = *(const float4 *)&A[r * KC_LD + 8 * h + 4 * g];
                    af[mi][0] = v.x; af[mi][1] = v.y; af[mi][2] = v.z; af[mi][3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) af[mi][j] = A[(8 * h + 4 * g + j) * A_LD + r];
                }
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                int c = wn * 64 + ni * 32 + l32;
                if (B_KC) {
                    float4 v = *(const float4 *)&B[c * KC_LD + 8 * h + 4 * g];
                    bf[ni][0] = v.x; bf[ni][1] = v.y; bf[ni][2] = v.z; bf[ni][3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) bf[ni][j] = B[(8 * h + 4 * g + j) * B_LD + c];
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi][j], bf[ni][j], acc[mi][ni], 0, 0, 0);
        }
    };

    // Software pipeline, loads two steps ahead: while step t is computed from LDS buffer t%2, the
    // registers of stage (t+1)%2 hold step t+1 (on its way or landed) and the loads of step t+2 are
    // issued into stage t%2.
    if (STAGES == 1 && kt0 < kt1) {
        const int64_t steps = kt1 - kt0;
        Present pm0{};
        int full0 = 0;
        if (ROWTAB) {
            fill_rows(kt0, 0);
            __syncthreads();
        }
        load_tiles(a_set0, b_set0, pm0, full0);
        store_tiles(0, a_set0, b_set0, pm0, full0);
        __syncthreads();
        for (int64_t t = 0; t + 1 < steps; ++t) {
            load_tiles(a_set0, b_set0, pm0, full0);
            __builtin_amdgcn_sched_barrier(0);
            compute((int)(t & 1));
            __builtin_amdgcn_sched_barrier(0);
            store_tiles((int)((t + 1) & 1), a_set0, b_set0, pm0, full0);
            __syncthreads();
        }
        compute((int)((steps - 1) & 1));
    } else if (kt0 < kt1) {
        const int64_t steps = kt1 - kt0;
        Present pm0{}, pm1{};
        int full0 = 0, full1 = 0;
        if (ROWTAB) {
            fill_rows(kt0, 0);
            __syncthreads();
        }
        load_tiles(a_set0, b_set0, pm0, full0);
        if (ROWTAB) __syncthreads();    // the second load writes the table entry the first one read
        if (steps > 1) load_tiles(a_set1, b_set1, pm1, full1);
        store_tiles(0, a_set0, b_set0, pm0, full0);
        __syncthreads();
        int64_t t = 0;
        // The scheduling fences keep the order loads -> MFMAs -> LDS write -> barrier: left alone, the
        // compiler hoists the LDS write (and with it the wait for the loads) above the MFMAs.
        // Steady state: both halves always issue their loads, so the number of loads in flight at
        // each LDS write is the same on every path and the wait can name exactly the older stage.
        for (; t + 3 < steps; t += 2) {
            // even step: LDS buffer 0, next step waits in stage 1
            load_tiles(a_set0, b_set0, pm0, full0);
            __builtin_amdgcn_sched_barrier(0);
            compute(0);
            __builtin_amdgcn_sched_barrier(0);
            store_tiles(1, a_set1, b_set1, pm1, full1);
            __syncthreads();
            // odd step: LDS buffer 1, next step waits in stage 0
            load_tiles(a_set1, b_set1, pm1, full1);
            __builtin_amdgcn_sched_barrier(0);
            compute(1);
            __builtin_amdgcn_sched_barrier(0);
            store_tiles(0, a_set0, b_set0, pm0, full0);
            __syncthreads();
        }
        // Drain: one to three steps are left; step t sits in buffer 0, step t+1 (if any) in stage 1.
        if (t + 2 < steps) load_tiles(a_set0, b_set0, pm0, full0);
        compute(0);
        if (t + 1 < steps) {
            store_tiles(1, a_set1, b_set1, pm1, full1);
            __syncthreads();
            compute(1);
            if (t + 2 < steps) {
                store_tiles(0, a_set0, b_set0, pm0, full0);
                __syncthreads();
                compute(0);
            }
        }
    }

    // ---------------- epilogue: lane holds column l32 of rows 8*(v/4) + 4*g + v%4 of each 32x32 block
    float *out = ta.out;
    if (!meet) out += (int64_t)split * ta.out_elems;
    const bool do_acc = MODE != WGRAD && ta.accumulate && (nsplit == 1 || meet);
    if (MODE != WGRAD && meet) {
        // Leave this range's partial tile (register order: 16 float4 per lane, each wave instruction writes
        // 1 KiB in a row), then count the arrival.  Release before the count and acquire after it order the
        // parts of the other workgroups, on whichever XCD they ran, before the loads below.
        const int64_t uid = (MODE == DGRAD ? (int64_t)blockIdx.z * (ta.total_tiles - ta.main_tiles) : 0) + (logical - ta.main_tiles);
        float *tile_part = ta.part + uid * nsplit * (int64_t)(64 * NT);
        {
            float4 *mine = (float4 *)(tile_part + (int64_t)split * (64 * NT));
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const floatx16 &a = acc[b >> 1][b & 1];
                    mine[(b * 4 + q4) * NT + tid] = float4{a[4 * q4], a[4 * q4 + 1], a[4 * q4 + 2], a[4 * q4 + 3]};
                }
        }
        __threadfence();
        __syncthreads();                                       // also: every wave is done with the operand tiles in LDS
        unsigned *slot = (unsigned *)&As[0][0];                // LDS is full (four workgroups per CU): borrow a word
        if (tid == 0) *slot = atomicAdd(&g_meet_arrivals[uid], 1u);
        __syncthreads();
        const unsigned arrived = *slot;
        if (arrived != (unsigned)(nsplit - 1)) return;
        __threadfence();
        if (tid == 0) g_meet_arrivals[uid] = 0;
        // last to arrive: add the parts in range order (its own comes back from memory like the others, so
        // the sum does not depend on which range arrived last)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            floatx16 t;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float4 v = ((const float4 *)tile_part)[(b * 4 + q4) * NT + tid];
                t[4 * q4] = v.x; t[4 * q4 + 1] = v.y; t[4 * q4 + 2] = v.z; t[4 * q4 + 3] = v.w;
            }
            for (int z = 1; z < nsplit; ++z) {
                const float4 *src = (const float4 *)(tile_part + (int64_t)z * (64 * NT));
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    float4 v = src[(b * 4 + q4) * NT + tid];
                    t[4 * q4] += v.x; t[4 * q4 + 1] += v.y; t[4 * q4 + 2] += v.z; t[4 * q4 + 3] += v.w;
                }
            }
            acc[b >> 1][b & 1] = t;
        }
    }
    if (FAST && (ta.Ng & 3) == 0) {
        // Vector path: each wave transposes its 64x64 result through a private 16x64 LDS patch, four
        // passes of 16 rows, and writes whole 16-byte pieces, 256 contiguous bytes per row.
        constexpr int NW = WM * WN;
        __syncthreads();   // every wave has finished reading the operand tiles
        float *stage = (2 * A_SZ >= NW * 1024 ? &As[0][0] : &Bs[0][0]) + wave * 1024;
        const bool want_stats = MODE == FWD && ta.stats_part != nullptr;
        LaneStats ls;
        ls.init();
        // a lane writes the same four columns in every pass: one pair of BatchNorm coefficients each
        const bool want_affine = MODE == FWD && ta.affine.gamma != nullptr;
        float bn_a[4] = {1, 1, 1, 1}, bn_b[4] = {0, 0, 0, 0};
        if (MODE == FWD && want_affine) {
            const int c0 = col0 + wn * 64 + 4 * (lane & 15);
            if (c0 < ta.Ng) {
#pragma unroll
                for (int j = 0; j < 4; ++j) bn_affine_coeffs(ta.affine.gamma, ta.affine.beta, ta.affine.stats, ta.Ng, c0 + j, bn_a[j], bn_b[j]);
            }
        }
        // the sign code of a ReLU applied here: per row one word per 64 columns, i.e. per wave; the values are read once more
        // from the LDS patch with lane = column, so that one ballot is one word
        const bool want_mask = MODE == FWD && want_affine && ta.affine.relu && ta.affine.mask != nullptr && col0 + wn * 64 < ta.Ng;
        float bn_ac = 1.0f, bn_bc = 0.0f;
        if (MODE == FWD && want_mask) bn_affine_coeffs(ta.affine.gamma, ta.affine.beta, ta.affine.stats, ta.Ng, col0 + wn * 64 + lane, bn_ac, bn_bc);
        // A tile that lies inside the result whole (all but the last row of tiles and, for widths that are no multiple
        // of the tile, the last column) writes through buffer addressing: the descriptor starts at the tile, a lane's
        // byte offset inside the tile never changes and the row of a pass is a scalar offset, so a store costs no vector
        // instruction for its address and none for a bounds test.
        const bool inside = row0 + BM <= Mg && col0 + BN <= ta.Ng && ta.Ng < (1 << 24) && !(MODE == DGRAD && cs.stride > 1);
        const unsigned row_bytes = (unsigned)ta.Ng * 4u;
        const int64_t tile_at = (row0 + wm * 64) * ta.Ng + col0 + wn * 64;
        const __amdgpu_buffer_rsrc_t r_out = buffer_of(out + tile_at);
        const __amdgpu_buffer_rsrc_t r_relu = buffer_of(MODE == FWD && ta.affine.relu_out ? ta.affine.relu_out + tile_at : out + tile_at);
        const unsigned t_voff = (unsigned)(lane >> 4) * row_bytes + 16u * (unsigned)(lane & 15);
        auto emit = [&](auto whole_tile) {
            constexpr bool IN = decltype(whole_tile)::value;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int mi = q >> 1, vbase = 8 * (q & 1);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int vv = 0; vv < 8; ++vv)
                        stage[(8 * (vv >> 2) + 4 * g + (vv & 3)) * 64 + ni * 32 + l32] = acc[mi][ni][vbase + vv];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = lane + 64 * i, rl = idx >> 4, c4 = idx & 15;
                    float4 val = *(const float4 *)&stage[rl * 64 + 4 * c4];
                    const int64_t row = row0 + wm * 64 + 16 * q + rl;
                    const int col = col0 + wn * 64 + 4 * c4;
                    if (IN || (row < Mg && col < ta.Ng)) {
                        const unsigned t_soff = (unsigned)(16 * q + 4 * i) * row_bytes;
                        int64_t orow = row;
                        if (!IN && MODE == DGRAD && cs.stride > 1) {
                            // rows are bounded below 2^31 by the host: 32-bit divisions
                            const unsigned r32 = (unsigned)row, t = r32 / (unsigned)Wc, n = t / (unsigned)Hc;
                            const int wc = (int)(r32 - t * (unsigned)Wc), hc = (int)(t - n * (unsigned)Hc);
                            orow = ((int64_t)n * cs.H + (hc * cs.stride + ph)) * cs.W + (wc * cs.stride + pw);
                        }
                        float4 *dst = (float4 *)(out + orow * ta.Ng + col);
                        if (do_acc) {
                            float4 o;
                            if (IN) { const bf4 t = buffer_load4(r_out, t_voff, t_soff); o = make_float4(t.x, t.y, t.z, t.w); }
                            else o = *dst;
                            val.x += o.x; val.y += o.y; val.z += o.z; val.w += o.w;
                        }
                        if (MODE == FWD && want_affine)
                            val = float4{bn_affine(val.x, bn_a[0], bn_b[0]), bn_affine(val.y, bn_a[1], bn_b[1]), bn_affine(val.z, bn_a[2], bn_b[2]),
                                         bn_affine(val.w, bn_a[3], bn_b[3])};
                        if (MODE == FWD && want_affine && ta.affine.relu) {
                            const float4 rv = float4{relu_clamp(val.x, ta.affine.relu), relu_clamp(val.y, ta.affine.relu),
                                                     relu_clamp(val.z, ta.affine.relu), relu_clamp(val.w, ta.affine.relu)};
                            if (ta.affine.relu_out) {
                                if (IN) buffer_store4(r_relu, t_voff, t_soff, bf4{rv.x, rv.y, rv.z, rv.w});
                                else *(float4 *)(ta.affine.relu_out + orow * ta.Ng + col) = rv;
                            } else val = rv;
                        }
                        if (IN) buffer_store4(r_out, t_voff, t_soff, bf4{val.x, val.y, val.z, val.w});
                        else *dst = val;
                        if (MODE == FWD && want_stats) {
                            if (!IN) ls.add(val.x, val.y, val.z, val.w);
                            else if (q == 0 && i == 0) ls.add_first(val.x, val.y, val.z, val.w);
                            else ls.add_next(val.x, val.y, val.z, val.w);
                        }
                    }
                }
                if (MODE == FWD && want_mask) {      // uniform over the wave
                    unsigned w_lo = 0, w_hi = 0;
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr) {
                        const float e = bn_affine(stage[rr * 64 + lane], bn_ac, bn_bc);
                        const bool pass = ta.affine.relu == 2 ? (e > 0.0f && e < 6.0f) : e > 0.0f;
                        const unsigned long long word = __ballot(pass);
                        if (lane == rr) { w_lo = (unsigned)word; w_hi = (unsigned)(word >> 32); }
                    }
                    const int64_t mrow = row0 + wm * 64 + 16 * q + lane;       // lanes 0 .. 15 hold the words of the pass's rows
                    if (lane < 16 && mrow < Mg) ta.affine.mask[(mrow * ta.Ng + col0 + wn * 64) >> 6] = ((unsigned long long)w_hi << 32) | w_lo;
                }
            }
        };
        if (inside) emit(std::true_type{});
        else emit(std::false_type{});
        if (MODE == FWD && want_stats) {
            // this wave's 64 rows are one row group of the statistics; lanes l, l^16, l^32, l^48 share their columns
            float n, mean[4], m2[4];
            merge_lane_stats(ls, lane, n, mean, m2);
            const int64_t first = row0 + wm * 64;
            if (first < Mg) store_group_stats(ta.stats_part, first / STAT_ROWS, ta.Ng, col0 + wn * 64 + 4 * (lane & 15), lane, mean, m2);
        }
        return;
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int64_t row = row0 + wm * 64 + mi * 32 + 8 * (v / 4) + 4 * g + (v % 4);
            if (row >= Mg) continue;
            int64_t orow = row;
            if (MODE == DGRAD && cs.stride > 1) {   // class row (n,hc,wc) -> position (n, hc*st+ph, wc*st+pw)
                const unsigned r32 = (unsigned)row, t = r32 / (unsigned)Wc, n = t / (unsigned)Hc;      // rows are bounded below 2^31 by the host
                const int wc = (int)(r32 - t * (unsigned)Wc), hc = (int)(t - n * (unsigned)Hc);
                orow = ((int64_t)n * cs.H + (hc * cs.stride + ph)) * cs.W + (wc * cs.stride + pw);
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                int col = col0 + wn * 64 + ni * 32 + l32;
                if (col < ta.Ng) {
                    float *dst = out + orow * ta.Ng + col;
                    float r = acc[mi][ni][v];
                    if (do_acc) r += *dst;
                    *dst = r;
                }
            }
        }
}

// Sums `splits` partial results in a fixed order.  Block = SL waves; wave sl adds splits sl, sl+SL, ...
// of 64 consecutive elements (four independent partial sums per lane to keep loads in flight),
// then the SL per-wave sums are added in wave order.
template <int SL>
__global__ __launch_bounds__(64 * SL) void split_reduce_kernel(const float *__restrict__ ws, float *dw, int64_t n, int splits, int accumulate) {
    __shared__ float sh[SL][64];
    const int lane = threadIdx.x & 63, sl = threadIdx.x >> 6;
    for (int64_t base = (int64_t)blockIdx.x * 64; base < n; base += (int64_t)gridDim.x * 64) {
        const int64_t i = base + lane;
        float s0 = 0, s1 = 0, s2 = 0, s3 = 0;
        if (i < n) {
            int z = sl;
            for (; z + 3 * SL < splits; z += 4 * SL) {
                s0 += ws[(int64_t)z * n + i];
                s1 += ws[(int64_t)(z + SL) * n + i];
                s2 += ws[(int64_t)(z + 2 * SL) * n + i];
                s3 += ws[(int64_t)(z + 3 * SL) * n + i];
            }
            for (; z < splits; z += SL) s0 += ws[(int64_t)z * n + i];
        }
        sh[sl][lane] = (s0 + s1) + (s2 + s3);
        __syncthreads();
        if (sl == 0 && i < n) {
            float s = sh[0][lane];
#pragma unroll
            for (int j = 1; j < SL; ++j) s += sh[j][lane];
            dw[i] = accumulate ? dw[i] + s : s;
        }
        __syncthreads();
    }
}

void launch_split_reduce(hipStream_t st, const float *ws, float *dw, int64_t n, int splits, bool accumulate) {
    const int acc = accumulate ? 1 : 0;
    int grid = (int)std::min<int64_t>((n + 63) / 64, 8192);
    if (splits >= 64) hipLaunchKernelGGL((split_reduce_kernel<16>), dim3(grid), dim3(1024), 0, st, ws, dw, n, splits, acc);
    else if (splits >= 16) hipLaunchKernelGGL((split_reduce_kernel<4>), dim3(grid), dim3(256), 0, st, ws, dw, n, splits, acc);
    else hipLaunchKernelGGL((split_reduce_kernel<1>), dim3(grid), dim3(64), 0, st, ws, dw, n, splits, acc);
    hip_check(hipGetLastError(), "split reduce launch");
}

// floor(n / d) = umulhi(n, mul) >> shift for every n < 2^31 (d >= 2): mul = ceil(2^(31 + l) / d) with l = ceil(log2 d)
// fits 32 bits, and its excess over 2^(31 + l) / d, below d / 2^(31 + l) <= 2^-31, times n stays below one unit
void magic_of(unsigned d, unsigned &mul, unsigned &shift) {
    mul = 0; shift = 0;
    if (d < 2) return;
    unsigned l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    mul = (unsigned)((((uint64_t)1 << (31 + l)) + d - 1) / d);
    shift = l - 1;
}
void set_row_magic(TileArgs &ta) {
    magic_of((unsigned)ta.cs.Q, ta.q_mul, ta.q_shift);
    magic_of((unsigned)ta.cs.P, ta.p_mul, ta.p_shift);
    magic_of((unsigned)ta.cs.W, ta.w_mul, ta.w_shift);
    magic_of((unsigned)ta.cs.H, ta.h_mul, ta.h_shift);
}

void check_shape(const ConvShape &cs) {
    if (cs.N <= 0 || cs.H <= 0 || cs.W <= 0 || cs.C <= 0 || cs.K <= 0 || cs.R <= 0 || cs.S <= 0 || cs.stride <= 0 || cs.pad < 0)
        throw KernelError("conv: bad shape");
    if (cs.P != (cs.H + 2 * cs.pad - cs.R) / cs.stride + 1 || cs.Q != (cs.W + 2 * cs.pad - cs.S) / cs.stride + 1 || cs.P <= 0 || cs.Q <= 0)
        throw KernelError("conv: output size does not match input, filter, stride and padding");
    if ((int64_t)cs.R * cs.S * cs.C > (1ll << 24) || (int64_t)cs.R * cs.S * cs.K > (1ll << 24) || cs.M() > (1ll << 31) - 64 ||
        (int64_t)cs.N * cs.H * cs.W > (1ll << 31) - 64 || (int64_t)cs.H * cs.W >= (1 << 24) || cs.R > 127 || cs.S > 127)
        throw KernelError("conv: shape too large");
    if (cs.stride > 8) throw KernelError("conv: stride too large");
}

// How a launch divides its reduction.  `splits` > 1 asks for that many ranges on every tile: partial results go
// to `splits` full-size slabs that a second kernel adds in range order.  `splits` == 1 with a workspace (FWD /
// DGRAD at stride 1) lets the ragged last round, the tiles beyond a multiple of the CU count, be cut as far as the
// workspace allows; those partial tiles meet inside the kernel.  (Letting every tile of a launch meet that way
// was measured too: the device-wide release each split workgroup performs costs more than the second kernel.)
constexpr int NUM_CU = 256;

template <int MODE, int WM, int WN, int TAG = 0>
void launch_tile(hipStream_t st, TileArgs ta, bool fast, int zdim, float *out, int splits, float *ws, size_t ws_bytes, int64_t steps,
                 bool accumulate, const char *who) {
    constexpr int BM = 64 * WM, BN = 64 * WN, NT = 64 * WM * WN;
    if (splits < 1) throw KernelError(std::string(who) + ": splits must be >= 1");
    set_row_magic(ta);
    if (splits > steps) splits = (int)std::max<int64_t>(steps, 1);
    int64_t tiles_m = (ta.Mg + BM - 1) / BM;
    ta.tiles_n = (ta.Ng + BN - 1) / BN;
    ta.total_tiles = tiles_m * ta.tiles_n;
    ta.out = out;
    ta.splits = 1;
    ta.accumulate = accumulate ? 1 : 0;
    ta.main_tiles = 0;
    ta.meet_splits = 0;
    ta.part = nullptr;
    const size_t tile_bytes = (size_t)BM * BN * sizeof(float);
    bool slabs = false;
    if (splits > 1) {
        if (!ws || ws_bytes < (size_t)splits * ta.out_elems * 4) throw KernelError(std::string(who) + ": workspace too small for the requested splits");
        slabs = true;
        ta.out = ws;
        ta.splits = splits;
    } else if (MODE != WGRAD && zdim == 1 && ws && ta.total_tiles % NUM_CU) {
        const int64_t tail = ta.total_tiles % NUM_CU;
        int64_t s = std::min<int64_t>({NUM_CU / tail, steps / 4, 16, (int64_t)(ws_bytes / (tail * tile_bytes))});
        if (s >= 2) {
            ta.main_tiles = ta.total_tiles - tail;
            ta.meet_splits = (int)s;
            ta.part = ws;
        }
    }
    int64_t blocks;
    if (ta.meet_splits > 1) {
        const int64_t nt = (ta.total_tiles - ta.main_tiles) * ta.meet_splits;
        blocks = (ta.main_tiles / NUM_XCD + (nt + NUM_XCD - 1) / NUM_XCD) * NUM_XCD;
    } else {
        blocks = (ta.total_tiles * ta.splits + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    }
    if (blocks > 0x7fffffffll) throw KernelError("conv: too many tiles");
    dim3 grid((unsigned)blocks, 1, (unsigned)zdim);
    if constexpr (TAG != 0) {
        if (!fast) throw KernelError("conv: batched GEMMs need aligned shapes");
        hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, 1, TAG>), grid, dim3(NT), 0, st, ta);
    } else {
        // a forward or input-gradient reduction that is no multiple of 16 (the host admits that for 1x1 layers only)
        const bool part = MODE == FWD ? ta.cs.C % BK != 0 : MODE == DGRAD ? ta.cs.K % BK != 0 : false;
        if constexpr (MODE != WGRAD) {
            if (fast && part) { hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, 2>), grid, dim3(NT), 0, st, ta); }
            else if (fast) { hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, 1>), grid, dim3(NT), 0, st, ta); }
            else { hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, 0>), grid, dim3(NT), 0, st, ta); }
        } else {
            if (fast) { hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, 1>), grid, dim3(NT), 0, st, ta); }
            else { hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, 0>), grid, dim3(NT), 0, st, ta); }
        }
    }
    hip_check(hipGetLastError(), "conv launch");
    if (slabs) launch_split_reduce(st, ws, out, ta.out_elems, splits, MODE != WGRAD && accumulate);
}

// Tile shapes: index -> waves (rows x columns of 64x64 wave tiles)
//   0: 128x128   1: 256x64   2: 64x256   3: 128x64   4: 64x128   5: 64x64
int g_cfg_override = -1;   // tuning aid: force one tile shape for every launch

// Choice measured on the ResNet-50 b184 layer set: the square four-wave tile unless the GEMM is
// narrower than it, then the four-wave (or smaller) tile that covers the narrow side exactly.
int pick_cfg(int mode, int64_t Mg, int64_t Ng) {
    if (g_cfg_override >= 0) return g_cfg_override;
    if (mode == WGRAD) {
        if (Mg <= 64) return Ng % 256 == 0 ? 2 : 5;
        if (Ng <= 64) return Mg >= 256 ? 1 : 3;
        return 0;
    }
    return Ng <= 64 ? 1 : 0;
}

template <int MODE, class... Rest>
void launch_cfg(int cfg, Rest... rest) {
    switch (cfg) {
        case 0: launch_tile<MODE, 2, 2>(rest...); break;
        case 1: launch_tile<MODE, 4, 1>(rest...); break;
        case 2: launch_tile<MODE, 1, 4>(rest...); break;
        case 3: launch_tile<MODE, 2, 1>(rest...); break;
        case 4: launch_tile<MODE, 1, 2>(rest...); break;
        default: launch_tile<MODE, 1, 1>(rest...); break;
    }
}

// the batched GEMMs only ever see the two tile shapes the forward heuristic picks
template <int TAG, class... Rest>
void launch_batched(int cfg, Rest... rest) {
    if (cfg == 1) launch_tile<FWD, 4, 1, TAG>(rest...);
    else launch_tile<FWD, 2, 2, TAG>(rest...);
}

}  // namespace

void conv_force_tile(int cfg) { g_cfg_override = cfg; }

// reduction steps of 16 must not straddle filter taps: C % 16 == 0, or a 1x1 layer (one tap) with C % 4 == 0, whose last
// step is partly empty
bool conv_fwd_aligned(const ConvShape &cs) { return cs.C % BK == 0 || (cs.R == 1 && cs.S == 1 && cs.C % 4 == 0); }

bool conv_epilogue_writes_mask(const ConvShape &cs, bool winograd_fused) {
    (void)winograd_fused;      // both forms: a word of the code is 64 consecutive channels of one position
    return cs.K % 64 == 0;
}

void split_reduce(hipStream_t st, const float *ws, float *out, int64_t n, int splits, bool accumulate) {
    launch_split_reduce(st, ws, out, n, splits, accumulate);
}

namespace {
struct SplitGemm { int64_t rows, cols, steps; int classes; };
SplitGemm split_gemm_of(int which, const ConvShape &cs) {
    if (which == 0) return {cs.M(), cs.K, (cs.RSC() + BK - 1) / BK, 1};
    const int st = cs.stride;
    return {(int64_t)cs.N * ((cs.H + st - 1) / st) * ((cs.W + st - 1) / st), cs.C,
            ((int64_t)std::max(1, cs.R / st) * std::max(1, cs.S / st) * cs.K + BK - 1) / BK, st * st};
}
}  // namespace

void conv_reset_arrivals(hipStream_t st) {
    hipLaunchKernelGGL(meet_reset_kernel, dim3(MEET_SLOTS / 256), dim3(256), 0, st);
    hip_check(hipGetLastError(), "arrival table reset launch");
}

size_t conv_workspace_bytes(int which, const ConvShape &cs, int splits) {
    check_shape(cs);
    const SplitGemm sg = split_gemm_of(which, cs);
    if (splits > sg.steps) splits = (int)std::max<int64_t>(sg.steps, 1);
    if (splits > 1) return (size_t)splits * 4 * (which == 0 ? cs.M() * cs.K : (int64_t)cs.N * cs.H * cs.W * cs.C);
    static const int shape[6][2] = {{128, 128}, {256, 64}, {64, 256}, {128, 64}, {64, 128}, {64, 64}};
    const int cfg = pick_cfg(FWD, sg.rows, sg.cols);
    const int64_t bm = shape[cfg][0], bn = shape[cfg][1];
    const int64_t tiles = ((sg.rows + bm - 1) / bm) * ((sg.cols + bn - 1) / bn);
    const int64_t tail = tiles % NUM_CU;
    if (sg.classes != 1 || tail == 0) return 0;
    const int64_t s = std::min<int64_t>({NUM_CU / tail, sg.steps / 4, 16});
    return s >= 2 ? (size_t)(s * tail * bm * bn * 4) : 0;
}

namespace {
}  // namespace

void gemm_batched(hipStream_t st, const float *a, const float *b, float *out, int batch, int64_t rows, int cols, int red, bool adjoint_use) {
    if (batch < 1 || rows < 1 || cols < 1 || red < 1 || red % BK || cols % 4) throw KernelError("gemm_batched: bad shape");
    // the aligned loader addresses each operand plane with 32-bit byte offsets
    if (rows * red * 4 >= ((int64_t)1 << 32) - (1 << 20) || (int64_t)cols * red * 4 >= ((int64_t)1 << 32) - (1 << 20))
        throw KernelError("gemm_batched: an operand plane of 4 GiB or more");
    ConvShape cs{1, 1, (int)rows, red, cols, 1, 1, 1, 0, 1, (int)rows};
    check_shape(cs);
    TileArgs ta{};
    ta.a = a; ta.b = b; ta.cs = cs;
    ta.Mg = rows; ta.Ng = cols; ta.Kg = red;
    ta.out_elems = rows * cols;
    ta.batch_a = rows * red; ta.batch_b = (int64_t)cols * red; ta.batch_out = rows * cols;
    const int cfg = cols <= 64 ? 1 : 0;
    if (adjoint_use) launch_batched<2>(cfg, st, ta, true, batch, out, 1, (float *)nullptr, (size_t)0, (int64_t)red / BK, false, "gemm_batched");
    else launch_batched<1>(cfg, st, ta, true, batch, out, 1, (float *)nullptr, (size_t)0, (int64_t)red / BK, false, "gemm_batched");
}

// out[z][m][n] = sum_t a[z][t][m] b[z][t][n]: the reduction runs over the rows of both operands (weight-gradient form);
// `splits` partial results per GEMM go to ws (splits * batch * m * n floats) and are added in range order
void gemm_tn_batched(hipStream_t st, const float *a, const float *b, float *out, int batch, int64_t red, int m, int n, int splits,
                     float *ws, size_t ws_bytes) {
    if (batch < 1 || red < 1 || m < 1 || n < 1 || m % 4 || n % 4) throw KernelError("gemm_tn_batched: bad shape");
    ConvShape cs{1, 1, (int)red, n, m, 1, 1, 1, 0, 1, (int)red};
    check_shape(cs);
    TileArgs ta{};
    ta.a = a; ta.b = b; ta.cs = cs;
    ta.Mg = m; ta.Ng = n; ta.Kg = red;
    ta.out_elems = (int64_t)batch * m * n;
    ta.batch_a = red * m; ta.batch_b = red * n; ta.batch_out = (int64_t)m * n;
    // the aligned loader addresses each operand plane with 32-bit byte offsets
    if (red * m * 4 >= ((int64_t)1 << 32) - (1 << 20) || red * n * 4 >= ((int64_t)1 << 32) - (1 << 20))
        throw KernelError("gemm_tn_batched: an operand plane of 4 GiB or more");
    launch_tile<WGRAD, 2, 2, 3>(st, ta, true, batch, out, splits, ws, ws_bytes, (red + BK - 1) / BK, false, "gemm_tn_batched");
}

void conv_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs, int splits, float *ws, size_t ws_bytes,
              bool accumulate, float *stats_part, const BnAffine *affine) {
    check_shape(cs);
    // first layers (three input channels): input rows staged in LDS as they lie in memory (stem.hip)
    if (g_cfg_override < 0 && splits == 1 && !accumulate && !stats_part && !affine && stem_applies(cs)) {
        stem_fwd(st, x, w, y, cs);
        return;
    }
    TileArgs ta{};
    ta.a = x; ta.b = w; ta.cs = cs;
    ta.Mg = cs.M(); ta.Ng = cs.K; ta.Kg = cs.RSC();
    ta.out_elems = ta.Mg * ta.Ng;
    // the aligned loader addresses both operands with 32-bit byte offsets (plus one tap's reach) and keeps one bit per filter tap
    const int64_t span32 = ((int64_t)1 << 32) - (1 << 20);
    const int64_t reach = ((int64_t)(cs.R + cs.pad) * cs.W + cs.S + cs.pad) * cs.C * 4;
    bool fast = conv_fwd_aligned(cs) && cs.R * cs.S <= 32 && (int64_t)cs.N * cs.H * cs.W * cs.C * 4 + reach < span32 && cs.K * cs.RSC() * 4 < span32;
    if ((stats_part || affine) && (!fast || cs.K % 4 || splits != 1 || accumulate))
        throw KernelError("conv_fwd: statistics or BatchNorm in the epilogue need C % 16 == 0 (1x1: C % 4 == 0), K % 4 == 0, splits == 1 and no accumulation");
    if (stats_part && affine) throw KernelError("conv_fwd: either the statistics of the output or its BatchNorm apply step, not both");
    if (affine && (!affine->gamma || !affine->beta || !affine->stats)) throw KernelError("conv_fwd: incomplete BatchNorm coefficients");
    if (affine && affine->mask && (!affine->relu || cs.K % 64)) throw KernelError("conv_fwd: a sign code in the epilogue needs the ReLU and K % 64 == 0");
    ta.stats_part = stats_part;
    if (affine) ta.affine = *affine;
    launch_cfg<FWD>(pick_cfg(FWD, ta.Mg, ta.Ng), st, ta, fast, 1, y, splits, ws, ws_bytes, (ta.Kg + BK - 1) / BK, accumulate, "conv_fwd");
}

void conv_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, const ConvShape &cs, bool accumulate, int splits, float *ws,
                size_t ws_bytes) {
    check_shape(cs);
    TileArgs ta{};
    ta.a = dy; ta.b = w; ta.cs = cs;
    const SplitGemm sg = split_gemm_of(1, cs);   // rows of residue class (0,0), the largest; the shortest class reduction bounds the splits
    ta.Mg = sg.rows;
    ta.Ng = cs.C;
    ta.Kg = 0;   // per class, computed in the kernel
    ta.out_elems = (int64_t)cs.N * cs.H * cs.W * cs.C;
    const int64_t span32 = ((int64_t)1 << 32) - (1 << 20);
    const int64_t reach = ((int64_t)cs.R * cs.Q + cs.S) * cs.K * 4;
    // reduction steps of 16 must not straddle filter taps: K % 16 == 0, or a 1x1 layer (one tap) with K % 4 == 0, whose last
    // step is partly empty
    const bool k_ok = cs.K % BK == 0 || (cs.R == 1 && cs.S == 1 && cs.K % 4 == 0);
    bool fast = k_ok && cs.C % 4 == 0 && cs.R * cs.S <= 32 && cs.M() * cs.K * 4 + reach < span32 && cs.K * cs.RSC() * 4 < span32;
    launch_cfg<DGRAD>(pick_cfg(DGRAD, ta.Mg, ta.Ng), st, ta, fast, sg.classes, dx, splits, ws, ws_bytes, sg.steps, accumulate, "conv_dgrad");
}

void conv_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws, size_t ws_bytes) {
    check_shape(cs);
    // first layers (three input channels): input rows staged in LDS as they lie in memory (stem.hip)
    if (g_cfg_override < 0 && ws && stem_wgrad_applies(cs, splits, ws_bytes)) {
        stem_wgrad(st, x, dy, dw, cs, splits, ws, ws_bytes);
        return;
    }
    // 1x1 layers with at most 32 channels on one side: streamed straight into the matrix instruction (pointwise.hip)
    if (g_cfg_override < 0 && ws && pointwise_wgrad_applies(cs, splits, ws_bytes)) {
        pointwise_wgrad(st, x, dy, dw, cs, splits, ws, ws_bytes);
        return;
    }
    TileArgs ta{};
    ta.a = dy; ta.b = x; ta.cs = cs;
    ta.Mg = cs.K; ta.Ng = (int)cs.RSC(); ta.Kg = cs.M();
    ta.out_elems = (int64_t)cs.K * cs.RSC();
    // the aligned loader addresses both operands with 32-bit byte offsets and keeps one bit per filter tap
    const int64_t span32 = ((int64_t)1 << 32) - (1 << 20);
    const int64_t lead = ((int64_t)cs.pad * cs.W + cs.pad) * cs.C * 4;
    bool fast = cs.K % 4 == 0 && cs.C % 4 == 0 && cs.R * cs.S <= 32 && cs.M() * cs.K * 4 < span32 &&
                (int64_t)cs.N * cs.H * cs.W * cs.C * 4 + lead < span32;
    launch_cfg<WGRAD>(pick_cfg(WGRAD, ta.Mg, ta.Ng), st, ta, fast, 1, dw, splits, ws, ws_bytes, (ta.Kg + BK - 1) / BK, false, "conv_wgrad");
}

}  // namespace monet
