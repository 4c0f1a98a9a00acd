// First layers: convolutions of a three-channel image (7x7 / stride 2, 3x3 / stride 1 or 2).  With C = 3 a reduction
// step of the tile kernel in conv.hip straddles filter taps, so its loader goes element by element (46-56 TFLOP/s on the
// ResNet-50 stem).  Here the input rows a tile of output positions needs are copied to LDS once, as they lie in memory
// (N,H,W,3: the S taps of a filter row are S*3 consecutive floats), and the matrix instruction's operand is read from
// there directly:
//
//   y[m][k] = sum_r sum_j  x_row(m, r)[j] * w[k][r][j],   j = 3 s + c in [0, 3 S),
//   x_row(m, r) = LDS row (pr * ST + r), starting at column (qq * ST) * 3        (m = (pr, qq) inside the tile)
//
// so consecutive output positions are ST*3 floats apart in LDS and no patch matrix is ever formed.  The reduction of a
// filter row is padded from 3 S to the next even number (the matrix instruction takes two reduction indices; the filter
// value of the padding is zero, its input value a float of the position's own window read a second time).
//
// Forward: mfma_f32_32x32x2f32 with A = positions x reduction (lane (m, h) reads LDS[off(m) + r * rowlen + 2 t + h]),
// B = the filters of 32 output channels, resident in registers for the whole launch (R * ceil(3 S / 2) values per lane).
// A wave takes four blocks of 32 consecutive positions and 32 output channels; a workgroup (K / 32 waves per group of
// four blocks, at most four waves) one tile of up to 224 positions: whole output rows if they fit, else a segment of
// one row.  Workgroups loop over tiles.
//
// Filter gradient: dw[k][r][j] = sum_m dy[m][k] * x_row(m, r)[j]: A = dy (positions are the reduction index now, read
// from memory in the instruction's layout: lane (k, h) loads dy[m + h][k]), B = lane (col, h) reads
// LDS[off(m + h) + r(col) * rowlen + j(col)] with col = (r, j) flattened.  Wave kb of a workgroup owns the 32 output
// channels 32 kb .. 32 kb + 31 and all R * 3 S columns; the workgroups' partial results are added in a fixed order by
// split_reduce.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "buffer_addr.hpp"
#include "kernels.hpp"

namespace monet {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct StemGeom {
    int N, H, W, P, Q, K, pad;
    int nrow, qn;            // tile: nrow output rows x qn output columns (qn == Q, or nrow == 1)
    int row_tiles, col_tiles;
    int64_t tiles;           // N * row_tiles * col_tiles
    int rows_in;             // input rows under a tile: (nrow - 1) * ST + R
    int rowlen;              // floats per LDS row (multiple of 4)
    int xlead;               // LDS column of the tile's first input float (the float (q0 * ST - pad) * 3 of an image row)
};

// Copies the input rows under tile (n, p0, q0) to LDS, zero where the image ends, in two steps: the loads into registers
// (piece tid + k * nthreads of the tile's rows_in x rowlen / 4 pieces of 16 bytes, k < FILL: the host checks that this
// covers the tile) and the LDS writes, so that other work can be issued between the two.  LDS column e of row ri holds
// float fbase + e of image row h0 + ri, fbase = (q0 * ST - pad) * 3 - xlead (a multiple of 4 whenever W is one, so that
// the 16-byte pieces stay aligned).
constexpr int FILL = 8;
template <int ST>
__device__ __forceinline__ void stem_fill_load(float4 (&v)[FILL], const float *__restrict__ x, const StemGeom &gm, int n, int p0, int q0, int tid,
                                               int nthreads, int k0 = 0) {
    const int row4 = gm.rowlen / 4, rowf = gm.W * 3;
    const int h0 = p0 * ST - gm.pad, fbase = (q0 * ST - gm.pad) * 3 - gm.xlead;
    const bool aligned = (gm.W & 3) == 0 && (fbase & 3) == 0 && ((uintptr_t)x & 15) == 0;
    const float *img = x + (int64_t)n * gm.H * rowf;
    const int first = tid + k0 * nthreads;      // pieces first + k * nthreads, k < FILL
    int ri = first / row4, e4 = first - ri * row4;
    const int dr = nthreads / row4, de = nthreads - dr * row4;
#pragma unroll
    for (int k = 0; k < FILL; ++k) {
        v[k] = make_float4(0, 0, 0, 0);
        const int h = h0 + ri, f = fbase + 4 * e4;
        if (ri < gm.rows_in && (unsigned)h < (unsigned)gm.H) {
            const float *src = img + (int64_t)h * rowf;
            if (aligned && f >= 0 && f + 3 < rowf) v[k] = *(const float4 *)(src + f);
            else {
                if ((unsigned)f < (unsigned)rowf) v[k].x = src[f];
                if ((unsigned)(f + 1) < (unsigned)rowf) v[k].y = src[f + 1];
                if ((unsigned)(f + 2) < (unsigned)rowf) v[k].z = src[f + 2];
                if ((unsigned)(f + 3) < (unsigned)rowf) v[k].w = src[f + 3];
            }
        }
        ri += dr; e4 += de;
        if (e4 >= row4) { e4 -= row4; ++ri; }
    }
}
__device__ __forceinline__ void stem_fill_write(float *lds, const float4 (&v)[FILL], const StemGeom &gm, int tid, int nthreads, int k0 = 0) {
    const int total = gm.rows_in * (gm.rowlen / 4);
#pragma unroll
    for (int k = 0; k < FILL; ++k) {
        const int idx = tid + (k0 + k) * nthreads;
        if (idx < total) *(float4 *)&lds[4 * idx] = v[k];
    }
}

__device__ __forceinline__ void tile_origin(const StemGeom &gm, int64_t tile, int &n, int &p0, int &q0) {
    const int per_img = gm.row_tiles * gm.col_tiles;
    n = (int)(tile / per_img);
    const int t = (int)(tile - (int64_t)n * per_img);
    p0 = (t / gm.col_tiles) * gm.nrow;
    q0 = (t % gm.col_tiles) * gm.qn;
}

template <int R, int S, int ST>
__global__ __launch_bounds__(256, 2) void stem_fwd_kernel(const float *__restrict__ x, const float *__restrict__ w, float *__restrict__ y, StemGeom gm) {
    extern __shared__ float lds[];
    constexpr int RUN = 3 * S, KP = (RUN + 1) / 2, MBW = 4;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nb = wave % (gm.K / 32);      // this wave's block of 32 output channels ...
    const int mg = wave / (gm.K / 32);      // ... and group of MBW position blocks
    const int nthreads = blockDim.x;
    // filters of channel 32 nb + l32: w[k][r][2 t + h], zero beyond the row's 3 S values
    float wr[R][KP];
    {
        const float *wk = w + (int64_t)(nb * 32 + l32) * (R * RUN);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < KP; ++t) wr[r][t] = 2 * t + h < RUN ? wk[r * RUN + 2 * t + h] : 0.0f;
    }
    // LDS offset of this lane's position in every block (position 32 b + l32 of the tile; positions beyond the tile read
    // position 0), plus h: the lane's share of a reduction pair
    int aoff[MBW];
#pragma unroll
    for (int b = 0; b < MBW; ++b) {
        int m = 32 * (MBW * mg + b) + l32;
        if (m >= gm.nrow * gm.qn) m = 0;
        const int pr = gm.nrow == 1 ? 0 : m / gm.qn, qq = m - pr * gm.qn;
        aoff[b] = pr * ST * gm.rowlen + qq * ST * 3 + gm.xlead + h;
    }
    float4 staged[FILL];
    if ((int64_t)blockIdx.x < gm.tiles) {
        int n, p0, q0;
        tile_origin(gm, blockIdx.x, n, p0, q0);
        stem_fill_load<ST>(staged, x, gm, n, p0, q0, tid, nthreads);
        stem_fill_write(lds, staged, gm, tid, nthreads);
    }
    __syncthreads();
    for (int64_t tile = blockIdx.x; tile < gm.tiles; tile += gridDim.x) {
        int n, p0, q0;
        tile_origin(gm, tile, n, p0, q0);
        // the compiler must not carry the addresses derived from these offsets (one per filter row and block) from tile to
        // tile in registers: they cost one addition each and there are more of them than registers to spare
#pragma unroll
        for (int b = 0; b < MBW; ++b) asm volatile("" : "+v"(aoff[b]));
        floatx16 acc[MBW];
#pragma unroll
        for (int b = 0; b < MBW; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
        // position blocks of the nominal tile this wave works on (the last group may hold fewer than MBW)
        const int nblk = min(MBW, (gm.nrow * gm.qn + 31) / 32 - MBW * mg);
        // one reduction pair ahead: the LDS reads of pair s + 1 are issued before the matrix instructions of pair s
        float a_cur[MBW], a_nxt[MBW];
        auto read_pair = [&](int r, int t, float (&a)[MBW]) {
            const float *row = lds + r * gm.rowlen + 2 * t;
#pragma unroll
            for (int b = 0; b < MBW; ++b) {
                // the padding slot of an odd row length (h = 1 of the last pair, filter value zero) reads the value of
                // h = 0 again: a float of this position's own window, so that nothing foreign can turn 0 * x into NaN
                a[b] = row[(RUN & 1) && t == KP - 1 ? aoff[b] - h : aoff[b]];
            }
        };
        read_pair(0, 0, a_cur);
#pragma unroll
        for (int s = 0; s < R * KP; ++s) {
            if (s + 1 < R * KP) read_pair((s + 1) / KP, (s + 1) % KP, a_nxt);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < MBW; ++b)
                if (b < nblk) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_cur[b], wr[s / KP][s % KP], acc[b], 0, 0, 0);      // uniform over the wave
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < MBW; ++b) a_cur[b] = a_nxt[b];
        }
        // The next tile's input is requested before this tile's results are stored and goes to LDS after them: its latency
        // passes while the stores are issued, and the stores drain while the next tile is computed (memory operations
        // complete in the order of issue, so waiting for these loads does not wait for the stores behind them).
        const int64_t next = tile + gridDim.x;
        if (next < gm.tiles) {      // uniform over the workgroup
            int n2, p2, q2;
            tile_origin(gm, next, n2, p2, q2);
            stem_fill_load<ST>(staged, x, gm, n2, p2, q2, tid, nthreads);
        }
        __builtin_amdgcn_sched_barrier(0);
        // positions of the tile are consecutive in y when the tile is whole rows or part of one row: position m lies m * K
        // floats behind the tile's first.  Buffer addressing: the lane's part of the offset (4 h rows, its channel) never
        // changes, the rest is the same for every lane.
        const int rows_here = min(gm.nrow, gm.P - p0), cols_here = min(gm.qn, gm.Q - q0);
        const int npos = gm.nrow == 1 ? cols_here : rows_here * gm.qn;
        const __amdgpu_buffer_rsrc_t ry = buffer_of(y + (((int64_t)n * gm.P + p0) * gm.Q + q0) * gm.K);
        const unsigned kbytes = (unsigned)gm.K * 4u;
        const unsigned voff = (unsigned)(32 * MBW * mg + 4 * h) * kbytes + (unsigned)(nb * 32 + l32) * 4u;
        if (npos >= 32 * (MBW * mg + nblk)) {      // uniform over the wave: every position of its blocks exists
#pragma unroll
            for (int b = 0; b < MBW; ++b)
                if (b < nblk) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) buffer_store(ry, voff, (unsigned)(32 * b + 8 * (i / 4) + (i % 4)) * kbytes, acc[b][i]);
                }
        } else {
#pragma unroll
            for (int b = 0; b < MBW; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int m = 32 * (MBW * mg + b) + 8 * (i / 4) + 4 * h + (i % 4);
                    if (b < nblk && m < npos) buffer_store(ry, voff, (unsigned)(32 * b + 8 * (i / 4) + (i % 4)) * kbytes, acc[b][i]);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();      // every wave has read this tile from LDS
        if (next < gm.tiles) stem_fill_write(lds, staged, gm, tid, nthreads);
        __syncthreads();
    }
}

// Filter gradient: a workgroup of K / 32 waves walks tiles like the forward kernel; wave kb keeps the 32 x (R * 3 S)
// block of dw of its output channels in registers (NBC column blocks of 32) over all its tiles and leaves it in
// part[workgroup] at the end.
template <int R, int S, int ST>
__global__ __launch_bounds__(256, 2) void stem_wgrad_kernel(const float *__restrict__ x, const float *__restrict__ dy, float *__restrict__ part, StemGeom gm) {
    extern __shared__ float lds[];
    constexpr int RUN = 3 * S, COLS = R * RUN, NBC = (COLS + 31) / 32, U = NBC >= 4 ? 8 : 16;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const int kb = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x;
    // LDS offset of this lane's column (r, j) in every column block relative to a position's window; a column beyond
    // R * 3 S reads the window's first float into a result column that is never written
    int coloff[NBC];
#pragma unroll
    for (int c = 0; c < NBC; ++c) {
        int col = 32 * c + l32;
        if (col >= COLS) col = 0;
        coloff[c] = (col / RUN) * gm.rowlen + col % RUN;
    }
    floatx16 acc[NBC];
#pragma unroll
    for (int c = 0; c < NBC; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.0f;
    const int total4 = gm.rows_in * (gm.rowlen / 4);
    for (int64_t tile = blockIdx.x; tile < gm.tiles; tile += gridDim.x) {
        int n, p0, q0;
        tile_origin(gm, tile, n, p0, q0);
        __syncthreads();      // the previous tile has been read
        for (int k0 = 0; k0 * nthreads < total4; k0 += FILL) {
            float4 staged[FILL];
            stem_fill_load<ST>(staged, x, gm, n, p0, q0, tid, nthreads, k0);
            stem_fill_write(lds, staged, gm, tid, nthreads, k0);
        }
        __syncthreads();
        const int rows_here = min(gm.nrow, gm.P - p0), cols_here = min(gm.qn, gm.Q - q0);
        const int npos = gm.nrow == 1 ? cols_here : rows_here * gm.qn;      // positions of the tile that exist: m * K floats apart in dy
        const __amdgpu_buffer_rsrc_t rdy = buffer_of(dy + (((int64_t)n * gm.P + p0) * gm.Q + q0) * gm.K);
        const unsigned kbytes = (unsigned)gm.K * 4u, lbytes = (unsigned)(kb * 32 + l32) * 4u;
        // groups of U position pairs, two register sets: the dy loads of the next group are issued before the matrix
        // instructions of the current one.  A position beyond the tile contributes zero (its window in LDS is finite).
        struct Set { float a[U]; int po[U]; };
        auto load = [&](Set &t, int m0) {      // pairs (m0 + 2 u, m0 + 2 u + 1), this lane takes position m0 + 2 u + h
            int m = m0 + h;
            int pr = gm.nrow == 1 ? 0 : m / gm.qn, qq = m - pr * gm.qn;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float got = buffer_load(rdy, (m < npos ? (unsigned)m * kbytes : 0u) + lbytes, 0u);      // in bounds either way
                t.a[u] = m < npos ? got : 0.0f;
                const bool in = pr < gm.nrow;      // a nominal position: its window lies in the staged rows
                t.po[u] = in ? pr * ST * gm.rowlen + qq * ST * 3 + gm.xlead : gm.xlead;
                m += 2; qq += 2;
                if (qq >= gm.qn) { qq -= gm.qn; ++pr; }
            }
        };
        auto compute = [&](const Set &t) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < NBC; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(t.a[u], lds[t.po[u] + coloff[c]], acc[c], 0, 0, 0);
        };
        const int groups = (npos + 2 * U - 1) / (2 * U);
        Set s0, s1;
        if (groups > 0) load(s0, 0);
        for (int g = 0; g < groups; g += 2) {
            if (g + 1 < groups) load(s1, (g + 1) * 2 * U);
            __builtin_amdgcn_sched_barrier(0);
            compute(s0);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 2 < groups) load(s0, (g + 2) * 2 * U);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 1 < groups) compute(s1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // this workgroup's partial result, laid out as dw[k][r][s][c]: lane holds column l32 of rows 8 (i / 4) + 4 h + i % 4
    float *mine = part + (int64_t)blockIdx.x * gm.K * COLS;
#pragma unroll
    for (int c = 0; c < NBC; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = kb * 32 + 8 * (i / 4) + 4 * h + (i % 4), col = 32 * c + l32;
            if (col < COLS) mine[row * COLS + col] = acc[c][i];
        }
}

struct StemPlan { bool ok; int R, S, ST, mbw; StemGeom gm; size_t lds_bytes; };

StemPlan stem_plan(const ConvShape &cs) {
    StemPlan sp{};
    if (cs.C != 3 || cs.R != cs.S || cs.K % 32 || cs.K < 32 || cs.K > 128) return sp;
    if (!((cs.R == 7 && cs.stride == 2) || (cs.R == 3 && (cs.stride == 1 || cs.stride == 2)))) return sp;
    if (cs.pad < 0 || cs.pad > cs.R || (int64_t)cs.N * cs.H * cs.W * 3 >= ((int64_t)1 << 31) || cs.M() * cs.K >= ((int64_t)1 << 40)) return sp;
    sp.R = cs.R; sp.S = cs.S; sp.ST = cs.stride;
    StemGeom &gm = sp.gm;
    gm.N = cs.N; gm.H = cs.H; gm.W = cs.W; gm.P = cs.P; gm.Q = cs.Q; gm.K = cs.K; gm.pad = cs.pad;
    // a tile: as many whole output rows as 224 positions hold (seven blocks of 32: two waves' worth), else segments of one
    // row; with 96 or 128 output channels one wave's worth, so that a workgroup stays within four waves
    const int cap = cs.K > 64 ? 128 : 224;
    if (cs.Q <= cap) { gm.nrow = std::max(1, std::min(cap / cs.Q, cs.P)); gm.qn = cs.Q; }
    else { gm.nrow = 1; gm.qn = cap; }
    const int blocks = (gm.nrow * gm.qn + 31) / 32;
    sp.mbw = (blocks + 3) / 4;      // groups of four position blocks, one wave each per 32 output channels
    if (sp.mbw * (cs.K / 32) > 4) return sp;
    gm.row_tiles = (cs.P + gm.nrow - 1) / gm.nrow;
    gm.col_tiles = (cs.Q + gm.qn - 1) / gm.qn;
    gm.tiles = (int64_t)cs.N * gm.row_tiles * gm.col_tiles;
    gm.rows_in = (gm.nrow - 1) * cs.stride + cs.R;
    gm.xlead = (4 - (cs.pad * 3) % 4) % 4;
    // floats of an LDS row: up to the last tap of the tile's last position, plus the reduction padding, rounded up
    const int need = gm.xlead + ((gm.qn - 1) * cs.stride + cs.S) * 3 + 2;
    gm.rowlen = (need + 3) / 4 * 4;
    sp.lds_bytes = (size_t)gm.rows_in * gm.rowlen * sizeof(float);
    if (sp.lds_bytes > 64 * 1024 || gm.rows_in * (gm.rowlen / 4) > FILL * 64 * (cs.K / 32) * sp.mbw) return sp;
    sp.ok = true;
    return sp;
}

template <int R, int S, int ST>
void launch_stem_fwd(hipStream_t st, const float *x, const float *w, float *y, const StemPlan &sp) {
    const unsigned block = 64u * (unsigned)(sp.gm.K / 32) * (unsigned)sp.mbw;
    // workgroups of a launch: each keeps its filters for all its tiles (measured on the ResNet-50, MobileNetV2 and VGG-16
    // first layers: 1024 workgroups at or near the best time, 256 and one per tile 10-25 % slower)
    const unsigned grid = (unsigned)std::min<int64_t>(sp.gm.tiles, 1024);
    hipLaunchKernelGGL((stem_fwd_kernel<R, S, ST>), dim3(grid), dim3(block), sp.lds_bytes, st, x, w, y, sp.gm);
    hip_check(hipGetLastError(), "stem_fwd launch");
}

// workgroups of the filter gradient: one partial result each, as many as the caller's split count allows
int stem_wgrad_groups(const StemPlan &sp, int splits) { return (int)std::min<int64_t>({(int64_t)splits, (int64_t)1024, sp.gm.tiles}); }

template <int R, int S, int ST>
void launch_stem_wgrad(hipStream_t st, const float *x, const float *dy, float *ws, const StemPlan &sp, int groups) {
    hipLaunchKernelGGL((stem_wgrad_kernel<R, S, ST>), dim3((unsigned)groups), dim3(64u * (unsigned)(sp.gm.K / 32)), sp.lds_bytes, st, x, dy, ws, sp.gm);
    hip_check(hipGetLastError(), "stem_wgrad launch");
}

}  // namespace

bool stem_applies(const ConvShape &cs) { return stem_plan(cs).ok; }

bool stem_wgrad_applies(const ConvShape &cs, int splits, size_t ws_bytes) {
    const StemPlan sp = stem_plan(cs);
    if (!sp.ok || splits < 2) return false;
    // the filter gradient fills LDS in rounds of FILL pieces per thread: any tile the forward plan accepts will do
    return ws_bytes >= (size_t)stem_wgrad_groups(sp, splits) * cs.K * cs.RSC() * sizeof(float);
}

void stem_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws, size_t ws_bytes) {
    if (!stem_wgrad_applies(cs, splits, ws_bytes)) throw KernelError("stem_wgrad: shape, split count or workspace not supported");
    const StemPlan sp = stem_plan(cs);
    const int groups = stem_wgrad_groups(sp, splits);
    if (sp.R == 7) launch_stem_wgrad<7, 7, 2>(st, x, dy, ws, sp, groups);
    else if (sp.ST == 2) launch_stem_wgrad<3, 3, 2>(st, x, dy, ws, sp, groups);
    else launch_stem_wgrad<3, 3, 1>(st, x, dy, ws, sp, groups);
    split_reduce(st, ws, dw, (int64_t)cs.K * cs.RSC(), groups, false);
}

void stem_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs) {
    const StemPlan sp = stem_plan(cs);
    if (!sp.ok) throw KernelError("stem_fwd: needs three input channels, a 7x7 / stride 2 or 3x3 / stride 1 or 2 filter and 32, 64, 96 or 128 output channels");
    if (sp.R == 7) launch_stem_fwd<7, 7, 2>(st, x, w, y, sp);
    else if (sp.ST == 2) launch_stem_fwd<3, 3, 2>(st, x, w, y, sp);
    else launch_stem_fwd<3, 3, 1>(st, x, w, y, sp);
}

}  // namespace monet
