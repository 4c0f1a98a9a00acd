// Bandwidth-bound kernels: ReLU forward with 1-bit sign packing (one ballot per 64
// elements), ReLU backward from input / output / packed mask, add, copy, fill, max-pool with
// an 8-bit window index, global average pool, losses.  The operator variants are the ones
// listed in the paper's Appendix D ("Operator optimizations").  NHWC, fp32, wave64.
#include "kernels.hpp"

namespace monet {

static inline int grid_for(int64_t work_items, int per_block, int cap = 1 << 16) {
    int64_t g = (work_items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

// ------------------------------------------------------------------ ReLU forward (+ mask)
// Each wave walks chunks of 64*U consecutive elements; lane l takes elements l, 64+l, ...
// so that one ballot is exactly one mask word.  y may alias x.
template <int U, bool SIX, bool MASK>
__global__ __launch_bounds__(256) void relu_fwd_kernel(const float *x, float *y, uint64_t *__restrict__ mask,
                                                       int64_t n) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    const int64_t chunk = 64 * U;
    const int64_t nchunks = (n + chunk - 1) / chunk;
    for (int64_t ch = wave; ch < nchunks; ch += nwaves) {
        const int64_t base = ch * chunk;
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t e = base + u * 64 + lane;
            v[u] = e < n ? x[e] : 0.0f;
        }
        uint64_t mine = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            bool pass = SIX ? (v[u] > 0.0f && v[u] < 6.0f) : (v[u] > 0.0f);
            if (MASK) {
                uint64_t b = __ballot(pass);
                if (lane == u) mine = b;
            }
            float r = v[u] > 0.0f ? v[u] : 0.0f;       // NaN and -0.0 map to +0.0
            if (SIX) r = r < 6.0f ? r : 6.0f;
            int64_t e = base + u * 64 + lane;
            if (e < n) y[e] = r;
        }
        if (MASK && lane < U) {
            int64_t w = base / 64 + lane;
            if (w * 64 < n) mask[w] = mine;
        }
    }
}

void relu_fwd(hipStream_t st, const float *x, float *y, uint64_t *mask, int64_t n, bool six) {
    if (n <= 0) return;
    // whole float4s: the 16-byte streaming kernel (same predicate, same mask words); this one takes the rest
    if (n % 4 == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)y % 16) == 0) {
        fwd_chain(st, x, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr, y, mask, n, six);
        return;
    }
    constexpr int U = 8;
    int grid = grid_for(n, 256 * U, 16384);
#define RL(SIX, MASK) hipLaunchKernelGGL((relu_fwd_kernel<U, SIX, MASK>), dim3(grid), dim3(256), 0, st, x, y, mask, n)
    if (six) { if (mask) RL(true, true); else RL(true, false); }
    else     { if (mask) RL(false, true); else RL(false, false); }
#undef RL
    hip_check(hipGetLastError(), "relu_fwd launch");
}

// ------------------------------------------------------------------ ReLU backward
template <int U, int MODE, bool SIX, bool ACC>
__global__ __launch_bounds__(256) void relu_bwd_kernel(const float *__restrict__ dz, const void *__restrict__ t, float *dx,
                                                       int64_t n) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    const int64_t chunk = 64 * U;
    const int64_t nchunks = (n + chunk - 1) / chunk;
    const float *tf = (const float *)t;
    const uint64_t *tm = (const uint64_t *)t;
    for (int64_t ch = wave; ch < nchunks; ch += nwaves) {
        const int64_t base = ch * chunk;
        float g[U], f[U], old[U];
        uint64_t word[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t e = base + u * 64 + lane;
            bool in = e < n;
            g[u] = in ? dz[e] : 0.0f;
            if (MODE == RELU_FROM_MASK) word[u] = (base + u * 64 < n) ? tm[base / 64 + u] : 0;
            else f[u] = in ? tf[e] : 0.0f;
            if (ACC) old[u] = in ? dx[e] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            bool pass;
            if (MODE == RELU_FROM_MASK) pass = (word[u] >> lane) & 1;
            else pass = SIX ? (f[u] > 0.0f && f[u] < 6.0f) : (f[u] > 0.0f);
            float r = pass ? g[u] : 0.0f;
            if (ACC) r += old[u];
            int64_t e = base + u * 64 + lane;
            if (e < n) dx[e] = r;
        }
    }
}

void relu_bwd(hipStream_t st, const float *dz, const void *t, int mode, float *dx, int64_t n, bool six, bool accumulate) {
    if (n <= 0) return;
    if (n % 4 == 0 && ((uintptr_t)dz % 16) == 0 && ((uintptr_t)dx % 16) == 0 && ((uintptr_t)t % 16) == 0 &&
        (mode == RELU_FROM_MASK || mode == RELU_FROM_INPUT || mode == RELU_FROM_OUTPUT)) {
        relu_bwd_fanout(st, dz, t, mode, dx, accumulate, nullptr, false, n, six);
        return;
    }
    constexpr int U = 8;
    int grid = grid_for(n, 256 * U, 16384);
#define RB(MODE, SIX, ACC) hipLaunchKernelGGL((relu_bwd_kernel<U, MODE, SIX, ACC>), dim3(grid), dim3(256), 0, st, dz, t, dx, n)
#define RB2(MODE)                                                      \
    do {                                                               \
        if (six) { if (accumulate) RB(MODE, true, true); else RB(MODE, true, false); }   \
        else     { if (accumulate) RB(MODE, false, true); else RB(MODE, false, false); } \
    } while (0)
    if (mode == RELU_FROM_MASK) RB2(RELU_FROM_MASK);
    else if (mode == RELU_FROM_INPUT) RB2(RELU_FROM_INPUT);
    else if (mode == RELU_FROM_OUTPUT) RB2(RELU_FROM_OUTPUT);
    else throw KernelError("relu_bwd: unknown mode");
#undef RB2
#undef RB
    hip_check(hipGetLastError(), "relu_bwd launch");
}

// ------------------------------------------------------------------ add / copy / fill
template <int OP>   // 0: y = a + b, 1: y = a, 2: y += a
__global__ __launch_bounds__(256) void ew_kernel(const float *__restrict__ a, const float *__restrict__ b, float *y, int64_t n) {
    // one contiguous range per workgroup, four 16-byte pieces per thread in flight, streaming loads and
    // stores (the measured fastest form of a plain copy on this chip: about 6 TB/s read + write at 1 GiB)
    typedef float f4 __attribute__((ext_vector_type(4)));
    constexpr int U = 4;
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t per = ((n4 + gridDim.x - 1) / gridDim.x + 255) / 256 * 256;
    const int64_t r0 = (int64_t)blockIdx.x * per;
    const int64_t r1 = r0 + per < n4 ? r0 + per : n4;
    for (int64_t base = r0 + threadIdx.x; base < r1; base += U * 256) {
        f4 va[U], vb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            if (i >= r1) continue;
            va[u] = __builtin_nontemporal_load((const f4 *)a + i);
            if (OP == 0) vb[u] = __builtin_nontemporal_load((const f4 *)b + i);
            if (OP == 2) vb[u] = __builtin_nontemporal_load((const f4 *)y + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            if (i >= r1) continue;
            f4 r = va[u];
            if (OP == 0) r = va[u] + vb[u];
            if (OP == 2) r = vb[u] + va[u];
            __builtin_nontemporal_store(r, (f4 *)y + i);
        }
    }
    for (int64_t i = n4 * 4 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (OP == 0) y[i] = a[i] + b[i];
        else if (OP == 1) y[i] = a[i];
        else y[i] += a[i];
    }
}

void add_fwd(hipStream_t st, const float *a, const float *b, float *y, int64_t n) {
    if (n <= 0) return;
    hipLaunchKernelGGL((ew_kernel<0>), dim3(grid_for(n, 8192, 65536)), dim3(256), 0, st, a, b, y, n);
    hip_check(hipGetLastError(), "add_fwd launch");
}

void copy_or_accumulate(hipStream_t st, const float *src, float *dst, int64_t n, bool accumulate) {
    if (n <= 0) return;
    int grid = grid_for(n, 8192, 65536);
    if (accumulate) hipLaunchKernelGGL((ew_kernel<2>), dim3(grid), dim3(256), 0, st, src, (const float *)nullptr, dst, n);
    else hipLaunchKernelGGL((ew_kernel<1>), dim3(grid), dim3(256), 0, st, src, (const float *)nullptr, dst, n);
    hip_check(hipGetLastError(), "copy launch");
}

__global__ __launch_bounds__(256) void fill_kernel(uint32_t *dst, int64_t n, uint32_t v) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = v;
}

void fill_u32(hipStream_t st, uint32_t *dst, int64_t n, uint32_t v) {
    if (n <= 0) return;
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n, 1024, 8192)), dim3(256), 0, st, dst, n, v);
    hip_check(hipGetLastError(), "fill launch");
}

void fill_f32(hipStream_t st, float *dst, int64_t n, float v) {
    uint32_t bits;
    __builtin_memcpy(&bits, &v, 4);
    fill_u32(st, (uint32_t *)dst, n, bits);
}

// ------------------------------------------------------------------ max pool
// One thread per output (n,p,q, 4 channels).  Index = r*k+s of the first maximum under a
// strict '>' scan; padded taps are never selected.
template <bool IDX>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                          uint8_t *__restrict__ idx, PoolShape ps) {
    const int C4 = ps.C / 4;
    const int64_t total = (int64_t)ps.N * ps.P * ps.Q * C4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int c4 = (int)(i % C4);
        int64_t pix = i / C4;
        int q = (int)(pix % ps.Q);
        int64_t t = pix / ps.Q;
        int p = (int)(t % ps.P);
        int n = (int)(t / ps.P);
        float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        int bi[4] = {0, 0, 0, 0};
        for (int r = 0; r < ps.k; ++r) {
            int h = p * ps.stride - ps.pad + r;
            if (h < 0 || h >= ps.H) continue;
            for (int s = 0; s < ps.k; ++s) {
                int w = q * ps.stride - ps.pad + s;
                if (w < 0 || w >= ps.W) continue;
                float4 v = ((const float4 *)x)[(((int64_t)n * ps.H + h) * ps.W + w) * C4 + c4];
                float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (vv[j] > best[j]) { best[j] = vv[j]; bi[j] = r * ps.k + s; }
            }
        }
        ((float4 *)y)[i] = make_float4(best[0], best[1], best[2], best[3]);
        if (IDX) ((uchar4 *)idx)[i] = make_uchar4((uint8_t)bi[0], (uint8_t)bi[1], (uint8_t)bi[2], (uint8_t)bi[3]);
    }
}

// 3x3 / stride 1 / pad 1 (the pool branch of an inception module) over row segments: one thread per (output row,
// segment of L consecutive outputs, four channels) loads the 3 x (L + 2) inputs under the segment once; every input
// serves up to three outputs from registers (4.5 loads per output at L = 4 instead of 9).  Taps are compared in the
// general kernel's order (row-major, strictly greater wins), so values and indices are the same bits.
template <int L, bool IDX>
__global__ __launch_bounds__(256) void maxpool3s1_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, uint8_t *__restrict__ idx,
                                                             int N, int H, int W, int C4, int segs, int64_t items) {
    // a contiguous share of the items per XCD (hardware deals workgroups to the 8 XCDs in turn; the grid is a multiple of
    // 8): the output rows that read the same input rows meet in one L2
    const int64_t i = ((int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) * 256 + threadIdx.x;
    if (i >= items) return;
    const int c4 = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int p = (int)(t % H);
    const int n = (int)(t / H);
    const int q0 = seg * L;
    const float4 *base = (const float4 *)x + (int64_t)n * H * W * C4 + c4;
    float4 v[3][L + 2];
    bool ok[3][L + 2];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int h = p - 1 + r;
#pragma unroll
        for (int c = 0; c < L + 2; ++c) {
            const int w = q0 - 1 + c;
            ok[r][c] = (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
            v[r][c] = base[ok[r][c] ? ((int64_t)h * W + w) * C4 : 0];
        }
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (q0 + j >= W) break;
        float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        int bi[4] = {0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) {
                if (!ok[r][j + sx]) continue;
                const float vv[4] = {v[r][j + sx].x, v[r][j + sx].y, v[r][j + sx].z, v[r][j + sx].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (vv[e] > best[e]) { best[e] = vv[e]; bi[e] = r * 3 + sx; }
            }
        const int64_t o = (((int64_t)n * H + p) * W + q0 + j) * C4 + c4;
        ((float4 *)y)[o] = make_float4(best[0], best[1], best[2], best[3]);
        if (IDX) ((uchar4 *)idx)[o] = make_uchar4((uint8_t)bi[0], (uint8_t)bi[1], (uint8_t)bi[2], (uint8_t)bi[3]);
    }
}

void maxpool_fwd(hipStream_t st, const float *x, float *y, uint8_t *idx, const PoolShape &ps) {
    if (ps.C % 4) throw KernelError("maxpool: C must be a multiple of 4");
    if (ps.k * ps.k > 255) throw KernelError("maxpool: window too large for an 8-bit index");
    int64_t total = (int64_t)ps.N * ps.P * ps.Q * (ps.C / 4);
    if (total <= 0) return;
    if (ps.k == 3 && ps.stride == 1 && ps.pad == 1 && ps.P == ps.H && ps.Q == ps.W) {
        constexpr int L = 4;
        const int segs = (ps.W + L - 1) / L;
        const int64_t items = (int64_t)ps.N * ps.H * segs * (ps.C / 4);
        if ((items + 255) / 256 >= 0x7ffffff0ll) throw KernelError("maxpool: too many work items");
        const dim3 g1((unsigned)(((items + 255) / 256 + 7) / 8 * 8)), blk(256);
        if (idx) hipLaunchKernelGGL((maxpool3s1_fwd_kernel<L, true>), g1, blk, 0, st, x, y, idx, ps.N, ps.H, ps.W, ps.C / 4, segs, items);
        else hipLaunchKernelGGL((maxpool3s1_fwd_kernel<L, false>), g1, blk, 0, st, x, y, idx, ps.N, ps.H, ps.W, ps.C / 4, segs, items);
        hip_check(hipGetLastError(), "maxpool_fwd launch");
        return;
    }
    int grid = grid_for(total, 256, 1 << 16);
    if (idx) hipLaunchKernelGGL((maxpool_fwd_kernel<true>), dim3(grid), dim3(256), 0, st, x, y, idx, ps);
    else hipLaunchKernelGGL((maxpool_fwd_kernel<false>), dim3(grid), dim3(256), 0, st, x, y, idx, ps);
    hip_check(hipGetLastError(), "maxpool_fwd launch");
}

// Gather form: one thread per input (n,h,w, 4 channels) sums the windows that selected it,
// in fixed (p,q) order -- no atomics, so the result is deterministic.
template <bool FROM_IDX, bool ACC>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                          const uint8_t *__restrict__ idx, float *dx, PoolShape ps) {
    const int C4 = ps.C / 4;
    const int64_t total = (int64_t)ps.N * ps.H * ps.W * C4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int c4 = (int)(i % C4);
        int64_t pix = i / C4;
        int w = (int)(pix % ps.W);
        int64_t t = pix / ps.W;
        int h = (int)(t % ps.H);
        int n = (int)(t / ps.H);
        float acc[4] = {0, 0, 0, 0};
        // windows p with p*stride - pad <= h <= p*stride - pad + k - 1
        int p_lo = h + ps.pad - ps.k + 1;
        p_lo = p_lo <= 0 ? 0 : (p_lo + ps.stride - 1) / ps.stride;
        int p_hi = (h + ps.pad) / ps.stride;
        if (p_hi > ps.P - 1) p_hi = ps.P - 1;
        int q_lo = w + ps.pad - ps.k + 1;
        q_lo = q_lo <= 0 ? 0 : (q_lo + ps.stride - 1) / ps.stride;
        int q_hi = (w + ps.pad) / ps.stride;
        if (q_hi > ps.Q - 1) q_hi = ps.Q - 1;
        for (int p = p_lo; p <= p_hi; ++p)
            for (int q = q_lo; q <= q_hi; ++q) {
                int64_t o = (((int64_t)n * ps.P + p) * ps.Q + q) * C4 + c4;
                int mine = (h - (p * ps.stride - ps.pad)) * ps.k + (w - (q * ps.stride - ps.pad));
                int sel[4];
                if (FROM_IDX) {
                    uchar4 ix = ((const uchar4 *)idx)[o];
                    sel[0] = ix.x; sel[1] = ix.y; sel[2] = ix.z; sel[3] = ix.w;
                } else {
                    float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                    sel[0] = sel[1] = sel[2] = sel[3] = 0;
                    for (int r = 0; r < ps.k; ++r) {
                        int hh = p * ps.stride - ps.pad + r;
                        if (hh < 0 || hh >= ps.H) continue;
                        for (int s = 0; s < ps.k; ++s) {
                            int ww = q * ps.stride - ps.pad + s;
                            if (ww < 0 || ww >= ps.W) continue;
                            float4 v = ((const float4 *)x)[(((int64_t)n * ps.H + hh) * ps.W + ww) * C4 + c4];
                            float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (vv[j] > best[j]) { best[j] = vv[j]; sel[j] = r * ps.k + s; }
                        }
                    }
                }
                float4 g = ((const float4 *)dy)[o];
                float gg[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (sel[j] == mine) acc[j] += gg[j];
            }
        float4 r = make_float4(acc[0], acc[1], acc[2], acc[3]);
        if (ACC) { float4 o = ((float4 *)dx)[i]; r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w; }
        ((float4 *)dx)[i] = r;
    }
}

// The same gather from the stored window index with window edge and stride known at compile time: the (at most
// ceil(K / STRIDE)^2) windows that contain a pixel are enumerated without divisions and all their loads are issued
// before the first use.  One thread per (pixel, four channels), one pass, no grid-stride loop.
template <int K, int STRIDE, bool ACC>
__global__ __launch_bounds__(256) void maxpool_bwd_idx_kernel(const float *__restrict__ dy, const uint8_t *__restrict__ idx, float *dx, PoolShape ps) {
    constexpr int CAND = (K + STRIDE - 1) / STRIDE;
    const int C4 = ps.C / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)ps.N * ps.H * ps.W * C4) return;
    const int c4 = (int)(i % C4);
    int64_t pix = i / C4;
    const int w = (int)(pix % ps.W);
    pix /= ps.W;
    const int h = (int)(pix % ps.H);
    const int n = (int)(pix / ps.H);
    const int p_hi = STRIDE == 1 ? h + ps.pad : (STRIDE == 2 ? (h + ps.pad) >> 1 : (h + ps.pad) / STRIDE);
    const int q_hi = STRIDE == 1 ? w + ps.pad : (STRIDE == 2 ? (w + ps.pad) >> 1 : (w + ps.pad) / STRIDE);
    float4 g[CAND][CAND];
    uchar4 ix[CAND][CAND];
    int mine[CAND][CAND];
#pragma unroll
    for (int a = 0; a < CAND; ++a)
#pragma unroll
        for (int b = 0; b < CAND; ++b) {
            const int p = p_hi - a, q = q_hi - b;
            const int r = h - (p * STRIDE - ps.pad), sx = w - (q * STRIDE - ps.pad);      // position inside window (p, q)
            const bool ok = p >= 0 && p < ps.P && q >= 0 && q < ps.Q && r < K && sx < K;
            const int64_t o = ok ? (((int64_t)n * ps.P + p) * ps.Q + q) * C4 + c4 : 0;
            g[a][b] = ((const float4 *)dy)[o];
            ix[a][b] = ((const uchar4 *)idx)[o];
            mine[a][b] = ok ? r * K + sx : -1;
        }
    // accumulate in the order of the general kernel: windows by ascending p, then ascending q
    float acc[4] = {0, 0, 0, 0};
#pragma unroll
    for (int a = CAND - 1; a >= 0; --a)
#pragma unroll
        for (int b = CAND - 1; b >= 0; --b) {
            const float gg[4] = {g[a][b].x, g[a][b].y, g[a][b].z, g[a][b].w};
            const int sel[4] = {ix[a][b].x, ix[a][b].y, ix[a][b].z, ix[a][b].w};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (sel[j] == mine[a][b]) acc[j] += gg[j];
        }
    float4 r = make_float4(acc[0], acc[1], acc[2], acc[3]);
    if (ACC) { float4 o = ((float4 *)dx)[i]; r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w; }
    ((float4 *)dx)[i] = r;
}

// 3x3 / stride 1 / pad 1 from the stored index over row segments, like the forward kernel: one thread per (input row, segment
// of L consecutive pixels, four channels) loads the 3 x (L + 2) windows that contain a pixel of the segment once (gradient and
// index); every window serves up to three pixels from registers (4.5 loads of each kind per pixel at L = 4 instead of 9).
// Windows are added in the general kernel's order (ascending p, then ascending q): the same bits.
template <int L, bool ACC>
__global__ __launch_bounds__(256) void maxpool3s1_bwd_kernel(const float *__restrict__ dy, const uint8_t *__restrict__ idx, float *dx,
                                                             int N, int H, int W, int C4, int segs, int64_t items) {
    // a contiguous share of the items per XCD (the grid is a multiple of 8): neighbouring rows read the same windows
    const int64_t i = ((int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) * 256 + threadIdx.x;
    if (i >= items) return;
    const int c4 = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    const int w0 = seg * L;
    const int64_t img = (int64_t)n * H * W * C4 + c4;
    float4 g[3][L + 2];
    uchar4 ix[3][L + 2];
    bool ok[3][L + 2];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const int p = h - 1 + a;
#pragma unroll
        for (int b = 0; b < L + 2; ++b) {
            const int q = w0 - 1 + b;
            ok[a][b] = (unsigned)p < (unsigned)H && (unsigned)q < (unsigned)W;
            const int64_t o = ok[a][b] ? img + ((int64_t)p * W + q) * C4 : 0;
            g[a][b] = ((const float4 *)dy)[o];
            ix[a][b] = ((const uchar4 *)idx)[o];
        }
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (w0 + j >= W) break;
        float acc[4] = {0, 0, 0, 0};
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = j; b < j + 3; ++b) {
                // pixel (h, w0 + j) inside window (p, q) = (h - 1 + a, w0 - 1 + b): row 2 - a, column j - b + 2
                const int mine = ok[a][b] ? (2 - a) * 3 + (j - b + 2) : -1;
                const float gg[4] = {g[a][b].x, g[a][b].y, g[a][b].z, g[a][b].w};
                const int sel[4] = {ix[a][b].x, ix[a][b].y, ix[a][b].z, ix[a][b].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (sel[e] == mine) acc[e] += gg[e];
            }
        const int64_t o = img + ((int64_t)h * W + w0 + j) * C4;
        float4 r = make_float4(acc[0], acc[1], acc[2], acc[3]);
        if (ACC) { const float4 was = ((const float4 *)dx)[o]; r.x += was.x; r.y += was.y; r.z += was.z; r.w += was.w; }
        ((float4 *)dx)[o] = r;
    }
}

// 3x3 / stride 1 / pad 1 from the pool's input (the standard variant: no index was kept) over row segments: one thread per
// (input row, segment of L consecutive pixels, four channels).  For each of the three window rows p = h - 1 .. h + 1 it
// loads the 3 x (L + 4) inputs under the L + 2 windows that touch the segment, finds each window's maximum once (the forward
// kernel's scan: row-major, strictly greater wins, taps outside the map skipped) and adds the window's gradient to the pixel
// it selected: 4.5 windows and 13.5 inputs loaded per pixel instead of 9 and 81.  Windows are added in the general
// kernel's order (ascending p, then ascending q): the same bits.
template <int L, bool ACC>
__global__ __launch_bounds__(256) void maxpool3s1_bwd_input_kernel(const float *__restrict__ dy, const float *__restrict__ x, float *dx,
                                                                   int N, int H, int W, int C4, int segs, int64_t items) {
    const int64_t i = ((int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) * 256 + threadIdx.x;      // a contiguous share per XCD
    if (i >= items) return;
    const int c4 = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    const int w0 = seg * L;
    const int64_t img = (int64_t)n * H * W * C4 + c4;
    float acc[L][4];
#pragma unroll
    for (int j = 0; j < L; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] = 0.0f;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const int p = h - 1 + a;
        if ((unsigned)p >= (unsigned)H) continue;      // no such window row (uniform over few lanes; nothing below is shared)
        float4 v[3][L + 4];
        bool in[3][L + 4];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int hh = p - 1 + r;
#pragma unroll
            for (int c = 0; c < L + 4; ++c) {
                const int ww = w0 - 2 + c;
                in[r][c] = (unsigned)hh < (unsigned)H && (unsigned)ww < (unsigned)W;
                v[r][c] = ((const float4 *)x)[in[r][c] ? img + ((int64_t)hh * W + ww) * C4 : 0];
            }
        }
        float4 g[L + 2];
        bool okq[L + 2];
#pragma unroll
        for (int b = 0; b < L + 2; ++b) {
            const int q = w0 - 1 + b;
            okq[b] = (unsigned)q < (unsigned)W;
            g[b] = ((const float4 *)dy)[okq[b] ? img + ((int64_t)p * W + q) * C4 : 0];
        }
#pragma unroll
        for (int b = 0; b < L + 2; ++b) {
            if (!okq[b]) continue;
            // window (p, q = w0 - 1 + b) covers columns q - 1 .. q + 1 = patch columns b .. b + 2
            float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            int sel[4] = {0, 0, 0, 0};
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int sx = 0; sx < 3; ++sx) {
                    if (!in[r][b + sx]) continue;
                    const float vv[4] = {v[r][b + sx].x, v[r][b + sx].y, v[r][b + sx].z, v[r][b + sx].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (vv[e] > best[e]) { best[e] = vv[e]; sel[e] = r * 3 + sx; }
                }
            const float gg[4] = {g[b].x, g[b].y, g[b].z, g[b].w};
            // pixel (h, w0 + j) sits at row 2 - a, column j - b + 2 of this window, for j = b - 2 .. b
#pragma unroll
            for (int j = 0; j < L; ++j) {
                if (j < b - 2 || j > b) continue;
                const int mine = (2 - a) * 3 + (j - b + 2);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (sel[e] == mine) acc[j][e] += gg[e];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (w0 + j >= W) break;
        const int64_t o = img + ((int64_t)h * W + w0 + j) * C4;
        float4 r = make_float4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
        if (ACC) { const float4 was = ((const float4 *)dx)[o]; r.x += was.x; r.y += was.y; r.z += was.z; r.w += was.w; }
        ((float4 *)dx)[o] = r;
    }
}

// 3x3 / stride 2 / pad 1 from the stored index over row segments of four pixels (w0 a multiple of 4): the pixels lie in the
// window rows p = (h + 1) / 2 - 1 (odd h only) and (h + 1) / 2 and in the windows q = w0 / 2 .. w0 / 2 + 2, whose gradients
// and indices are loaded once (1.5 loads of each kind per pixel instead of 4).  Windows are added in the general kernel's
// order (ascending p, then ascending q): the same bits.
template <bool ACC>
__global__ __launch_bounds__(256) void maxpool3s2_bwd_idx_kernel(const float *__restrict__ dy, const uint8_t *__restrict__ idx, float *dx,
                                                                 int N, int H, int W, int P, int Q, int C4, int segs, int64_t items) {
    constexpr int L = 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= items) return;
    const int c4 = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    const int w0 = seg * L, q0 = w0 >> 1;
    const int64_t gimg = (int64_t)n * P * Q * C4 + c4;
    float4 g[2][3];
    uchar4 ix[2][3];
    int row[2];
    bool ok[2][3];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int p = ((h + 1) >> 1) - 1 + a;
        row[a] = h - 2 * p + 1;                  // of pixel row h inside window row p
        const bool pok = (unsigned)p < (unsigned)P && row[a] <= 2;
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            ok[a][b] = pok && q0 + b < Q;
            const int64_t o = ok[a][b] ? gimg + ((int64_t)p * Q + q0 + b) * C4 : 0;
            g[a][b] = ((const float4 *)dy)[o];
            ix[a][b] = ((const uchar4 *)idx)[o];
        }
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (w0 + j >= W) break;
        float acc[4] = {0, 0, 0, 0};
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                if (j < 2 * b - 1 || j > 2 * b + 1) continue;      // pixel w0 + j sits at column j - 2 b + 1 of window q0 + b
                const int mine = ok[a][b] ? row[a] * 3 + (j - 2 * b + 1) : -1;
                const float gg[4] = {g[a][b].x, g[a][b].y, g[a][b].z, g[a][b].w};
                const int sel[4] = {ix[a][b].x, ix[a][b].y, ix[a][b].z, ix[a][b].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (sel[e] == mine) acc[e] += gg[e];
            }
        const int64_t o = ((int64_t)n * H * W + (int64_t)h * W + w0 + j) * C4 + c4;
        float4 r = make_float4(acc[0], acc[1], acc[2], acc[3]);
        if (ACC) { const float4 was = ((const float4 *)dx)[o]; r.x += was.x; r.y += was.y; r.z += was.z; r.w += was.w; }
        ((float4 *)dx)[o] = r;
    }
}

// The same for 3x3 / stride 2 / pad 1 (the pool behind a network's first layer): a pixel row h lies in the window rows
// p = (h + 1) / 2 - 1 and (h + 1) / 2 (the first only for odd h), the four pixels w0 .. w0 + 3 (w0 a multiple of 4) in the
// windows q = w0 / 2 .. w0 / 2 + 2; per window row 3 x 7 inputs and 3 gradients are loaded (10.5 inputs per pixel
// instead of 36).  Same order of windows, same bits as the general kernel.
template <bool ACC>
__global__ __launch_bounds__(256) void maxpool3s2_bwd_input_kernel(const float *__restrict__ dy, const float *__restrict__ x, float *dx,
                                                                   int N, int H, int W, int P, int Q, int C4, int segs, int64_t items) {
    constexpr int L = 4;
    const int64_t i = ((int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) * 256 + threadIdx.x;      // a contiguous share per XCD
    if (i >= items) return;
    const int c4 = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    const int w0 = seg * L, q0 = w0 >> 1;
    const int64_t img = (int64_t)n * H * W * C4 + c4, gimg = (int64_t)n * P * Q * C4 + c4;
    float acc[L][4];
#pragma unroll
    for (int j = 0; j < L; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] = 0.0f;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int p = ((h + 1) >> 1) - 1 + a;
        const int row = h - 2 * p + 1;                  // of pixel row h inside window row p
        if ((unsigned)p >= (unsigned)P || row > 2) continue;
        float4 v[3][7];
        bool in[3][7];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int hh = 2 * p - 1 + r;
#pragma unroll
            for (int c = 0; c < 7; ++c) {
                const int ww = w0 - 1 + c;
                in[r][c] = (unsigned)hh < (unsigned)H && (unsigned)ww < (unsigned)W;
                v[r][c] = ((const float4 *)x)[in[r][c] ? img + ((int64_t)hh * W + ww) * C4 : 0];
            }
        }
        float4 g[3];
        bool okq[3];
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            okq[b] = q0 + b < Q;
            g[b] = ((const float4 *)dy)[okq[b] ? gimg + ((int64_t)p * Q + q0 + b) * C4 : 0];
        }
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            if (!okq[b]) continue;
            // window (p, q0 + b) covers columns 2 (q0 + b) - 1 .. + 1 = patch columns 2 b .. 2 b + 2
            float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            int sel[4] = {0, 0, 0, 0};
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int sx = 0; sx < 3; ++sx) {
                    if (!in[r][2 * b + sx]) continue;
                    const float vv[4] = {v[r][2 * b + sx].x, v[r][2 * b + sx].y, v[r][2 * b + sx].z, v[r][2 * b + sx].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (vv[e] > best[e]) { best[e] = vv[e]; sel[e] = r * 3 + sx; }
                }
            const float gg[4] = {g[b].x, g[b].y, g[b].z, g[b].w};
            // pixel w0 + j sits at column j - 2 b + 1 of this window, for j = 2 b - 1 .. 2 b + 1
#pragma unroll
            for (int j = 0; j < L; ++j) {
                if (j < 2 * b - 1 || j > 2 * b + 1) continue;
                const int mine = row * 3 + (j - 2 * b + 1);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (sel[e] == mine) acc[j][e] += gg[e];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (w0 + j >= W) break;
        const int64_t o = img + ((int64_t)h * W + w0 + j) * C4;
        float4 r = make_float4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
        if (ACC) { const float4 was = ((const float4 *)dx)[o]; r.x += was.x; r.y += was.y; r.z += was.z; r.w += was.w; }
        ((float4 *)dx)[o] = r;
    }
}

void maxpool_bwd(hipStream_t st, const float *dy, const float *x, const uint8_t *idx, float *dx, const PoolShape &ps,
                 bool accumulate) {
    if (ps.C % 4) throw KernelError("maxpool: C must be a multiple of 4");
    if (!idx && !x) throw KernelError("maxpool_bwd: needs the input or the index");
    int64_t total = (int64_t)ps.N * ps.H * ps.W * (ps.C / 4);
    if (total <= 0) return;
    if (idx && ps.k == 3 && ps.stride == 1 && ps.pad == 1 && ps.P == ps.H && ps.Q == ps.W) {
        constexpr int L = 4;
        const int segs = (ps.W + L - 1) / L;
        const int64_t items = (int64_t)ps.N * ps.H * segs * (ps.C / 4);
        if ((items + 255) / 256 >= 0x7ffffff0ll) throw KernelError("maxpool_bwd: too many work items");
        const dim3 g1((unsigned)(((items + 255) / 256 + 7) / 8 * 8)), blk(256);
        if (accumulate) hipLaunchKernelGGL((maxpool3s1_bwd_kernel<L, true>), g1, blk, 0, st, dy, idx, dx, ps.N, ps.H, ps.W, ps.C / 4, segs, items);
        else hipLaunchKernelGGL((maxpool3s1_bwd_kernel<L, false>), g1, blk, 0, st, dy, idx, dx, ps.N, ps.H, ps.W, ps.C / 4, segs, items);
        hip_check(hipGetLastError(), "maxpool_bwd launch");
        return;
    }
    if (!idx && ps.k == 3 && ps.stride == 1 && ps.pad == 1 && ps.P == ps.H && ps.Q == ps.W) {
        constexpr int L = 4;
        const int segs = (ps.W + L - 1) / L;
        const int64_t items = (int64_t)ps.N * ps.H * segs * (ps.C / 4);
        if ((items + 255) / 256 >= 0x7ffffff0ll) throw KernelError("maxpool_bwd: too many work items");
        const dim3 g1((unsigned)(((items + 255) / 256 + 7) / 8 * 8)), blk(256);
        if (accumulate) hipLaunchKernelGGL((maxpool3s1_bwd_input_kernel<L, true>), g1, blk, 0, st, dy, x, dx, ps.N, ps.H, ps.W, ps.C / 4, segs, items);
        else hipLaunchKernelGGL((maxpool3s1_bwd_input_kernel<L, false>), g1, blk, 0, st, dy, x, dx, ps.N, ps.H, ps.W, ps.C / 4, segs, items);
        hip_check(hipGetLastError(), "maxpool_bwd launch");
        return;
    }
    if (!idx && ps.k == 3 && ps.stride == 2 && ps.pad == 1) {
        const int segs = (ps.W + 3) / 4;
        const int64_t items = (int64_t)ps.N * ps.H * segs * (ps.C / 4);
        if ((items + 255) / 256 >= 0x7ffffff0ll) throw KernelError("maxpool_bwd: too many work items");
        const dim3 g1((unsigned)(((items + 255) / 256 + 7) / 8 * 8)), blk(256);
        if (accumulate) hipLaunchKernelGGL((maxpool3s2_bwd_input_kernel<true>), g1, blk, 0, st, dy, x, dx, ps.N, ps.H, ps.W, ps.P, ps.Q, ps.C / 4, segs, items);
        else hipLaunchKernelGGL((maxpool3s2_bwd_input_kernel<false>), g1, blk, 0, st, dy, x, dx, ps.N, ps.H, ps.W, ps.P, ps.Q, ps.C / 4, segs, items);
        hip_check(hipGetLastError(), "maxpool_bwd launch");
        return;
    }
    if (idx && ps.k == 3 && ps.stride == 2 && ps.pad == 1) {
        const int segs = (ps.W + 3) / 4;
        const int64_t items = (int64_t)ps.N * ps.H * segs * (ps.C / 4);
        if ((items + 255) / 256 > 0x7fffffffll) throw KernelError("maxpool_bwd: too many work items");
        const dim3 g1((unsigned)((items + 255) / 256)), blk(256);
        if (accumulate) hipLaunchKernelGGL((maxpool3s2_bwd_idx_kernel<true>), g1, blk, 0, st, dy, idx, dx, ps.N, ps.H, ps.W, ps.P, ps.Q, ps.C / 4, segs, items);
        else hipLaunchKernelGGL((maxpool3s2_bwd_idx_kernel<false>), g1, blk, 0, st, dy, idx, dx, ps.N, ps.H, ps.W, ps.P, ps.Q, ps.C / 4, segs, items);
        hip_check(hipGetLastError(), "maxpool_bwd launch");
        return;
    }
    if (idx && (total + 255) / 256 <= 0x7fffffffll && ps.pad >= 0 && ps.pad < ps.k &&
        ((ps.k == 3 && (ps.stride == 1 || ps.stride == 2)) || (ps.k == 2 && ps.stride == 2))) {
        const dim3 g1((unsigned)((total + 255) / 256)), blk(256);
#define MPI(K, S) do { if (accumulate) hipLaunchKernelGGL((maxpool_bwd_idx_kernel<K, S, true>), g1, blk, 0, st, dy, idx, dx, ps); \
                       else hipLaunchKernelGGL((maxpool_bwd_idx_kernel<K, S, false>), g1, blk, 0, st, dy, idx, dx, ps); } while (0)
        if (ps.k == 3 && ps.stride == 1) MPI(3, 1);
        else if (ps.k == 3) MPI(3, 2);
        else MPI(2, 2);
#undef MPI
        hip_check(hipGetLastError(), "maxpool_bwd launch");
        return;
    }
    int grid = grid_for(total, 256, 1 << 16);
#define MP(F, A) hipLaunchKernelGGL((maxpool_bwd_kernel<F, A>), dim3(grid), dim3(256), 0, st, dy, x, idx, dx, ps)
    if (idx) { if (accumulate) MP(true, true); else MP(true, false); }
    else     { if (accumulate) MP(false, true); else MP(false, false); }
#undef MP
    hip_check(hipGetLastError(), "maxpool_bwd launch");
}

// ------------------------------------------------------------------ global average pool
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, int N, int HW, int C) {
    const int64_t total = (int64_t)N * C;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int c = (int)(i % C);
        int n = (int)(i / C);
        float s = 0;
        for (int p = 0; p < HW; ++p) s += x[((int64_t)n * HW + p) * C + c];
        y[i] = s / (float)HW;
    }
}
template <bool ACC>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const float *__restrict__ dy, float *dx, int N, int HW, int C) {
    const int64_t total = (int64_t)N * HW * C;
    const float inv = 1.0f / (float)HW;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int c = (int)(i % C);
        int n = (int)(i / ((int64_t)HW * C));
        float v = dy[(int64_t)n * C + c] * inv;
        dx[i] = ACC ? dx[i] + v : v;
    }
}
void avgpool_fwd(hipStream_t st, const float *x, float *y, int N, int HW, int C) {
    hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(grid_for((int64_t)N * C, 256)), dim3(256), 0, st, x, y, N, HW, C);
    hip_check(hipGetLastError(), "avgpool_fwd launch");
}
void avgpool_bwd(hipStream_t st, const float *dy, float *dx, int N, int HW, int C, bool accumulate) {
    int grid = grid_for((int64_t)N * HW * C, 256);
    if (accumulate) hipLaunchKernelGGL((avgpool_bwd_kernel<true>), dim3(grid), dim3(256), 0, st, dy, dx, N, HW, C);
    else hipLaunchKernelGGL((avgpool_bwd_kernel<false>), dim3(grid), dim3(256), 0, st, dy, dx, N, HW, C);
    hip_check(hipGetLastError(), "avgpool_bwd launch");
}

// ------------------------------------------------------------------ block reductions (fixed order: deterministic)
__device__ inline float block_sum(float v, float *sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    if (lane == 0) sh[wid] = v;
    __syncthreads();
    float r = 0;
    if (threadIdx.x == 0)
        for (int i = 0; i < (int)(blockDim.x >> 6); ++i) r += sh[i];
    __syncthreads();
    return r;   // valid in thread 0
}
__device__ inline float block_max(float v, float *sh) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_down(v, o, 64));
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    if (lane == 0) sh[wid] = v;
    __syncthreads();
    float r = sh[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmaxf(r, sh[i]);
    __syncthreads();
    return r;   // valid in every thread
}

// ------------------------------------------------------------------ softmax cross-entropy (mean over rows)
__global__ __launch_bounds__(256) void softmaxce_row_kernel(const float *__restrict__ logits, const int32_t *__restrict__ labels,
                                                            float *__restrict__ row_loss, int classes) {
    __shared__ float sh[8];
    const int n = blockIdx.x;
    const float *z = logits + (int64_t)n * classes;
    float m = -INFINITY;
    for (int c = threadIdx.x; c < classes; c += blockDim.x) m = fmaxf(m, z[c]);
    m = block_max(m, sh);
    float s = 0;
    for (int c = threadIdx.x; c < classes; c += blockDim.x) s += expf(z[c] - m);
    s = block_sum(s, sh);
    if (threadIdx.x == 0) row_loss[n] = logf(s) - (z[labels[n]] - m);
}
__global__ __launch_bounds__(256) void mean_kernel(const float *__restrict__ v, float *__restrict__ out, int64_t n, float scale) {
    __shared__ float sh[8];
    // two-level fixed-order sum; partial sums in double so that long inputs keep fp32 accuracy
    double s = 0;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) s += (double)v[i];
    float r = block_sum((float)s, sh);
    if (threadIdx.x == 0) out[0] = r * scale;
}
void softmaxce_fwd(hipStream_t st, const float *logits, const int32_t *labels, float *loss, int N, int classes, float *scratch) {
    hipLaunchKernelGGL(softmaxce_row_kernel, dim3(N), dim3(256), 0, st, logits, labels, scratch, classes);
    hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, st, (const float *)scratch, loss, (int64_t)N, 1.0f / (float)N);
    hip_check(hipGetLastError(), "softmaxce_fwd launch");
}
template <bool ACC>
__global__ __launch_bounds__(256) void softmaxce_bwd_kernel(const float *__restrict__ logits, const int32_t *__restrict__ labels,
                                                            float *dlogits, int classes, float invN) {
    __shared__ float sh[8];
    __shared__ float tot;
    const int n = blockIdx.x;
    const float *z = logits + (int64_t)n * classes;
    float m = -INFINITY;
    for (int c = threadIdx.x; c < classes; c += blockDim.x) m = fmaxf(m, z[c]);
    m = block_max(m, sh);
    float s = 0;
    for (int c = threadIdx.x; c < classes; c += blockDim.x) s += expf(z[c] - m);
    s = block_sum(s, sh);
    if (threadIdx.x == 0) tot = s;
    __syncthreads();
    const float inv = 1.0f / tot;
    const int lab = labels[n];
    for (int c = threadIdx.x; c < classes; c += blockDim.x) {
        float g = (expf(z[c] - m) * inv - (c == lab ? 1.0f : 0.0f)) * invN;
        float *d = dlogits + (int64_t)n * classes + c;
        *d = ACC ? *d + g : g;
    }
}
void softmaxce_bwd(hipStream_t st, const float *logits, const int32_t *labels, float *dlogits, int N, int classes, bool accumulate) {
    if (accumulate) hipLaunchKernelGGL((softmaxce_bwd_kernel<true>), dim3(N), dim3(256), 0, st, logits, labels, dlogits, classes, 1.0f / N);
    else hipLaunchKernelGGL((softmaxce_bwd_kernel<false>), dim3(N), dim3(256), 0, st, logits, labels, dlogits, classes, 1.0f / N);
    hip_check(hipGetLastError(), "softmaxce_bwd launch");
}

// ------------------------------------------------------------------ sum loss
__global__ __launch_bounds__(256) void partial_sum_kernel(const float *__restrict__ x, float *__restrict__ part, int64_t n) {
    __shared__ float sh[8];
    float s = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) s += x[i];
    s = block_sum(s, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = s;
}
// ------------------------------------------------------------------ linear-layer bias
__global__ __launch_bounds__(256) void bias_add_kernel(float *y, const float *__restrict__ b, int64_t total, int out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        y[i] += b[i % out];
}
__global__ __launch_bounds__(256) void bias_grad_kernel(const float *__restrict__ dy, float *__restrict__ db, int N, int out) {
    int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= out) return;
    float s = 0;
    for (int n = 0; n < N; ++n) s += dy[(int64_t)n * out + c];
    db[c] = s;
}
void linear_bias_add(hipStream_t st, float *y, const float *b, int N, int out) {
    int64_t total = (int64_t)N * out;
    hipLaunchKernelGGL(bias_add_kernel, dim3(grid_for(total, 256, 4096)), dim3(256), 0, st, y, b, total, out);
    hip_check(hipGetLastError(), "bias add launch");
}
void linear_bias_grad(hipStream_t st, const float *dy, float *db, int N, int out) {
    hipLaunchKernelGGL(bias_grad_kernel, dim3((out + 255) / 256), dim3(256), 0, st, dy, db, N, out);
    hip_check(hipGetLastError(), "bias grad launch");
}

void sumloss_fwd(hipStream_t st, const float *x, float *loss, int64_t n, float *scratch, size_t scratch_bytes) {
    int grid = grid_for(n, 256 * 16, 1024);
    if ((size_t)grid * 4 > scratch_bytes) throw KernelError("sumloss: scratch too small");
    hipLaunchKernelGGL(partial_sum_kernel, dim3(grid), dim3(256), 0, st, x, scratch, n);
    hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, st, (const float *)scratch, loss, (int64_t)grid, 1.0f);
    hip_check(hipGetLastError(), "sumloss_fwd launch");
}

}  // namespace monet
