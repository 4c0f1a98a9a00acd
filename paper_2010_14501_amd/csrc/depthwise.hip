// Bandwidth-bound operators of the segmentation and mobile networks: depthwise convolution
// (forward, input gradient, filter gradient), copies between tensors of different row length
// (channel concatenation and its backward), and cross-entropy over rows with few classes
// (per-pixel losses).  A depthwise filter touches one channel only, so there is no contraction to
// hand to the matrix cores: every output element costs R*S multiply-adds and the kernels are bound
// by HBM traffic (one read of the input, one write of the output).  NHWC, fp32, four channels per
// thread, filters staged in LDS in tap-major order so that four neighbouring channels are one
// 16-byte LDS read.
#include "bn_affine.hpp"
#include "kernels.hpp"

namespace monet {

namespace {

int grid_cap(int64_t items, int per_block, int cap) {
    int64_t g = (items + per_block - 1) / per_block;
    return (int)std::max<int64_t>(1, std::min<int64_t>(g, cap));
}

__device__ inline float4 ld4(const float *p) { return *(const float4 *)p; }
__device__ inline void fma4(float4 &a, const float4 &x, const float4 &w) {
    a.x += x.x * w.x; a.y += x.y * w.y; a.z += x.z * w.z; a.w += x.w * w.w;
}

// filters are stored C,R,S (channel-major); LDS copy is [tap][C]
__device__ inline void stage_filters(float *wl, const float *__restrict__ w, int C, int taps) {
    for (int i = threadIdx.x; i < C * taps; i += blockDim.x) {
        int c = i / taps, t = i - c * taps;
        wl[t * C + c] = w[i];
    }
    __syncthreads();
}

// ------------------------------------------------------------------ forward
// V = 4: C % 4 == 0, one thread per (pixel, four channels); V = 1: any C, one thread per element.
template <int V>
__global__ __launch_bounds__(256) void dw_fwd_kernel(const float *__restrict__ x, const float *__restrict__ w, float *__restrict__ y,
                                                     ConvShape cs) {
    extern __shared__ float wl[];
    const int C = cs.C, taps = cs.R * cs.S, CV = C / V;
    stage_filters(wl, w, C, taps);
    const int64_t total = cs.M() * CV;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int cv = (int)(i % CV);
        int64_t pix = i / CV;
        const int q = (int)(pix % cs.Q); pix /= cs.Q;
        const int p = (int)(pix % cs.P);
        const int n = (int)(pix / cs.P);
        const float *xn = x + (int64_t)n * cs.H * cs.W * C + cv * V;
        float4 acc = make_float4(0, 0, 0, 0);
        for (int r = 0; r < cs.R; ++r) {
            const int h = p * cs.stride + r - cs.pad;
            if ((unsigned)h >= (unsigned)cs.H) continue;
            for (int s = 0; s < cs.S; ++s) {
                const int v = q * cs.stride + s - cs.pad;
                if ((unsigned)v >= (unsigned)cs.W) continue;
                const float *px = xn + ((int64_t)h * cs.W + v) * C;
                const float *pw = wl + (r * cs.S + s) * C + cv * V;
                if (V == 4) fma4(acc, ld4(px), *(const float4 *)pw);
                else acc.x += px[0] * pw[0];
            }
        }
        if (V == 4) *(float4 *)(y + i * 4) = acc;
        else y[i] = acc.x;
    }
}

// ------------------------------------------------------------------ input gradient
template <int V, bool ACC>
__global__ __launch_bounds__(256) void dw_dgrad_kernel(const float *__restrict__ dy, const float *__restrict__ w, float *dx, ConvShape cs) {
    extern __shared__ float wl[];
    const int C = cs.C, taps = cs.R * cs.S, CV = C / V;
    stage_filters(wl, w, C, taps);
    const int64_t total = (int64_t)cs.N * cs.H * cs.W * CV;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int cv = (int)(i % CV);
        int64_t pix = i / CV;
        const int v = (int)(pix % cs.W); pix /= cs.W;
        const int h = (int)(pix % cs.H);
        const int n = (int)(pix / cs.H);
        const float *gn = dy + (int64_t)n * cs.P * cs.Q * C + cv * V;
        float4 acc = make_float4(0, 0, 0, 0);
        for (int r = 0; r < cs.R; ++r) {
            const int hp = h + cs.pad - r;
            if (hp < 0 || hp % cs.stride) continue;
            const int p = hp / cs.stride;
            if (p >= cs.P) continue;
            for (int s = 0; s < cs.S; ++s) {
                const int vq = v + cs.pad - s;
                if (vq < 0 || vq % cs.stride) continue;
                const int q = vq / cs.stride;
                if (q >= cs.Q) continue;
                const float *pg = gn + ((int64_t)p * cs.Q + q) * C;
                const float *pw = wl + (r * cs.S + s) * C + cv * V;
                if (V == 4) fma4(acc, ld4(pg), *(const float4 *)pw);
                else acc.x += pg[0] * pw[0];
            }
        }
        if (V == 4) {
            float4 *d = (float4 *)(dx + i * 4);
            if (ACC) { float4 o = *d; acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w; }
            *d = acc;
        } else {
            dx[i] = ACC ? dx[i] + acc.x : acc.x;
        }
    }
}

// ------------------------------------------------------------------ filter gradient
// Two levels, both in a fixed order (no float atomics): block (slab, channel chunk) sums its pixels into
// part[slab][tap][C]; the second kernel adds the slabs.  blockDim = (CL, 256 / CL): x = channel lane
// (V channels each), y = pixel lane.
constexpr int DW_MAX_TAPS = 9;

template <int V>
__global__ __launch_bounds__(256) void dw_wgrad_partial(const float *__restrict__ x, const float *__restrict__ dy, float *__restrict__ part,
                                                        ConvShape cs, int64_t pix_per_slab) {
    extern __shared__ float red[];   // [blockDim.y][taps][CL * V]
    const int C = cs.C, CV = C / V, taps = cs.R * cs.S;
    const int CL = blockDim.x, PL = blockDim.y;
    const int cv = blockIdx.y * CL + threadIdx.x;
    const bool live = cv < CV;
    float4 acc[DW_MAX_TAPS];
#pragma unroll
    for (int t = 0; t < DW_MAX_TAPS; ++t) acc[t] = make_float4(0, 0, 0, 0);
    const int64_t M = cs.M();
    const int64_t p0 = blockIdx.x * pix_per_slab;
    const int64_t p1 = p0 + pix_per_slab < M ? p0 + pix_per_slab : M;
    if (live) {
        for (int64_t pix = p0 + threadIdx.y; pix < p1; pix += PL) {
            int64_t t = pix;
            const int q = (int)(t % cs.Q); t /= cs.Q;
            const int p = (int)(t % cs.P);
            const int n = (int)(t / cs.P);
            float4 g = make_float4(0, 0, 0, 0);
            if (V == 4) g = ld4(dy + pix * C + cv * 4);
            else g.x = dy[pix * C + cv];
            const float *xn = x + (int64_t)n * cs.H * cs.W * C + cv * V;
#pragma unroll
            for (int tp = 0; tp < DW_MAX_TAPS; ++tp) {
                if (tp >= taps) break;
                const int r = tp / cs.S, s = tp - r * cs.S;
                const int h = p * cs.stride + r - cs.pad, v = q * cs.stride + s - cs.pad;
                if ((unsigned)h >= (unsigned)cs.H || (unsigned)v >= (unsigned)cs.W) continue;
                const float *px = xn + ((int64_t)h * cs.W + v) * C;
                if (V == 4) fma4(acc[tp], ld4(px), g);
                else acc[tp].x += px[0] * g.x;
            }
        }
    }
    // pixel lanes -> lane 0, in lane order
    const int width = CL * V;
#pragma unroll
    for (int tp = 0; tp < DW_MAX_TAPS; ++tp) {
        if (tp >= taps) break;
        float *dst = red + ((size_t)threadIdx.y * taps + tp) * width + threadIdx.x * V;
        if (V == 4) *(float4 *)dst = acc[tp];
        else dst[0] = acc[tp].x;
    }
    __syncthreads();
    if (threadIdx.y == 0 && live) {
        for (int tp = 0; tp < taps; ++tp) {
            float4 s = make_float4(0, 0, 0, 0);
            for (int l = 0; l < PL; ++l) {
                const float *src = red + ((size_t)l * taps + tp) * width + threadIdx.x * V;
                if (V == 4) { float4 a = *(const float4 *)src; s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w; }
                else s.x += src[0];
            }
            float *out = part + ((size_t)blockIdx.x * taps + tp) * C + cv * V;
            if (V == 4) *(float4 *)out = s;
            else out[0] = s.x;
        }
    }
}

// dw[c][tap] = sum over slabs.  Block = 4 outputs (consecutive channels of one tap) x 64 slab lanes: lane l
// adds slabs l, l+64, ... in order (four loads in flight), then the lanes are added by a fixed tree.  A
// single thread per output would be a chain of `slabs` dependent loads.
__global__ __launch_bounds__(256) void dw_wgrad_final(const float *__restrict__ part, float *__restrict__ dw, int C, int taps, int slabs) {
    __shared__ float sh[256];
    const int ol = threadIdx.x & 3, sl = threadIdx.x >> 2;
    const int i = blockIdx.x * 4 + ol;                      // over tap-major (tap, c)
    const bool live = i < C * taps;
    const int tp = live ? i / C : 0, c = live ? i - tp * C : 0;
    float s = 0;
    if (live)
        for (int b0 = sl; b0 < slabs; b0 += 4 * 64) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int b = b0 + u * 64;
                v[u] = b < slabs ? part[((size_t)b * taps + tp) * C + c] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (b0 + u * 64 < slabs) s += v[u];
        }
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int half = 32; half > 0; half >>= 1) {
        if (sl < half) sh[threadIdx.x] += sh[(sl + half) * 4 + ol];
        __syncthreads();
    }
    if (sl == 0 && live) dw[c * taps + tp] = sh[ol];
}

// ------------------------------------------------------------------ 3x3 filters, C % 4 == 0
// The common case, with the tap loops unrolled at compile time: all nine 16-byte loads of a thread are
// issued before the first multiply-add (out-of-range taps load the image's first pixel and are zeroed),
// and no integer division is left in the inner loop.
typedef float f4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void dw3_fwd_kernel(const float *__restrict__ x, const float *__restrict__ w, float *__restrict__ y,
                                                      ConvShape cs, int64_t pix_per_block) {
    // blockDim = (CL, 256 / CL): x = channel group, y = pixel lane; a block owns the pixel range
    // [blockIdx.x * pix_per_block, ...) and steps through it without divisions
    extern __shared__ float wl[];
    const int C = cs.C, C4 = C / 4;
    {   // filters: all threads of the 2-D block take part
        const int tid = threadIdx.y * blockDim.x + threadIdx.x;
        for (int i = tid; i < C * 9; i += 256) {
            int c = i / 9, t = i - c * 9;
            wl[t * C + c] = w[i];
        }
        __syncthreads();
    }
    const int CL = blockDim.x, PL = blockDim.y;
    const int cv = blockIdx.y * CL + threadIdx.x;
    if (cv >= C4) return;
    const int64_t M = cs.M();
    const int64_t p0 = (int64_t)blockIdx.x * pix_per_block;
    const int64_t p1 = p0 + pix_per_block < M ? p0 + pix_per_block : M;
    int64_t pix = p0 + threadIdx.y;
    if (pix >= p1) return;
    int q = (int)(pix % cs.Q);
    int64_t t2 = pix / cs.Q;
    int p = (int)(t2 % cs.P);
    int n = (int)(t2 / cs.P);
    f4 wv[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) wv[t] = *(const f4 *)(wl + t * C + cv * 4);
    for (; pix < p1; pix += PL) {
        const int h0 = p * cs.stride - cs.pad, v0 = q * cs.stride - cs.pad;
        const f4 *xn = (const f4 *)x + (int64_t)n * cs.H * cs.W * C4 + cv;
        f4 xv[9];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int h = h0 + r, v = v0 + s;
                const bool ok = (unsigned)h < (unsigned)cs.H && (unsigned)v < (unsigned)cs.W;
                const f4 t = xn[ok ? (h * cs.W + v) * C4 : 0];
                xv[r * 3 + s] = ok ? t : f4{0, 0, 0, 0};
            }
        f4 acc = f4{0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < 9; ++t) acc += xv[t] * wv[t];
        ((f4 *)y)[pix * C4 + cv] = acc;
        q += PL;
        while (q >= cs.Q) { q -= cs.Q; if (++p == cs.P) { p = 0; ++n; } }
    }
}

template <bool ACC>
__global__ __launch_bounds__(256) void dw3_dgrad_kernel(const float *__restrict__ dy, const float *__restrict__ w, float *dx, ConvShape cs,
                                                        int64_t pix_per_block) {
    // same block shape and stepping as dw3_fwd_kernel, over the pixels of dx
    extern __shared__ float wl[];
    const int C = cs.C, C4 = C / 4, st = cs.stride;
    {
        const int tid = threadIdx.y * blockDim.x + threadIdx.x;
        for (int i = tid; i < C * 9; i += 256) {
            int c = i / 9, t = i - c * 9;
            wl[t * C + c] = w[i];
        }
        __syncthreads();
    }
    const int CL = blockDim.x, PL = blockDim.y;
    const int cv = blockIdx.y * CL + threadIdx.x;
    if (cv >= C4) return;
    const int64_t M = (int64_t)cs.N * cs.H * cs.W;
    const int64_t p0 = (int64_t)blockIdx.x * pix_per_block;
    const int64_t p1 = p0 + pix_per_block < M ? p0 + pix_per_block : M;
    int64_t pix = p0 + threadIdx.y;
    if (pix >= p1) return;
    int v = (int)(pix % cs.W);
    int64_t t2 = pix / cs.W;
    int h = (int)(t2 % cs.H);
    int n = (int)(t2 / cs.H);
    f4 wv[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) wv[t] = *(const f4 *)(wl + t * C + cv * 4);
    for (; pix < p1; pix += PL) {
        const f4 *gn = (const f4 *)dy + (int64_t)n * cs.P * cs.Q * C4 + cv;
        f4 gv[9];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int hp = h + cs.pad - r, vq = v + cs.pad - s;
                const int p = st == 1 ? hp : (st == 2 ? hp >> 1 : hp / st), q = st == 1 ? vq : (st == 2 ? vq >> 1 : vq / st);
                const bool ok = hp >= 0 && vq >= 0 && p * st == hp && q * st == vq && p < cs.P && q < cs.Q;
                const f4 t = gn[ok ? (p * cs.Q + q) * C4 : 0];
                gv[r * 3 + s] = ok ? t : f4{0, 0, 0, 0};
            }
        f4 acc = f4{0, 0, 0, 0};
#pragma unroll
        for (int t = 0; t < 9; ++t) acc += gv[t] * wv[t];
        f4 *d = (f4 *)dx + pix * C4 + cv;
        if (ACC) acc += *d;
        *d = acc;
        v += PL;
        while (v >= cs.W) { v -= cs.W; if (++h == cs.H) { h = 0; ++n; } }
    }
}

// blockDim = (CL, 256 / CL) as in dw_wgrad_partial; part[slab][tap][C]
__global__ __launch_bounds__(256) void dw3_wgrad_partial(const float *__restrict__ x, const float *__restrict__ dy, float *__restrict__ part,
                                                         ConvShape cs, int64_t pix_per_slab) {
    extern __shared__ float red[];   // [blockDim.y][9][CL * 4]
    const int C = cs.C, C4 = C / 4;
    const int CL = blockDim.x, PL = blockDim.y;
    const int cv = blockIdx.y * CL + threadIdx.x;
    const bool live = cv < C4;
    f4 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[t] = f4{0, 0, 0, 0};
    const int64_t M = cs.M();
    const int64_t p0 = blockIdx.x * pix_per_slab;
    const int64_t p1 = p0 + pix_per_slab < M ? p0 + pix_per_slab : M;
    if (live) {
        int64_t pix = p0 + threadIdx.y;
        // position of the thread's first pixel; afterwards advanced by PL pixels without divisions
        int q = (int)(pix % cs.Q);
        int64_t t2 = pix / cs.Q;
        int p = (int)(t2 % cs.P);
        int n = (int)(t2 / cs.P);
        for (; pix < p1; pix += PL) {
            const f4 g = ((const f4 *)dy)[pix * C4 + cv];
            const f4 *xn = (const f4 *)x + (int64_t)n * cs.H * cs.W * C4 + cv;
            const int h0 = p * cs.stride - cs.pad, v0 = q * cs.stride - cs.pad;
            f4 xv[9];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const int h = h0 + r, v = v0 + s;
                    const bool ok = (unsigned)h < (unsigned)cs.H && (unsigned)v < (unsigned)cs.W;
                    const f4 t = xn[ok ? ((int64_t)h * cs.W + v) * C4 : 0];
                    xv[r * 3 + s] = ok ? t : f4{0, 0, 0, 0};
                }
#pragma unroll
            for (int t = 0; t < 9; ++t) acc[t] += xv[t] * g;
            q += PL;
            while (q >= cs.Q) { q -= cs.Q; if (++p == cs.P) { p = 0; ++n; } }
        }
    }
    const int width = CL * 4;
#pragma unroll
    for (int t = 0; t < 9; ++t) *(f4 *)(red + ((size_t)threadIdx.y * 9 + t) * width + threadIdx.x * 4) = acc[t];
    __syncthreads();
    // pixel lanes are added in lane order by the 9 * CL threads (tap, channel group) of the block
    for (int j = threadIdx.y * CL + threadIdx.x; j < 9 * CL; j += CL * PL) {
        const int t = j / CL, cl = j - t * CL;
        const int c4 = blockIdx.y * CL + cl;
        if (c4 >= C4) continue;
        f4 s = f4{0, 0, 0, 0};
        for (int l = 0; l < PL; ++l) s += *(const f4 *)(red + ((size_t)l * 9 + t) * width + cl * 4);
        *(f4 *)(part + ((size_t)blockIdx.x * 9 + t) * C + c4 * 4) = s;
    }
}

// ------------------------------------------------------------------ 3x3 filters, C % 4 == 0, pad 1: row segments
// One thread per (image row of the output, segment of L consecutive outputs, four channels).  The 3 x ((L-1)*STRIDE + 3)
// inputs under the segment are loaded once and every one of them serves up to three outputs from registers: 3.9 loads
// per output at L = 7 and stride 1 instead of 9, which is what moves these kernels from the L1 / address-unit limit
// towards the HBM one (L = 7 divides every map width of a 224-pixel network).  FLIP turns the filter by 180
// degrees: with stride 1 the input gradient is the forward operator applied to dy with the flipped filter.  Lanes
// that are neighbours in x are neighbours in channels, so each load instruction covers whole pixels.  Work items are
// ordered (image, row, segment, channels) and every XCD takes one contiguous share of them (workgroups go to the
// eight XCDs in turn), so that the three output rows that read an input row find it in the same L2.
// workgroup b of a grid of nb (a multiple of 8) -> position in the XCD-contiguous order
__device__ inline int64_t xcd_block(unsigned b, unsigned nb) { return (int64_t)(b & 7) * (nb >> 3) + (b >> 3); }

template <int STRIDE, int L, bool FLIP, bool ACC>
__global__ __launch_bounds__(256) void dw3_row_kernel(const float *__restrict__ in, const float *__restrict__ w, float *out, int N, int H, int W,
                                                      int P, int Q, int C4, int segs, int64_t items, BnAffine bn) {
    constexpr int COLS = (L - 1) * STRIDE + 3;
    const int64_t i = xcd_block(blockIdx.x, gridDim.x) * 256 + threadIdx.x;
    if (i >= items) return;
    const int cv = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int p = (int)(t % P);
    const int n = (int)(t / P);
    const int q0 = seg * L;
    f4 wv[9];      // filters are stored C,3,3: 36 consecutive floats for the thread's four channels
    {
        const float *wp = w + (int64_t)cv * 36;
#pragma unroll
        for (int tp = 0; tp < 9; ++tp) {
            const int src = FLIP ? 8 - tp : tp;
            wv[tp] = f4{wp[src], wp[9 + src], wp[18 + src], wp[27 + src]};
        }
    }
    const f4 *base = (const f4 *)in + (int64_t)n * H * W * C4 + cv;
    const int h0 = p * STRIDE - 1, v0 = q0 * STRIDE - 1;
    f4 xv[3][COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int h = h0 + r;
        const bool hok = (unsigned)h < (unsigned)H;
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            const int v = v0 + c;
            const bool ok = hok && (unsigned)v < (unsigned)W;
            const f4 ld = base[ok ? ((int64_t)h * W + v) * C4 : 0];
            xv[r][c] = ok ? ld : f4{0, 0, 0, 0};
        }
    }
    f4 *dst = (f4 *)out + (((int64_t)n * P + p) * Q + q0) * C4 + cv;
    // optional BatchNorm apply step of the result (a recomputed forward operator whose statistics are known)
    const bool affine = !FLIP && !ACC && bn.gamma != nullptr;
    float bn_a[4] = {1, 1, 1, 1}, bn_b[4] = {0, 0, 0, 0};
    if (affine) {
#pragma unroll
        for (int j = 0; j < 4; ++j) bn_affine_coeffs(bn.gamma, bn.beta, bn.stats, 4 * C4, 4 * cv + j, bn_a[j], bn_b[j]);
    }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        if (q0 + j >= Q) break;
        f4 acc = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) acc += xv[r][j * STRIDE + sx] * wv[r * 3 + sx];
        if (ACC) acc += dst[(int64_t)j * C4];
        if (affine) acc = f4{bn_affine(acc.x, bn_a[0], bn_b[0]), bn_affine(acc.y, bn_a[1], bn_b[1]), bn_affine(acc.z, bn_a[2], bn_b[2]), bn_affine(acc.w, bn_a[3], bn_b[3])};
        if (affine && bn.relu) {
            const f4 rv = f4{relu_clamp(acc.x, bn.relu), relu_clamp(acc.y, bn.relu), relu_clamp(acc.z, bn.relu), relu_clamp(acc.w, bn.relu)};
            if (bn.relu_out) ((f4 *)bn.relu_out + (dst - (f4 *)out))[(int64_t)j * C4] = rv;
            else acc = rv;
        }
        dst[(int64_t)j * C4] = acc;
    }
}

template <int STRIDE, int L, bool FLIP, bool ACC>
void launch_dw3_row(hipStream_t st, const float *in, const float *w, float *out, int N, int H, int W, int P, int Q, int C,
                    const BnAffine &bn = BnAffine{}) {
    const int segs = (Q + L - 1) / L;
    const int64_t items = (int64_t)N * P * segs * (C / 4);
    const int64_t blocks = ((items + 255) / 256 + 7) / 8 * 8;
    if (blocks > 0x7fffffffll) throw KernelError("depthwise: too many work items");
    hipLaunchKernelGGL((dw3_row_kernel<STRIDE, L, FLIP, ACC>), dim3((unsigned)blocks), dim3(256), 0, st, in, w, out, N, H, W, P, Q, C / 4, segs,
                       items, bn);
}

// Input gradient for stride 2 (pad 1): the 2x2 block of dx at (2p', 2q') reads the 2x2 block of dy at (p', q') --
//   dx[2p'  ][2q'  ] = dy[p'][q'] w11                      dx[2p'  ][2q'+1] = dy[p'][q'+1] w10 + dy[p'][q'] w12
//   dx[2p'+1][2q'  ] = dy[p'+1][q'] w01 + dy[p'][q'] w21   dx[2p'+1][2q'+1] = dy[p'+1][q'+1] w00 + dy[p'+1][q'] w02
//                                                                           + dy[p'][q'+1] w20 + dy[p'][q'] w22
// One thread per (dy row pair, segment of L block columns, four channels): 2 (L + 1) loads for 4 L outputs, where a
// kernel over dx pixels tests nine taps each.  The kernel is bound by writing dx, four times the size of dy.
template <int L, bool ACC>
__global__ __launch_bounds__(256) void dw3_dgrad_s2_kernel(const float *__restrict__ dy, const float *__restrict__ w, float *dx, int N, int H, int W,
                                                           int P, int Q, int C4, int rows2, int segs, int64_t items) {
    const int64_t i = xcd_block(blockIdx.x, gridDim.x) * 256 + threadIdx.x;
    if (i >= items) return;
    const int cv = (int)(i % C4);
    int64_t t = i / C4;
    const int seg = (int)(t % segs); t /= segs;
    const int pp = (int)(t % rows2);
    const int n = (int)(t / rows2);
    const int q0 = seg * L;
    f4 wv[9];
    {
        const float *wp = w + (int64_t)cv * 36;
#pragma unroll
        for (int tp = 0; tp < 9; ++tp) wv[tp] = f4{wp[tp], wp[9 + tp], wp[18 + tp], wp[27 + tp]};
    }
    const f4 *base = (const f4 *)dy + (int64_t)n * P * Q * C4 + cv;
    f4 g[2][L + 1];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int c = 0; c <= L; ++c) {
            const bool ok = pp + r < P && q0 + c < Q;
            const f4 ld = base[ok ? ((int64_t)(pp + r) * Q + q0 + c) * C4 : 0];
            g[r][c] = ok ? ld : f4{0, 0, 0, 0};
        }
#pragma unroll
    for (int j = 0; j < L; ++j) {
        const int v = 2 * (q0 + j);
        if (v >= W) break;
        const f4 a = g[0][j], b = g[0][j + 1], c = g[1][j], d = g[1][j + 1];
        f4 o[2][2];
        o[0][0] = a * wv[4];
        o[0][1] = b * wv[3] + a * wv[5];
        o[1][0] = c * wv[1] + a * wv[7];
        o[1][1] = d * wv[0] + c * wv[2] + b * wv[6] + a * wv[8];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int h = 2 * pp + r;
            if (h >= H) continue;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                if (v + e >= W) continue;
                f4 *dst = (f4 *)dx + (((int64_t)n * H + h) * W + v + e) * C4 + cv;
                *dst = ACC ? *dst + o[r][e] : o[r][e];
            }
        }
    }
}

// Filter gradient over row segments (pad 1): blockDim = (CL, 256 / CL) as in dw_wgrad_partial, but a pixel lane
// takes whole segments of L consecutive outputs of one row: it loads the L output gradients and, row by row, the
// (L-1)*STRIDE + 3 inputs under them, and every input serves up to three taps from registers (3.9 + 1 loads per
// output pixel at L = 7 and stride 1 instead of 10).  Slab `blockIdx.x` owns segments [blockIdx.x * per_slab, ...);
// sums are formed per lane in segment order, then over the lanes in lane order, then over the slabs by
// dw_wgrad_final: a fixed order throughout.
template <int STRIDE, int L>
__global__ __launch_bounds__(256) void dw3_wgrad_row_partial(const float *__restrict__ x, const float *__restrict__ dy, float *__restrict__ part,
                                                             int N, int H, int W, int P, int Q, int C, int segs, int64_t items, int64_t per_slab) {
    constexpr int COLS = (L - 1) * STRIDE + 3;
    extern __shared__ float red[];   // [blockDim.y][9][CL * 4]
    const int C4 = C / 4;
    const int CL = blockDim.x, PL = blockDim.y;
    const int cv = blockIdx.y * CL + threadIdx.x;
    const bool live = cv < C4;
    f4 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[t] = f4{0, 0, 0, 0};
    const int64_t i0 = (int64_t)blockIdx.x * per_slab;
    const int64_t i1 = i0 + per_slab < items ? i0 + per_slab : items;
    if (live) {
        for (int64_t it = i0 + threadIdx.y; it < i1; it += PL) {
            const int seg = (int)(it % segs);
            const int64_t row = it / segs;
            const int p = (int)(row % P), n = (int)(row / P);
            const int q0 = seg * L;
            const f4 *gp = (const f4 *)dy + (((int64_t)n * P + p) * Q + q0) * C4 + cv;
            f4 g[L];
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const bool ok = q0 + j < Q;
                const f4 ld = gp[ok ? (int64_t)j * C4 : 0];
                g[j] = ok ? ld : f4{0, 0, 0, 0};
            }
            const f4 *xn = (const f4 *)x + (int64_t)n * H * W * C4 + cv;
            const int h0 = p * STRIDE - 1, v0 = q0 * STRIDE - 1;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int h = h0 + r;
                const bool hok = (unsigned)h < (unsigned)H;
                f4 xv[COLS];
#pragma unroll
                for (int c = 0; c < COLS; ++c) {
                    const int v = v0 + c;
                    const bool ok = hok && (unsigned)v < (unsigned)W;
                    const f4 ld = xn[ok ? ((int64_t)h * W + v) * C4 : 0];
                    xv[c] = ok ? ld : f4{0, 0, 0, 0};
                }
#pragma unroll
                for (int sx = 0; sx < 3; ++sx)
#pragma unroll
                    for (int j = 0; j < L; ++j) acc[r * 3 + sx] += xv[j * STRIDE + sx] * g[j];
            }
        }
    }
    const int width = CL * 4;
#pragma unroll
    for (int t = 0; t < 9; ++t) *(f4 *)(red + ((size_t)threadIdx.y * 9 + t) * width + threadIdx.x * 4) = acc[t];
    __syncthreads();
    for (int j = threadIdx.y * CL + threadIdx.x; j < 9 * CL; j += CL * PL) {
        const int t = j / CL, cl = j - t * CL;
        const int c4 = blockIdx.y * CL + cl;
        if (c4 >= C4) continue;
        f4 sum = f4{0, 0, 0, 0};
        for (int l = 0; l < PL; ++l) sum += *(const f4 *)(red + ((size_t)l * 9 + t) * width + cl * 4);
        *(f4 *)(part + ((size_t)blockIdx.x * 9 + t) * C + c4 * 4) = sum;
    }
}

// block shape of the 3x3 kernels: CL channel groups (power of two, at most 64) x PL pixel lanes, 16 pixels per thread
struct Dw3Geom { int CL, PL, chunks; unsigned blocks; int64_t pix_per_block; };
Dw3Geom dw3_geom(int C4, int64_t pixels) {
    Dw3Geom g;
    g.CL = 1;
    while (g.CL < C4 && g.CL < 64) g.CL <<= 1;
    g.PL = 256 / g.CL;
    g.chunks = (C4 + g.CL - 1) / g.CL;
    g.pix_per_block = (int64_t)g.PL * 16;
    int64_t blocks = (pixels + g.pix_per_block - 1) / g.pix_per_block;
    if (blocks > 0x7fffffff) throw KernelError("depthwise: too many pixels");
    g.blocks = (unsigned)std::max<int64_t>(1, blocks);
    return g;
}

void check_dw(const ConvShape &cs, const char *who) {
    if (cs.K != cs.C) throw KernelError(std::string(who) + ": depthwise needs K == C");
    if (cs.R * cs.S > DW_MAX_TAPS) throw KernelError(std::string(who) + ": at most 9 filter taps");
    if (cs.N <= 0 || cs.C <= 0 || cs.P <= 0 || cs.Q <= 0 || cs.stride <= 0) throw KernelError(std::string(who) + ": bad shape");
    if (cs.P != (cs.H + 2 * cs.pad - cs.R) / cs.stride + 1 || cs.Q != (cs.W + 2 * cs.pad - cs.S) / cs.stride + 1)
        throw KernelError(std::string(who) + ": output extent does not match the input");
    if ((size_t)cs.C * cs.R * cs.S * 4 > 64 * 1024) throw KernelError(std::string(who) + ": filters do not fit in LDS");
    if ((int64_t)cs.H * cs.W * cs.C >= (1ll << 31) || (int64_t)cs.P * cs.Q * cs.C >= (1ll << 31))
        throw KernelError(std::string(who) + ": one image must hold fewer than 2^31 elements");
}

}  // namespace

bool dwconv_fwd_takes_affine(const ConvShape &cs) {
    return cs.C % 4 == 0 && cs.R == 3 && cs.S == 3 && cs.pad == 1 && (cs.stride == 1 || cs.stride == 2);
}

void dwconv_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs, const BnAffine *affine) {
    check_dw(cs, "dwconv_fwd");
    const size_t lds = (size_t)cs.C * cs.R * cs.S * 4;
    if (affine && (!dwconv_fwd_takes_affine(cs) || !affine->gamma || !affine->beta || !affine->stats))
        throw KernelError("dwconv_fwd: BatchNorm in the same kernel needs a 3x3 / pad 1 layer of stride 1 or 2 with C % 4 == 0 and all coefficients");
    if (affine && affine->mask) throw KernelError("dwconv_fwd: this kernel does not write a sign code");
    const BnAffine bn = affine ? *affine : BnAffine{};
    if (cs.C % 4 == 0 && cs.R == 3 && cs.S == 3 && cs.pad == 1 && cs.stride == 1) {
        launch_dw3_row<1, 7, false, false>(st, x, w, y, cs.N, cs.H, cs.W, cs.P, cs.Q, cs.C, bn);
    } else if (cs.C % 4 == 0 && cs.R == 3 && cs.S == 3 && cs.pad == 1 && cs.stride == 2) {
        launch_dw3_row<2, 4, false, false>(st, x, w, y, cs.N, cs.H, cs.W, cs.P, cs.Q, cs.C, bn);
    } else if (cs.C % 4 == 0 && cs.R == 3 && cs.S == 3) {
        const Dw3Geom gm = dw3_geom(cs.C / 4, cs.M());
        hipLaunchKernelGGL(dw3_fwd_kernel, dim3(gm.blocks, gm.chunks), dim3(gm.CL, gm.PL), lds, st, x, w, y, cs, gm.pix_per_block);
    } else if (cs.C % 4 == 0) {
        int grid = grid_cap(cs.M() * (cs.C / 4), 256, 8192);
        hipLaunchKernelGGL((dw_fwd_kernel<4>), dim3(grid), dim3(256), lds, st, x, w, y, cs);
    } else {
        int grid = grid_cap(cs.M() * cs.C, 256, 8192);
        hipLaunchKernelGGL((dw_fwd_kernel<1>), dim3(grid), dim3(256), lds, st, x, w, y, cs);
    }
    hip_check(hipGetLastError(), "dwconv_fwd launch");
}

void dwconv_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, const ConvShape &cs, bool accumulate) {
    check_dw(cs, "dwconv_dgrad");
    const size_t lds = (size_t)cs.C * cs.R * cs.S * 4;
    const int64_t pixels = (int64_t)cs.N * cs.H * cs.W;
#define DG(V, ACC) hipLaunchKernelGGL((dw_dgrad_kernel<V, ACC>), dim3(grid), dim3(256), lds, st, dy, w, dx, cs)
    if (cs.C % 4 == 0 && cs.R == 3 && cs.S == 3 && cs.pad == 1 && cs.stride == 1) {
        // stride 1: the forward operator on dy (same extent as dx) with the filter turned by 180 degrees
        if (accumulate) launch_dw3_row<1, 7, true, true>(st, dy, w, dx, cs.N, cs.P, cs.Q, cs.H, cs.W, cs.C);
        else launch_dw3_row<1, 7, true, false>(st, dy, w, dx, cs.N, cs.P, cs.Q, cs.H, cs.W, cs.C);
    } else if (cs.C % 4 == 0 && cs.R == 3 && cs.S == 3 && cs.pad == 1 && cs.stride == 2) {
        constexpr int L = 4;
        const int rows2 = (cs.H + 1) / 2, segs = ((cs.W + 1) / 2 + L - 1) / L;
        const int64_t items = (int64_t)cs.N * rows2 * segs * (cs.C / 4);
        const int64_t blocks = ((items + 255) / 256 + 7) / 8 * 8;
        if (blocks > 0x7fffffffll) throw KernelError("depthwise: too many work items");
        if (accumulate)
            hipLaunchKernelGGL((dw3_dgrad_s2_kernel<L, true>), dim3((unsigned)blocks), dim3(256), 0, st, dy, w, dx, cs.N, cs.H, cs.W, cs.P, cs.Q,
                               cs.C / 4, rows2, segs, items);
        else
            hipLaunchKernelGGL((dw3_dgrad_s2_kernel<L, false>), dim3((unsigned)blocks), dim3(256), 0, st, dy, w, dx, cs.N, cs.H, cs.W, cs.P, cs.Q,
                               cs.C / 4, rows2, segs, items);
    } else if (cs.C % 4 == 0 && cs.R == 3 && cs.S == 3) {
        const Dw3Geom gm = dw3_geom(cs.C / 4, pixels);
        if (accumulate) hipLaunchKernelGGL((dw3_dgrad_kernel<true>), dim3(gm.blocks, gm.chunks), dim3(gm.CL, gm.PL), lds, st, dy, w, dx, cs, gm.pix_per_block);
        else hipLaunchKernelGGL((dw3_dgrad_kernel<false>), dim3(gm.blocks, gm.chunks), dim3(gm.CL, gm.PL), lds, st, dy, w, dx, cs, gm.pix_per_block);
    } else if (cs.C % 4 == 0) {
        int grid = grid_cap(pixels * (cs.C / 4), 256, 8192);
        if (accumulate) DG(4, true); else DG(4, false);
    } else {
        int grid = grid_cap(pixels * cs.C, 256, 8192);
        if (accumulate) DG(1, true); else DG(1, false);
    }
#undef DG
    hip_check(hipGetLastError(), "dwconv_dgrad launch");
}

void dwconv_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, float *scratch, size_t scratch_bytes) {
    check_dw(cs, "dwconv_wgrad");
    const int taps = cs.R * cs.S;
    const int V = cs.C % 4 == 0 ? 4 : 1;
    const int CV = cs.C / V;
    int CL = 1;
    while (CL < CV && CL < 64) CL <<= 1;
    const int PL = 256 / CL;
    const int chunks = (CV + CL - 1) / CL;
    const int64_t M = cs.M();
    const size_t slab_bytes = (size_t)taps * cs.C * 4;
    if (V == 4 && cs.R == 3 && cs.S == 3 && cs.pad == 1 && (cs.stride == 1 || cs.stride == 2)) {
        // channel groups per workgroup: the channels' groups of four divided evenly over as few chunks as a limit of 64 allows,
        // no power of two needed (36 groups: 36 x 7 threads instead of 64 x 4 with 28 idle channel lanes)
        const int chunks = (CV + 63) / 64, CL = (CV + chunks - 1) / chunks, PL = 256 / CL;
        const int L = cs.stride == 1 ? 7 : 4;
        const int segs = (cs.Q + L - 1) / L;
        const int64_t items = (int64_t)cs.N * cs.P * segs;
        // about 2048 workgroups in all, at least eight segments per pixel lane (measured on MobileNetV2 b272: 2, 4, 8, 16
        // segments give 1.76, 1.70, 1.67, 1.81 ms for the class: fewer partial results to write and to add up)
        int64_t slabs = std::min<int64_t>({std::max<int64_t>(1, 2048 / chunks), (int64_t)(scratch_bytes / slab_bytes), (items + 8 * PL - 1) / (8 * PL)});
        if (slabs < 1) throw KernelError("dwconv_wgrad: scratch too small");
        const int64_t per = (items + slabs - 1) / slabs;
        slabs = (items + per - 1) / per;
        const size_t lds = (size_t)PL * 9 * CL * 4 * 4;
        if (lds > 64 * 1024) throw KernelError("dwconv_wgrad: reduction buffer does not fit in LDS");
        if (cs.stride == 1)
            hipLaunchKernelGGL((dw3_wgrad_row_partial<1, 7>), dim3((unsigned)slabs, chunks), dim3(CL, PL), lds, st, x, dy, scratch, cs.N, cs.H, cs.W,
                               cs.P, cs.Q, cs.C, segs, items, per);
        else
            hipLaunchKernelGGL((dw3_wgrad_row_partial<2, 4>), dim3((unsigned)slabs, chunks), dim3(CL, PL), lds, st, x, dy, scratch, cs.N, cs.H, cs.W,
                               cs.P, cs.Q, cs.C, segs, items, per);
        hipLaunchKernelGGL(dw_wgrad_final, dim3((cs.C * taps + 3) / 4), dim3(256), 0, st, (const float *)scratch, dw, cs.C, taps, (int)slabs);
        hip_check(hipGetLastError(), "dwconv_wgrad launch");
        return;
    }
    int64_t slabs = std::min<int64_t>({(int64_t)4096, (int64_t)(scratch_bytes / slab_bytes), (M + 4 * PL - 1) / (4 * PL)});
    if (slabs < 1) throw KernelError("dwconv_wgrad: scratch too small");
    const int64_t pps = (M + slabs - 1) / slabs;
    slabs = (M + pps - 1) / pps;
    const size_t lds = (size_t)PL * taps * CL * V * 4;
    if (lds > 64 * 1024) throw KernelError("dwconv_wgrad: reduction buffer does not fit in LDS");
    if (V == 4 && cs.R == 3 && cs.S == 3) hipLaunchKernelGGL(dw3_wgrad_partial, dim3((unsigned)slabs, chunks), dim3(CL, PL), lds, st, x, dy, scratch, cs, pps);
    else if (V == 4) hipLaunchKernelGGL((dw_wgrad_partial<4>), dim3((unsigned)slabs, chunks), dim3(CL, PL), lds, st, x, dy, scratch, cs, pps);
    else hipLaunchKernelGGL((dw_wgrad_partial<1>), dim3((unsigned)slabs, chunks), dim3(CL, PL), lds, st, x, dy, scratch, cs, pps);
    hipLaunchKernelGGL(dw_wgrad_final, dim3((cs.C * taps + 3) / 4), dim3(256), 0, st, (const float *)scratch, dw, cs.C, taps, (int)slabs);
    hip_check(hipGetLastError(), "dwconv_wgrad launch");
}

// ------------------------------------------------------------------ copies between row lengths
namespace {

template <int V, bool ACC>
__global__ __launch_bounds__(256) void column_copy_kernel(const float *__restrict__ src, int64_t src_ld, float *dst, int64_t dst_ld, int cols,
                                                          int64_t rows) {
    const int CV = cols / V;
    const int64_t total = rows * CV;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = i / CV;
        const int c = (int)(i - row * CV) * V;
        const float *s = src + row * src_ld + c;
        float *d = dst + row * dst_ld + c;
        if (V == 4) {
            float4 v = ld4(s);
            if (ACC) { float4 o = *(float4 *)d; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
            *(float4 *)d = v;
        } else {
            d[0] = ACC ? d[0] + s[0] : s[0];
        }
    }
}

}  // namespace

// dst[row][0..cols) (+)= src[row][0..cols), rows of src / dst are src_ld / dst_ld floats apart (the caller
// offsets the base pointers to the first column).
void column_copy(hipStream_t st, const float *src, int64_t src_ld, float *dst, int64_t dst_ld, int cols, int64_t rows, bool accumulate) {
    if (rows <= 0 || cols <= 0) return;
    if (src_ld < cols || dst_ld < cols) throw KernelError("column_copy: row length shorter than the copied columns");
    const bool vec = cols % 4 == 0 && src_ld % 4 == 0 && dst_ld % 4 == 0 && ((uintptr_t)src % 16) == 0 && ((uintptr_t)dst % 16) == 0;
#define CC(V, ACC) hipLaunchKernelGGL((column_copy_kernel<V, ACC>), dim3(grid), dim3(256), 0, st, src, src_ld, dst, dst_ld, cols, rows)
    if (vec) {
        int grid = grid_cap(rows * (cols / 4), 256 * 4, 8192);
        if (accumulate) CC(4, true); else CC(4, false);
    } else {
        int grid = grid_cap(rows * cols, 256 * 4, 8192);
        if (accumulate) CC(1, true); else CC(1, false);
    }
#undef CC
    hip_check(hipGetLastError(), "column_copy launch");
}

// ------------------------------------------------------------------ cross-entropy over many short rows
namespace {

constexpr int CE_BLOCKS = 1024;

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

// one thread per row; per-block partial sums of the row losses, fixed order
__global__ __launch_bounds__(256) void ce_rows_fwd_kernel(const float *__restrict__ logits, const int32_t *__restrict__ labels,
                                                          float *__restrict__ part, int64_t rows, int classes) {
    __shared__ float sh[4];
    float mine = 0;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += (int64_t)gridDim.x * blockDim.x) {
        const float *z = logits + r * classes;
        float m = z[0];
        for (int c = 1; c < classes; ++c) m = fmaxf(m, z[c]);
        float s = 0;
        for (int c = 0; c < classes; ++c) s += expf(z[c] - m);
        mine += logf(s) - (z[labels[r]] - m);
    }
    mine = wave_sum(mine);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__global__ __launch_bounds__(256) void ce_rows_final_kernel(const float *__restrict__ part, float *__restrict__ loss, int n, float scale) {
    __shared__ double sh[256];
    double s = 0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) s += (double)part[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = (float)(sh[0] * (double)scale);
}

template <bool ACC>
__global__ __launch_bounds__(256) void ce_rows_bwd_kernel(const float *__restrict__ logits, const int32_t *__restrict__ labels, float *dlogits,
                                                          int64_t rows, int classes, float inv_rows) {
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += (int64_t)gridDim.x * blockDim.x) {
        const float *z = logits + r * classes;
        float m = z[0];
        for (int c = 1; c < classes; ++c) m = fmaxf(m, z[c]);
        float s = 0;
        for (int c = 0; c < classes; ++c) s += expf(z[c] - m);
        const float inv = 1.0f / s;
        const int lab = labels[r];
        float *d = dlogits + r * classes;
        for (int c = 0; c < classes; ++c) {
            float g = (expf(z[c] - m) * inv - (c == lab ? 1.0f : 0.0f)) * inv_rows;
            d[c] = ACC ? d[c] + g : g;
        }
    }
}

}  // namespace

void softmaxce_rows_fwd(hipStream_t st, const float *logits, const int32_t *labels, float *loss, int64_t rows, int classes, float *scratch,
                        size_t scratch_bytes) {
    if (rows <= 0 || classes <= 0) throw KernelError("softmaxce: bad shape");
    int grid = grid_cap(rows, 256, CE_BLOCKS);
    if ((size_t)grid * 4 > scratch_bytes) throw KernelError("softmaxce: scratch too small");
    hipLaunchKernelGGL(ce_rows_fwd_kernel, dim3(grid), dim3(256), 0, st, logits, labels, scratch, rows, classes);
    hipLaunchKernelGGL(ce_rows_final_kernel, dim3(1), dim3(256), 0, st, (const float *)scratch, loss, grid, 1.0f / (float)rows);
    hip_check(hipGetLastError(), "softmaxce rows forward launch");
}

void softmaxce_rows_bwd(hipStream_t st, const float *logits, const int32_t *labels, float *dlogits, int64_t rows, int classes, bool accumulate) {
    if (rows <= 0 || classes <= 0) throw KernelError("softmaxce: bad shape");
    int grid = grid_cap(rows, 256, 8192);
    if (accumulate) hipLaunchKernelGGL((ce_rows_bwd_kernel<true>), dim3(grid), dim3(256), 0, st, logits, labels, dlogits, rows, classes, 1.0f / (float)rows);
    else hipLaunchKernelGGL((ce_rows_bwd_kernel<false>), dim3(grid), dim3(256), 0, st, logits, labels, dlogits, rows, classes, 1.0f / (float)rows);
    hip_check(hipGetLastError(), "softmaxce rows backward launch");
}

}  // namespace monet
