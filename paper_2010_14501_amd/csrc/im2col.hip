// Convolution through an explicit patch matrix (the third workspace-for-time form of Section 4, "Forward Operator
// Optimization", after the split reduction and the Winograd forms; Appendix I lists it among the library algorithms
// the solver chooses from).  The input patches of a chunk of whole images are written out as the rows of a matrix
// col[(n, p, q)][(r, s, c)], then the layer is one plain GEMM on the tile kernel of conv.hip (a 1x1 convolution with
// R*S*C input channels): forward y = col W^T, filter gradient dW = dy^T col.  The workspace argument decides the
// chunk: the smaller it is, the more chunks a layer is worked through in.
//
// Layout of the workspace: [padded filters K x ld] [col: rows x ld] [filter gradient only: K x ld result of a chunk and
// the partial results of its split reduction], ld = R*S*C rounded up to 16 floats (zero filled), so that the GEMM
// always takes its aligned loader.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "kernels.hpp"

namespace monet {
namespace {

constexpr int64_t COL_CHUNK_BYTES = (int64_t)256 << 20;     // recommended patch matrix of one chunk

inline int ld_of(const ConvShape &cs) { return (int)((cs.RSC() + 15) / 16 * 16); }

// one thread per group of four consecutive floats of a col row (VEC: C % 4 == 0, a group lies inside one tap and is
// loaded as 16 bytes; otherwise element by element)
template <bool VEC>
__global__ __launch_bounds__(256) void im2col_kernel(const float *__restrict__ x, float *__restrict__ col, ConvShape cs, int64_t rows, int ld) {
    const int ld4 = ld / 4;
    const int64_t total = rows * ld4;
    const int RSC = (int)cs.RSC();
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / ld4;
        const int kk = (int)(i - row * ld4) * 4;
        const unsigned m = (unsigned)row, t = m / (unsigned)cs.Q;
        const int q = (int)(m - t * (unsigned)cs.Q), p = (int)(t % (unsigned)cs.P), n = (int)(t / (unsigned)cs.P);
        const int h0 = p * cs.stride - cs.pad, w0 = q * cs.stride - cs.pad;
        float4 v = make_float4(0, 0, 0, 0);
        if (VEC) {
            if (kk < RSC) {
                const int tap = kk / cs.C, c = kk - tap * cs.C, r = tap / cs.S, s = tap - r * cs.S;
                const int h = h0 + r, w = w0 + s;
                if ((unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                    v = *(const float4 *)(x + (((int64_t)n * cs.H + h) * cs.W + w) * cs.C + c);
            }
        } else {
            float e[4] = {0, 0, 0, 0};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k1 = kk + u;
                if (k1 < RSC) {
                    const int tap = k1 / cs.C, c = k1 - tap * cs.C, r = tap / cs.S, s = tap - r * cs.S;
                    const int h = h0 + r, w = w0 + s;
                    if ((unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W) e[u] = x[(((int64_t)n * cs.H + h) * cs.W + w) * cs.C + c];
                }
            }
            v = make_float4(e[0], e[1], e[2], e[3]);
        }
        *(float4 *)(col + i * 4) = v;
    }
}

void im2col(hipStream_t st, const float *x, float *col, const ConvShape &part, int ld) {
    const int64_t rows = part.M(), total = rows * (ld / 4);
    const unsigned grid = (unsigned)std::min<int64_t>((total + 255) / 256, 256 * 32);
    if (part.C % 4 == 0) hipLaunchKernelGGL(im2col_kernel<true>, dim3(grid), dim3(256), 0, st, x, col, part, rows, ld);
    else hipLaunchKernelGGL(im2col_kernel<false>, dim3(grid), dim3(256), 0, st, x, col, part, rows, ld);
    hip_check(hipGetLastError(), "im2col launch");
}

// the layer as a 1x1 convolution over `rows` positions with ld input channels
ConvShape gemm_shape(int64_t rows, int ld, int K) { return ConvShape{1, 1, (int)rows, ld, K, 1, 1, 1, 0, 1, (int)rows}; }

struct ColPlan {
    int ld;
    int64_t wpad;        // floats of the padded filter copy (0: the filters are used where they are)
    int64_t per_img;     // col floats per image
    int imgs;            // images per chunk
    int splits;          // filter gradient: reduction ranges of a chunk's GEMM
    int64_t tail;        // filter gradient: floats after col (chunk result + partial results)
};

int even_chunk(int N, int cap) {
    if (cap < 1) return 0;
    const int chunks = (N + cap - 1) / cap;
    return (N + chunks - 1) / chunks;
}

ColPlan col_plan(const ConvShape &cs, bool wgrad, size_t ws_bytes, bool recommend) {
    ColPlan cp{};
    cp.ld = ld_of(cs);
    cp.wpad = (!wgrad && cp.ld != cs.RSC()) ? (int64_t)cs.K * cp.ld : 0;
    cp.per_img = (int64_t)cs.P * cs.Q * cp.ld;
    // rows of a chunk stay below 2^31 / 16 so that the GEMM's 32-bit byte offsets span col and the output
    const int64_t span = (((int64_t)1 << 30) - ((int64_t)1 << 18)) / std::max(cp.ld, cs.K);
    const int span_imgs = (int)std::min<int64_t>(cs.N, span / ((int64_t)cs.P * cs.Q));
    auto tail_of = [&](int imgs, int &splits) {
        if (!wgrad) { splits = 1; return (int64_t)0; }
        const int64_t steps = ((int64_t)imgs * cs.P * cs.Q + 15) / 16;
        const int64_t tiles = (int64_t)((cs.K + 127) / 128) * ((cp.ld + 127) / 128);
        splits = (int)std::max<int64_t>(1, std::min<int64_t>({(512 + tiles - 1) / tiles, steps / 4, 256}));
        return (int64_t)cs.K * cp.ld * (1 + (splits > 1 ? splits : 0));
    };
    if (recommend) {
        cp.imgs = (int)std::max<int64_t>(1, std::min<int64_t>(cs.N, COL_CHUNK_BYTES / 4 / cp.per_img));
        cp.imgs = even_chunk(cs.N, std::min(cp.imgs, std::max(span_imgs, 1)));
        cp.tail = tail_of(cp.imgs, cp.splits);
        return cp;
    }
    // the largest chunk the given workspace holds (the tail grows with the chunk only through the split count: bisect)
    const int64_t have = (int64_t)(ws_bytes / sizeof(float)) - cp.wpad;
    int lo = 0, hi = std::min(cs.N, std::max(span_imgs, 0)) + 1;
    while (hi - lo > 1) {
        const int mid = (lo + hi) / 2;
        int sp;
        if ((int64_t)mid * cp.per_img + tail_of(mid, sp) <= have) lo = mid; else hi = mid;
    }
    cp.imgs = even_chunk(cs.N, lo);
    cp.tail = cp.imgs ? tail_of(cp.imgs, cp.splits) : 0;
    return cp;
}

// filters [K][RSC] -> [K][ld], zero filled
__global__ __launch_bounds__(256) void pad_rows_kernel(const float *__restrict__ src, float *__restrict__ dst, int rows, int cols, int ld) {
    const int64_t total = (int64_t)rows * ld;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int r = (int)(i / ld), c = (int)(i - (int64_t)r * ld);
        dst[i] = c < cols ? src[(int64_t)r * cols + c] : 0.0f;
    }
}

void check(const ConvShape &cs, const char *who) {
    if (cs.N < 1 || cs.P < 1 || cs.Q < 1 || cs.C < 1 || cs.K < 1 || cs.K % 4 != 0)
        throw KernelError(std::string(who) + ": needs a non-empty layer with a multiple of four output channels");
    if ((int64_t)cs.P * cs.Q >= ((int64_t)1 << 31) / 16) throw KernelError(std::string(who) + ": image too large");
}

}  // namespace

bool conv_im2col_applies(const ConvShape &cs) { return cs.K % 4 == 0 && cs.R * cs.S > 1; }

size_t conv_im2col_workspace_bytes(const ConvShape &cs, bool wgrad) {
    check(cs, "conv_im2col_workspace_bytes");
    const ColPlan cp = col_plan(cs, wgrad, 0, true);
    return (size_t)(cp.wpad + (int64_t)cp.imgs * cp.per_img + cp.tail) * sizeof(float);
}

void conv_im2col_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs, float *ws, size_t ws_bytes,
                     bool accumulate) {
    check(cs, "conv_im2col_fwd");
    const ColPlan cp = col_plan(cs, false, ws_bytes, false);
    if (!ws || cp.imgs < 1) throw KernelError("conv_im2col_fwd: workspace too small for the patches of one image");
    const float *wp = w;
    float *col = ws;
    if (cp.wpad) {
        hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)std::min<int64_t>((cp.wpad + 255) / 256, 4096)), dim3(256), 0, st, w, ws, cs.K,
                           (int)cs.RSC(), cp.ld);
        hip_check(hipGetLastError(), "filter padding launch");
        wp = ws;
        col = ws + cp.wpad;
    }
    for (int img0 = 0; img0 < cs.N; img0 += cp.imgs) {
        ConvShape part = cs;
        part.N = std::min(cp.imgs, cs.N - img0);
        im2col(st, x + (int64_t)img0 * cs.H * cs.W * cs.C, col, part, cp.ld);
        conv_fwd(st, col, wp, y + (int64_t)img0 * cs.P * cs.Q * cs.K, gemm_shape(part.M(), cp.ld, cs.K), 1, nullptr, 0, accumulate);
    }
}

void conv_im2col_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, float *ws, size_t ws_bytes) {
    check(cs, "conv_im2col_wgrad");
    const ColPlan cp = col_plan(cs, true, ws_bytes, false);
    if (!ws || cp.imgs < 1) throw KernelError("conv_im2col_wgrad: workspace too small for the patches of one image");
    float *col = ws, *res = col + (int64_t)cp.imgs * cp.per_img, *parts = res + (int64_t)cs.K * cp.ld;
    const int RSC = (int)cs.RSC();
    for (int img0 = 0; img0 < cs.N; img0 += cp.imgs) {
        ConvShape part = cs;
        part.N = std::min(cp.imgs, cs.N - img0);
        im2col(st, x + (int64_t)img0 * cs.H * cs.W * cs.C, col, part, cp.ld);
        // the chunk's share of the gradient, [K][ld]; its first R*S*C columns are added to dw in chunk order
        const int64_t steps = (part.M() + 15) / 16;
        const int splits = (int)std::max<int64_t>(1, std::min<int64_t>(cp.splits, steps));
        conv_wgrad(st, col, dy + (int64_t)img0 * cs.P * cs.Q * cs.K, res, gemm_shape(part.M(), cp.ld, cs.K), splits,
                   splits > 1 ? parts : nullptr, splits > 1 ? (size_t)splits * cs.K * cp.ld * sizeof(float) : 0);
        column_copy(st, res, cp.ld, dw, RSC, RSC, cs.K, img0 > 0);
    }
}

}  // namespace monet
