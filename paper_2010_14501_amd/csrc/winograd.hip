// Winograd F(2x2, 3x3) convolution for 3x3 / stride 1 / pad 1 layers: the workspace-hungry, arithmetic-lean
// alternative to the implicit GEMM (the paper's Section 4 names Winograd among the implementations an operator can
// choose from; Appendix D's trade-off of workspace against time).
//
//   Y = A^T [ (G g G^T) .* (B^T d B) ] A      per 4x4 input tile d, 3x3 filter g, 2x2 output tile Y
//   B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]   G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]   A^T = [1 1 1 0; 0 1 -1 -1]
//
// Four kernels: filter transform U[16][Kout][Cred], input transform V[16][T][Cred] (T = N * ceil(H/2) * ceil(W/2)
// tiles), sixteen GEMMs M[z] = V[z] U[z]^T on the matrix cores (one launch of the implicit-GEMM kernel, z in
// gridDim.z), output transform.  2.25x fewer multiplications than the direct form, paid for with 4x the input plus
// 4x the output as workspace and the traffic to fill and drain it, so it pays where channels are many and maps
// small.  The input gradient of such a layer is the same computation on dy with the filter turned by 180 degrees
// and its two channel axes exchanged (`adjoint`).
#include "kernels.hpp"

namespace monet {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// one thread per (output channel row, reduction channel column) of the 16 transformed filters
// (ADJ, here and below: forward pass or input gradient -- two names in a profile, and for the filter two layouts)
template <bool ADJ>
__global__ __launch_bounds__(256) void wino_filter_kernel(const float *__restrict__ w, float *__restrict__ U, int K, int C) {
    constexpr int adjoint = ADJ ? 1 : 0;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int rows = adjoint ? C : K, cols = adjoint ? K : C;
    if (idx >= (int64_t)rows * cols) return;
    const int row = (int)(idx / cols), col = (int)(idx % cols);
    float g[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s)
            g[r][s] = adjoint ? w[((int64_t)col * 9 + (2 - r) * 3 + (2 - s)) * C + row] : w[((int64_t)row * 9 + r * 3 + s) * C + col];
    float t[4][3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        t[0][s] = g[0][s];
        t[1][s] = 0.5f * (g[0][s] + g[1][s] + g[2][s]);
        t[2][s] = 0.5f * (g[0][s] - g[1][s] + g[2][s]);
        t[3][s] = g[2][s];
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const float u0 = t[a][0], u1 = 0.5f * (t[a][0] + t[a][1] + t[a][2]), u2 = 0.5f * (t[a][0] - t[a][1] + t[a][2]), u3 = t[a][2];
        const int64_t plane = (int64_t)rows * cols;
        U[(4 * a + 0) * plane + idx] = u0;
        U[(4 * a + 1) * plane + idx] = u1;
        U[(4 * a + 2) * plane + idx] = u2;
        U[(4 * a + 3) * plane + idx] = u3;
    }
}

struct WinoGeom {
    int N, H, W, th, tw;
    int64_t T;
};

// one thread per (tile, four channels): V[z][tile][c] = (B^T d B)[z]
// USE (a name in profiles only): 0 forward pass, 1 input gradient, 2 filter gradient
template <int USE>
__global__ __launch_bounds__(256) void wino_input_kernel(const float *__restrict__ x, float *__restrict__ V, WinoGeom gm, int C) {
    const int C4 = C / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= gm.T * C4) return;
    const int c4 = (int)(idx % C4);
    const int64_t t = idx / C4;
    const int tj = (int)(t % gm.tw);
    const int64_t r = t / gm.tw;
    const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
    const int h0 = 2 * ti - 1, w0 = 2 * tj - 1;
    f4 d[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int h = h0 + a, w = w0 + b;
            d[a][b] = f4{0, 0, 0, 0};
            if ((unsigned)h < (unsigned)gm.H && (unsigned)w < (unsigned)gm.W)
                d[a][b] = *(const f4 *)(x + (((int64_t)n * gm.H + h) * gm.W + w) * C + 4 * c4);
        }
    f4 m[4][4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {      // B^T d
        m[0][b] = d[0][b] - d[2][b];
        m[1][b] = d[1][b] + d[2][b];
        m[2][b] = d[2][b] - d[1][b];
        m[3][b] = d[1][b] - d[3][b];
    }
    const int64_t plane = gm.T * C;
    float *dst = V + t * C + 4 * c4;
#pragma unroll
    for (int a = 0; a < 4; ++a) {      // (.) B
        *(f4 *)(dst + (4 * a + 0) * plane) = m[a][0] - m[a][2];
        *(f4 *)(dst + (4 * a + 1) * plane) = m[a][1] + m[a][2];
        *(f4 *)(dst + (4 * a + 2) * plane) = m[a][2] - m[a][1];
        *(f4 *)(dst + (4 * a + 3) * plane) = m[a][1] - m[a][3];
    }
}

// one thread per (tile, four channels): the 2x2 outputs A^T m A, written or accumulated
template <bool ADJ>
__global__ __launch_bounds__(256) void wino_output_kernel(const float *__restrict__ M, float *y, WinoGeom gm, int K, int accumulate) {
    const int K4 = K / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= gm.T * K4) return;
    const int k4 = (int)(idx % K4);
    const int64_t t = idx / K4;
    const int tj = (int)(t % gm.tw);
    const int64_t r = t / gm.tw;
    const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
    const int64_t plane = gm.T * K;
    const float *src = M + t * K + 4 * k4;
    f4 m[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) m[a][b] = *(const f4 *)(src + (4 * a + b) * plane);
    f4 s[2][4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {      // A^T m
        s[0][b] = m[0][b] + m[1][b] + m[2][b];
        s[1][b] = m[1][b] - m[2][b] - m[3][b];
    }
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int h = 2 * ti + a;
        if (h >= gm.H) continue;
        const f4 o[2] = {s[a][0] + s[a][1] + s[a][2], s[a][1] - s[a][2] - s[a][3]};
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int w = 2 * tj + b;
            if (w >= gm.W) continue;
            f4 *dst = (f4 *)(y + (((int64_t)n * gm.H + h) * gm.W + w) * K + 4 * k4);
            *dst = accumulate ? *dst + o[b] : o[b];
        }
    }
}

// one thread per (tile, four channels): D[z][tile][k] = (A dy A^T)[z] for the 2x2 output-gradient tile, A = [1 0; 1 1; 1 -1; 0 -1]
__global__ __launch_bounds__(256) void wino_dy_kernel(const float *__restrict__ dy, float *__restrict__ D, WinoGeom gm, int K) {
    const int K4 = K / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= gm.T * K4) return;
    const int k4 = (int)(idx % K4);
    const int64_t t = idx / K4;
    const int tj = (int)(t % gm.tw);
    const int64_t r = t / gm.tw;
    const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
    f4 e[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int h = 2 * ti + a, w = 2 * tj + b;
            e[a][b] = f4{0, 0, 0, 0};
            if (h < gm.H && w < gm.W) e[a][b] = *(const f4 *)(dy + (((int64_t)n * gm.H + h) * gm.W + w) * K + 4 * k4);
        }
    f4 m[4][2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {      // A dy
        m[0][b] = e[0][b];
        m[1][b] = e[0][b] + e[1][b];
        m[2][b] = e[0][b] - e[1][b];
        m[3][b] = -e[1][b];
    }
    const int64_t plane = gm.T * K;
    float *dst = D + t * K + 4 * k4;
#pragma unroll
    for (int a = 0; a < 4; ++a) {      // (.) A^T
        *(f4 *)(dst + (4 * a + 0) * plane) = m[a][0];
        *(f4 *)(dst + (4 * a + 1) * plane) = m[a][0] + m[a][1];
        *(f4 *)(dst + (4 * a + 2) * plane) = m[a][0] - m[a][1];
        *(f4 *)(dst + (4 * a + 3) * plane) = -m[a][1];
    }
}

// one thread per (k, c): dw[k][r][s][c] = (G^T dU G)[r][s]
__global__ __launch_bounds__(256) void wino_filter_back_kernel(const float *__restrict__ dU, float *__restrict__ dw, int K, int C) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t plane = (int64_t)K * C;
    if (idx >= plane) return;
    const int k = (int)(idx / C), c = (int)(idx % C);
    float u[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) u[a][b] = dU[(4 * a + b) * plane + idx];
    float t[3][4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {      // G^T dU
        t[0][b] = u[0][b] + 0.5f * (u[1][b] + u[2][b]);
        t[1][b] = 0.5f * (u[1][b] - u[2][b]);
        t[2][b] = 0.5f * (u[1][b] + u[2][b]) + u[3][b];
    }
#pragma unroll
    for (int r = 0; r < 3; ++r) {      // (.) G
        float *dst = dw + ((int64_t)k * 9 + r * 3) * C + c;
        dst[0] = t[r][0] + 0.5f * (t[r][1] + t[r][2]);
        dst[C] = 0.5f * (t[r][1] - t[r][2]);
        dst[2 * C] = 0.5f * (t[r][1] + t[r][2]) + t[r][3];
    }
}

WinoGeom geom_of(const ConvShape &cs) {
    WinoGeom gm;
    gm.N = cs.N; gm.H = cs.H; gm.W = cs.W;
    gm.th = (cs.H + 1) / 2; gm.tw = (cs.W + 1) / 2;
    gm.T = (int64_t)cs.N * gm.th * gm.tw;
    return gm;
}

}  // namespace

bool winograd_applies(const ConvShape &cs, bool adjoint) {
    if (cs.R != 3 || cs.S != 3 || cs.stride != 1 || cs.pad != 1) return false;
    const int red = adjoint ? cs.K : cs.C, out = adjoint ? cs.C : cs.K;
    return red % 16 == 0 && out % 4 == 0;
}

size_t winograd_workspace_bytes(const ConvShape &cs) {
    const WinoGeom gm = geom_of(cs);
    return (size_t)16 * ((size_t)cs.K * cs.C + (size_t)gm.T * cs.C + (size_t)gm.T * cs.K) * sizeof(float);
}

// adjoint = false: y[N,H,W,K] (+)= conv3x3(x[N,H,W,C], w[K,3,3,C]);  adjoint = true: in = dy[N,H,W,K], out = dx[N,H,W,C] (+)=
void conv_winograd(hipStream_t st, const float *in, const float *w, float *out, const ConvShape &cs, bool adjoint, bool accumulate,
                   float *ws, size_t ws_bytes) {
    if (!winograd_applies(cs, adjoint)) throw KernelError("conv_winograd: needs a 3x3 / stride 1 / pad 1 layer with aligned channel counts");
    if (!ws || ws_bytes < winograd_workspace_bytes(cs)) throw KernelError("conv_winograd: workspace too small");
    const WinoGeom gm = geom_of(cs);
    const int red = adjoint ? cs.K : cs.C, outc = adjoint ? cs.C : cs.K;
    if (gm.T * (std::max(red, outc) / 4) / 256 >= 0x7fffffffll || gm.T >= (1 << 24)) throw KernelError("conv_winograd: shape too large");
    float *U = ws, *V = U + (size_t)16 * cs.K * cs.C, *M = V + (size_t)16 * gm.T * red;
    const int64_t fe = (int64_t)cs.K * cs.C, ie = gm.T * (red / 4), oe = gm.T * (outc / 4);
    const dim3 fg((unsigned)((fe + 255) / 256)), ig((unsigned)((ie + 255) / 256)), og((unsigned)((oe + 255) / 256)), blk(256);
    if (adjoint) {
        hipLaunchKernelGGL(wino_filter_kernel<true>, fg, blk, 0, st, w, U, cs.K, cs.C);
        hipLaunchKernelGGL(wino_input_kernel<1>, ig, blk, 0, st, in, V, gm, red);
    } else {
        hipLaunchKernelGGL(wino_filter_kernel<false>, fg, blk, 0, st, w, U, cs.K, cs.C);
        hipLaunchKernelGGL(wino_input_kernel<0>, ig, blk, 0, st, in, V, gm, red);
    }
    hip_check(hipGetLastError(), "winograd transform launch");
    gemm_batched(st, V, U, M, 16, gm.T, outc, red, adjoint);
    if (adjoint) hipLaunchKernelGGL(wino_output_kernel<true>, og, blk, 0, st, (const float *)M, out, gm, outc, accumulate ? 1 : 0);
    else hipLaunchKernelGGL(wino_output_kernel<false>, og, blk, 0, st, (const float *)M, out, gm, outc, accumulate ? 1 : 0);
    hip_check(hipGetLastError(), "winograd output launch");
}

namespace {
// ranges of tiles per GEMM of the filter gradient: 16 x (K/128) x (C/128) output tiles, about 1024 workgroups in all,
// at least eight reduction steps each
int wgrad_ranges(const ConvShape &cs, int64_t T) {
    const int64_t tiles = 16 * ((cs.K + 127) / 128) * ((cs.C + 127) / 128);
    return (int)std::max<int64_t>(1, std::min<int64_t>(1024 / tiles, T / 128));
}
}  // namespace

size_t winograd_wgrad_workspace_bytes(const ConvShape &cs) {
    const WinoGeom gm = geom_of(cs);
    const int sp = wgrad_ranges(cs, gm.T);
    const size_t filt = (size_t)16 * cs.K * cs.C;
    return ((size_t)16 * gm.T * (cs.C + cs.K) + filt + (sp > 1 ? (size_t)sp * filt : 0)) * sizeof(float);
}

void conv_winograd_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, float *ws, size_t ws_bytes) {
    if (cs.R != 3 || cs.S != 3 || cs.stride != 1 || cs.pad != 1 || cs.C % 4 || cs.K % 4)
        throw KernelError("conv_winograd_wgrad: needs a 3x3 / stride 1 / pad 1 layer with channel counts that are multiples of 4");
    if (!ws || ws_bytes < winograd_wgrad_workspace_bytes(cs)) throw KernelError("conv_winograd_wgrad: workspace too small");
    const WinoGeom gm = geom_of(cs);
    if (gm.T * (std::max(cs.C, cs.K) / 4) / 256 >= 0x7fffffffll || gm.T >= (1 << 24)) throw KernelError("conv_winograd_wgrad: shape too large");
    const int sp = wgrad_ranges(cs, gm.T);
    const size_t filt = (size_t)16 * cs.K * cs.C;
    float *V = ws, *D = V + (size_t)16 * gm.T * cs.C, *dU = D + (size_t)16 * gm.T * cs.K, *slabs = dU + filt;
    const int64_t ie = gm.T * (cs.C / 4), de = gm.T * (cs.K / 4), fe = (int64_t)cs.K * cs.C;
    hipLaunchKernelGGL(wino_input_kernel<2>, dim3((unsigned)((ie + 255) / 256)), dim3(256), 0, st, x, V, gm, cs.C);
    hipLaunchKernelGGL(wino_dy_kernel, dim3((unsigned)((de + 255) / 256)), dim3(256), 0, st, dy, D, gm, cs.K);
    hip_check(hipGetLastError(), "winograd transform launch");
    gemm_tn_batched(st, D, V, dU, 16, gm.T, cs.K, cs.C, sp, sp > 1 ? slabs : nullptr, sp > 1 ? (size_t)sp * filt * sizeof(float) : 0);
    hipLaunchKernelGGL(wino_filter_back_kernel, dim3((unsigned)((fe + 255) / 256)), dim3(256), 0, st, (const float *)dU, dw, cs.K, cs.C);
    hip_check(hipGetLastError(), "winograd filter gradient launch");
}

}  // namespace monet
