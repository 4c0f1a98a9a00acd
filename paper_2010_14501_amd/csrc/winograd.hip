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
//
// The same scheme with 4x4 output tiles, F(4x4, 3x3), is the second set of kernels below: 6x6 input tiles, 36 GEMMs,
// 4x fewer multiplications than the direct form and 2.25x the input plus 2.25x the output as workspace (Lavin and
// Gray's matrices for the interpolation points 0, +-1, +-2 and infinity).  Its transforms have entries up to 8 and
// down to 1/24, so it rounds about five times more coarsely than F(2x2, 3x3) (normwise error of one layer about 2e-6 against
// 4e-7); both stay far inside the tolerances the parity tests use.
#include "bn_affine.hpp"
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
__global__ __launch_bounds__(256) void wino_output_kernel(const float *__restrict__ M, float *y, WinoGeom gm, int K, int accumulate, BnAffine bn) {
    const int K4 = K / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= gm.T * K4) return;
    const int k4 = (int)(idx % K4);
    float bn_a[4] = {1, 1, 1, 1}, bn_b[4] = {0, 0, 0, 0};
    if (!ADJ && bn.gamma) {
#pragma unroll
        for (int j = 0; j < 4; ++j) bn_affine_coeffs(bn.gamma, bn.beta, bn.stats, K, 4 * k4 + j, bn_a[j], bn_b[j]);
    }
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
            f4 v = accumulate ? *dst + o[b] : o[b];
            if (!ADJ && bn.gamma) v = f4{bn_affine(v.x, bn_a[0], bn_b[0]), bn_affine(v.y, bn_a[1], bn_b[1]), bn_affine(v.z, bn_a[2], bn_b[2]), bn_affine(v.w, bn_a[3], bn_b[3])};
            if (!ADJ && bn.gamma && bn.relu) {
                const f4 rv = f4{relu_clamp(v.x, bn.relu), relu_clamp(v.y, bn.relu), relu_clamp(v.z, bn.relu), relu_clamp(v.w, bn.relu)};
                if (bn.relu_out) *(f4 *)(bn.relu_out + ((float *)dst - y)) = rv;
                else v = rv;
            }
            *dst = v;
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

// ---------------------------------------------------------------- F(4x4, 3x3)
typedef float f2 __attribute__((ext_vector_type(2)));

// the five one-dimensional maps of F(4, 3)
//   B^T = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0; 0 2 -1 -2 1 0; 0 4 0 -5 0 1]
//   G   = [1/4 0 0; -1/6 -1/6 -1/6; -1/6 1/6 -1/6; 1/24 1/12 1/6; 1/24 -1/12 1/6; 0 0 1]
//   A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]
template <typename V>
__device__ inline void w4_bt(V v0, V v1, V v2, V v3, V v4, V v5, V (&o)[6]) {
    o[0] = 4.0f * v0 - 5.0f * v2 + v4;
    o[1] = (v3 + v4) - 4.0f * (v1 + v2);
    o[2] = 4.0f * (v1 - v2) + (v4 - v3);
    o[3] = 2.0f * (v3 - v1) + (v4 - v2);
    o[4] = 2.0f * (v1 - v3) + (v4 - v2);
    o[5] = 4.0f * v1 - 5.0f * v3 + v5;
}
__device__ inline void w4_g(float g0, float g1, float g2, float (&o)[6]) {
    o[0] = 0.25f * g0;
    o[1] = (-1.0f / 6.0f) * (g0 + g1 + g2);
    o[2] = (-1.0f / 6.0f) * (g0 - g1 + g2);
    o[3] = (1.0f / 24.0f) * g0 + (1.0f / 12.0f) * g1 + (1.0f / 6.0f) * g2;
    o[4] = (1.0f / 24.0f) * g0 - (1.0f / 12.0f) * g1 + (1.0f / 6.0f) * g2;
    o[5] = g2;
}
template <typename V>
__device__ inline void w4_at(V m0, V m1, V m2, V m3, V m4, V m5, V (&o)[4]) {
    const V p = m1 + m2, q = m1 - m2, r = m3 + m4, t = m3 - m4;
    o[0] = m0 + p + r;
    o[1] = q + 2.0f * t;
    o[2] = p + 4.0f * r;
    o[3] = q + 8.0f * t + m5;
}
template <typename V>
__device__ inline void w4_a(V e0, V e1, V e2, V e3, V (&o)[6]) {      // A e: the transpose of w4_at's map
    o[0] = e0;
    o[1] = (e0 + e2) + (e1 + e3);
    o[2] = (e0 + e2) - (e1 + e3);
    o[3] = (e0 + 4.0f * e2) + (2.0f * e1 + 8.0f * e3);
    o[4] = (e0 + 4.0f * e2) - (2.0f * e1 + 8.0f * e3);
    o[5] = e3;
}
__device__ inline void w4_gt(float u0, float u1, float u2, float u3, float u4, float u5, float (&o)[3]) {   // G^T u
    o[0] = 0.25f * u0 - (1.0f / 6.0f) * (u1 + u2) + (1.0f / 24.0f) * (u3 + u4);
    o[1] = (1.0f / 6.0f) * (u2 - u1) + (1.0f / 12.0f) * (u3 - u4);
    o[2] = (1.0f / 6.0f) * ((u3 + u4) - (u1 + u2)) + u5;
}

// one thread per (output channel row, reduction channel column) of the 36 transformed filters
template <bool ADJ>
__global__ __launch_bounds__(256) void wino4_filter_kernel(const float *__restrict__ w, float *__restrict__ U, int K, int C) {
    constexpr int adjoint = ADJ ? 1 : 0;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int rows = adjoint ? C : K, cols = adjoint ? K : C;
    const int64_t plane = (int64_t)rows * cols;
    if (idx >= plane) return;
    const int row = (int)(idx / cols), col = (int)(idx % cols);
    float g[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s)
            g[r][s] = adjoint ? w[((int64_t)col * 9 + (2 - r) * 3 + (2 - s)) * C + row] : w[((int64_t)row * 9 + r * 3 + s) * C + col];
    float t[3][6];      // t[s][a] = (G g)[a][s]
#pragma unroll
    for (int s = 0; s < 3; ++s) w4_g(g[0][s], g[1][s], g[2][s], t[s]);
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        float u[6];
        w4_g(t[0][a], t[1][a], t[2][a], u);
#pragma unroll
        for (int b = 0; b < 6; ++b) U[(6 * a + b) * plane + idx] = u[b];
    }
}

// one thread per (tile, two channels): V[z][tile][c] = (B^T d B)[z] of the 6x6 input tile
template <int USE>
__global__ __launch_bounds__(256) void wino4_input_kernel(const float *__restrict__ x, float *__restrict__ V, WinoGeom gm, int C) {
    const int C2 = C / 2;
    // a contiguous share of the tiles per XCD (hardware deals workgroups to the 8 XCDs in turn; the grid is a multiple of 8):
    // neighbouring tile rows, which share two of their six input rows, meet in one L2
    const int64_t idx = ((int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) * 256 + threadIdx.x;
    if (idx >= gm.T * C2) return;
    const int c2 = (int)(idx % C2);
    const int64_t t = idx / C2;
    const int tj = (int)(t % gm.tw);
    const int64_t r = t / gm.tw;
    const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
    const int h0 = 4 * ti - 1, w0 = 4 * tj - 1;
    f2 m[6][6];      // m[b][a] = (B^T d)[a][b]
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        f2 d[6];
        const int w = w0 + b;
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            const int h = h0 + a;
            d[a] = f2{0, 0};
            if ((unsigned)h < (unsigned)gm.H && (unsigned)w < (unsigned)gm.W)
                d[a] = *(const f2 *)(x + (((int64_t)n * gm.H + h) * gm.W + w) * C + 2 * c2);
        }
        w4_bt(d[0], d[1], d[2], d[3], d[4], d[5], m[b]);
    }
    const int64_t plane = gm.T * C;
    float *dst = V + t * C + 2 * c2;
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        f2 o[6];
        w4_bt(m[0][a], m[1][a], m[2][a], m[3][a], m[4][a], m[5][a], o);
#pragma unroll
        for (int b = 0; b < 6; ++b) *(f2 *)(dst + (6 * a + b) * plane) = o[b];
    }
}

// one thread per (tile, two channels): the 4x4 outputs A^T m A, written or accumulated
template <bool ADJ>
__global__ __launch_bounds__(256) void wino4_output_kernel(const float *__restrict__ M, float *y, WinoGeom gm, int K, int accumulate, BnAffine bn) {
    const int K2 = K / 2;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= gm.T * K2) return;
    const int k2 = (int)(idx % K2);
    float bn_a[2] = {1, 1}, bn_b[2] = {0, 0};
    if (!ADJ && bn.gamma) {
#pragma unroll
        for (int j = 0; j < 2; ++j) bn_affine_coeffs(bn.gamma, bn.beta, bn.stats, K, 2 * k2 + j, bn_a[j], bn_b[j]);
    }
    const int64_t t = idx / K2;
    const int tj = (int)(t % gm.tw);
    const int64_t r = t / gm.tw;
    const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
    const int64_t plane = gm.T * K;
    const float *src = M + t * K + 2 * k2;
    f2 s[6][4];      // s[b][a] = (A^T m)[a][b]
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        f2 m[6];
#pragma unroll
        for (int a = 0; a < 6; ++a) m[a] = *(const f2 *)(src + (6 * a + b) * plane);
        w4_at(m[0], m[1], m[2], m[3], m[4], m[5], s[b]);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int h = 4 * ti + a;
        if (h >= gm.H) continue;
        f2 o[4];
        w4_at(s[0][a], s[1][a], s[2][a], s[3][a], s[4][a], s[5][a], o);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int w = 4 * tj + b;
            if (w >= gm.W) continue;
            f2 *dst = (f2 *)(y + (((int64_t)n * gm.H + h) * gm.W + w) * K + 2 * k2);
            f2 v = accumulate ? *dst + o[b] : o[b];
            if (!ADJ && bn.gamma) v = f2{bn_affine(v.x, bn_a[0], bn_b[0]), bn_affine(v.y, bn_a[1], bn_b[1])};
            if (!ADJ && bn.gamma && bn.relu) {
                const f2 rv = f2{relu_clamp(v.x, bn.relu), relu_clamp(v.y, bn.relu)};
                if (bn.relu_out) *(f2 *)(bn.relu_out + ((float *)dst - y)) = rv;
                else v = rv;
            }
            *dst = v;
        }
    }
}

// one thread per (tile, two channels): D[z][tile][k] = (A dy A^T)[z] for the 4x4 output-gradient tile
__global__ __launch_bounds__(256) void wino4_dy_kernel(const float *__restrict__ dy, float *__restrict__ D, WinoGeom gm, int K) {
    const int K2 = K / 2;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= gm.T * K2) return;
    const int k2 = (int)(idx % K2);
    const int64_t t = idx / K2;
    const int tj = (int)(t % gm.tw);
    const int64_t r = t / gm.tw;
    const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
    f2 m[4][6];      // m[b][a] = (A dy)[a][b]
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        f2 e[4];
        const int w = 4 * tj + b;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int h = 4 * ti + a;
            e[a] = f2{0, 0};
            if (h < gm.H && w < gm.W) e[a] = *(const f2 *)(dy + (((int64_t)n * gm.H + h) * gm.W + w) * K + 2 * k2);
        }
        w4_a(e[0], e[1], e[2], e[3], m[b]);
    }
    const int64_t plane = gm.T * K;
    float *dst = D + t * K + 2 * k2;
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        f2 o[6];
        w4_a(m[0][a], m[1][a], m[2][a], m[3][a], o);
#pragma unroll
        for (int b = 0; b < 6; ++b) *(f2 *)(dst + (6 * a + b) * plane) = o[b];
    }
}

// one thread per (k, c): dw[k][r][s][c] = (G^T dU G)[r][s]
__global__ __launch_bounds__(256) void wino4_filter_back_kernel(const float *__restrict__ dU, float *__restrict__ dw, int K, int C) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t plane = (int64_t)K * C;
    if (idx >= plane) return;
    const int k = (int)(idx / C), c = (int)(idx % C);
    float t[6][3];      // t[b][r] = (G^T dU)[r][b]
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        float u[6];
#pragma unroll
        for (int a = 0; a < 6; ++a) u[a] = dU[(6 * a + b) * plane + idx];
        w4_gt(u[0], u[1], u[2], u[3], u[4], u[5], t[b]);
    }
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        float o[3];
        w4_gt(t[0][r], t[1][r], t[2][r], t[3][r], t[4][r], t[5][r], o);
        float *dst = dw + ((int64_t)k * 9 + r * 3) * C + c;
        dst[0] = o[0];
        dst[C] = o[1];
        dst[2 * C] = o[2];
    }
}

WinoGeom geom_of(const ConvShape &cs, int m) {
    WinoGeom gm;
    gm.N = cs.N; gm.H = cs.H; gm.W = cs.W;
    gm.th = (cs.H + m - 1) / m; gm.tw = (cs.W + m - 1) / m;
    gm.T = (int64_t)cs.N * gm.th * gm.tw;
    return gm;
}

void check_tile(int m, const char *who) {
    if (m != 2 && m != 4) throw KernelError(std::string(who) + ": output tile edge must be 2 or 4");
}

}  // namespace

bool winograd_applies(const ConvShape &cs, bool adjoint) {
    if (cs.R != 3 || cs.S != 3 || cs.stride != 1 || cs.pad != 1) return false;
    const int red = adjoint ? cs.K : cs.C, out = adjoint ? cs.C : cs.K;
    return red % 16 == 0 && out % 4 == 0;
}

// Workspace: the transformed filters, then the transformed input and the products of one chunk of whole images.
// A layer is worked through in as many chunks as the workspace asks for (the filters are transformed once); chunks
// whose transformed tensors hold about half a GiB cost 0-2 % of time against a single chunk and cap the workspace
// of the largest layers (5 GB for 176 x 112 x 112 x 128) at a tenth -- the knob Appendix D describes.
constexpr size_t WINO_CHUNK_BYTES = (size_t)512 << 20;

namespace {
// the chunks of a layer are made equal: ceil(N / cap) chunks of ceil(N / chunks) images (0 stays 0)
int even_chunk(int N, int cap) {
    if (cap < 1) return 0;
    const int chunks = (N + cap - 1) / cap;
    return (N + chunks - 1) / chunks;
}

struct WinoPlan {
    size_t filt, per_img;      // floats: all transformed filters; transformed input + products of one image
    int imgs;                  // images per chunk
};
WinoPlan wino_plan(const ConvShape &cs, int m, size_t ws_bytes, bool recommend) {
    const int planes = (m + 2) * (m + 2);
    WinoPlan wp;
    wp.filt = (size_t)planes * cs.K * cs.C;
    wp.per_img = (size_t)planes * ((cs.H + m - 1) / m) * ((cs.W + m - 1) / m) * ((size_t)cs.C + cs.K);
    if (recommend) {
        wp.imgs = (int)std::min<size_t>((size_t)cs.N, std::max<size_t>(1, (WINO_CHUNK_BYTES / 4 + wp.per_img - 1) / wp.per_img));
    } else {
        const size_t have = ws_bytes / sizeof(float);
        wp.imgs = have > wp.filt ? (int)std::min<size_t>((size_t)cs.N, (have - wp.filt) / wp.per_img) : 0;
    }
    // the batched GEMMs address one position's plane of a chunk with 32-bit byte offsets
    const size_t plane_img = (size_t)((cs.H + m - 1) / m) * ((cs.W + m - 1) / m) * (size_t)std::max(cs.C, cs.K);
    wp.imgs = (int)std::min<size_t>((size_t)wp.imgs, (((size_t)1 << 30) - ((size_t)1 << 18)) / plane_img);
    wp.imgs = even_chunk(cs.N, wp.imgs);
    return wp;
}
}  // namespace

size_t winograd_workspace_bytes(const ConvShape &cs, int m) {
    check_tile(m, "winograd_workspace_bytes");
    const WinoPlan wp = wino_plan(cs, m, 0, true);
    return (wp.filt + (size_t)wp.imgs * wp.per_img) * sizeof(float);
}

// adjoint = false: y[N,H,W,K] (+)= conv3x3(x[N,H,W,C], w[K,3,3,C]);  adjoint = true: in = dy[N,H,W,K], out = dx[N,H,W,C] (+)=
void conv_winograd(hipStream_t st, const float *in, const float *w, float *out, const ConvShape &cs, int m, bool adjoint, bool accumulate,
                   float *ws, size_t ws_bytes, const BnAffine *affine) {
    check_tile(m, "conv_winograd");
    if (affine && (adjoint || accumulate || !affine->gamma || !affine->beta || !affine->stats))
        throw KernelError("conv_winograd: a BatchNorm apply step goes with the forward form, without accumulation, and needs all coefficients");
    if (affine && affine->mask) throw KernelError("conv_winograd: this form does not write a sign code");
    const BnAffine bn = affine ? *affine : BnAffine{};
    if (!winograd_applies(cs, adjoint)) throw KernelError("conv_winograd: needs a 3x3 / stride 1 / pad 1 layer with aligned channel counts");
    const WinoPlan wp = wino_plan(cs, m, ws_bytes, false);
    if (!ws || wp.imgs < 1) throw KernelError("conv_winograd: workspace too small for the transformed filters and one image");
    const int red = adjoint ? cs.K : cs.C, outc = adjoint ? cs.C : cs.K, planes = (m + 2) * (m + 2), vec = m == 2 ? 4 : 2;
    float *U = ws;
    const int64_t fe = (int64_t)cs.K * cs.C;
    const dim3 fg((unsigned)((fe + 255) / 256)), blk(256);
    if (m == 2) {
        if (adjoint) hipLaunchKernelGGL(wino_filter_kernel<true>, fg, blk, 0, st, w, U, cs.K, cs.C);
        else hipLaunchKernelGGL(wino_filter_kernel<false>, fg, blk, 0, st, w, U, cs.K, cs.C);
    } else {
        if (adjoint) hipLaunchKernelGGL(wino4_filter_kernel<true>, fg, blk, 0, st, w, U, cs.K, cs.C);
        else hipLaunchKernelGGL(wino4_filter_kernel<false>, fg, blk, 0, st, w, U, cs.K, cs.C);
    }
    hip_check(hipGetLastError(), "winograd filter transform launch");
    const int acc = accumulate ? 1 : 0;
    for (int img0 = 0; img0 < cs.N; img0 += wp.imgs) {
        ConvShape part = cs;
        part.N = std::min(wp.imgs, cs.N - img0);
        const WinoGeom gm = geom_of(part, m);
        if (gm.T * (std::max(red, outc) / vec) / 256 >= 0x7fffffffll || gm.T >= (1 << 24)) throw KernelError("conv_winograd: shape too large");
        const float *pin = in + (size_t)img0 * cs.H * cs.W * red;
        float *pout = out + (size_t)img0 * cs.H * cs.W * outc;
        float *V = U + wp.filt, *M = V + (size_t)planes * gm.T * red;
        const int64_t ie = gm.T * (red / vec), oe = gm.T * (outc / vec);
        const dim3 ig((unsigned)(((ie + 255) / 256 + 7) / 8 * 8)), og((unsigned)((oe + 255) / 256));
        if (m == 2) {
            if (adjoint) hipLaunchKernelGGL(wino_input_kernel<1>, ig, blk, 0, st, pin, V, gm, red);
            else hipLaunchKernelGGL(wino_input_kernel<0>, ig, blk, 0, st, pin, V, gm, red);
        } else {
            if (adjoint) hipLaunchKernelGGL(wino4_input_kernel<1>, ig, blk, 0, st, pin, V, gm, red);
            else hipLaunchKernelGGL(wino4_input_kernel<0>, ig, blk, 0, st, pin, V, gm, red);
        }
        hip_check(hipGetLastError(), "winograd transform launch");
        gemm_batched(st, V, U, M, planes, gm.T, outc, red, adjoint);
        if (m == 2) {
            if (adjoint) hipLaunchKernelGGL(wino_output_kernel<true>, og, blk, 0, st, (const float *)M, pout, gm, outc, acc, bn);
            else hipLaunchKernelGGL(wino_output_kernel<false>, og, blk, 0, st, (const float *)M, pout, gm, outc, acc, bn);
        } else {
            if (adjoint) hipLaunchKernelGGL(wino4_output_kernel<true>, og, blk, 0, st, (const float *)M, pout, gm, outc, acc, bn);
            else hipLaunchKernelGGL(wino4_output_kernel<false>, og, blk, 0, st, (const float *)M, pout, gm, outc, acc, bn);
        }
        hip_check(hipGetLastError(), "winograd output launch");
    }
}

namespace {
// ranges of tiles per GEMM of the filter gradient: planes x (K/128) x (C/128) output tiles, about 1024 workgroups in all,
// at least eight reduction steps each
int wgrad_ranges(const ConvShape &cs, int64_t T, int planes) {
    const int64_t tiles = (int64_t)planes * ((cs.K + 127) / 128) * ((cs.C + 127) / 128);
    return (int)std::max<int64_t>(1, std::min<int64_t>(1024 / tiles, T / 128));
}

// Filter gradient: transformed input and output gradient of one chunk of images, the transformed filter gradient and
// one more buffer of its size for a chunk's share (added to the former chunk after chunk, i.e. in a fixed order), and
// the partial sums of a chunk's reduction ranges.
struct WinoWgradPlan {
    size_t filt, per_img;
    int imgs, ranges;
    size_t floats() const { return (size_t)imgs * per_img + 2 * filt + (ranges > 1 ? (size_t)ranges * filt : 0); }
};
WinoWgradPlan wino_wgrad_plan(const ConvShape &cs, int m, int imgs) {
    const int planes = (m + 2) * (m + 2);
    WinoWgradPlan wp;
    wp.filt = (size_t)planes * cs.K * cs.C;
    const int64_t tiles_img = (int64_t)((cs.H + m - 1) / m) * ((cs.W + m - 1) / m);
    wp.per_img = (size_t)planes * tiles_img * ((size_t)cs.C + cs.K);
    wp.imgs = imgs > 0 ? imgs : (int)std::min<size_t>((size_t)cs.N, std::max<size_t>(1, (WINO_CHUNK_BYTES / 4 + wp.per_img - 1) / wp.per_img));
    wp.imgs = even_chunk(cs.N, wp.imgs);
    wp.ranges = wgrad_ranges(cs, (int64_t)wp.imgs * tiles_img, planes);
    return wp;
}
}  // namespace

size_t winograd_wgrad_workspace_bytes(const ConvShape &cs, int m) {
    check_tile(m, "winograd_wgrad_workspace_bytes");
    return wino_wgrad_plan(cs, m, 0).floats() * sizeof(float);
}

void conv_winograd_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int m, float *ws, size_t ws_bytes) {
    check_tile(m, "conv_winograd_wgrad");
    if (cs.R != 3 || cs.S != 3 || cs.stride != 1 || cs.pad != 1 || cs.C % 4 || cs.K % 4)
        throw KernelError("conv_winograd_wgrad: needs a 3x3 / stride 1 / pad 1 layer with channel counts that are multiples of 4");
    // the largest chunk the workspace holds
    WinoWgradPlan wp = wino_wgrad_plan(cs, m, cs.N);
    if (!ws || wp.floats() * sizeof(float) > ws_bytes) {
        int lo = 0, hi = cs.N;                        // floats() grows with imgs over the range that matters: bisect
        while (hi - lo > 1) {
            const int mid = (lo + hi) / 2;
            if (ws && wino_wgrad_plan(cs, m, mid).floats() * sizeof(float) <= ws_bytes) lo = mid; else hi = mid;
        }
        if (lo < 1) throw KernelError("conv_winograd_wgrad: workspace too small");
        wp = wino_wgrad_plan(cs, m, lo);
    }
    const int planes = (m + 2) * (m + 2), vec = m == 2 ? 4 : 2;
    float *VD = ws, *dU = VD + (size_t)wp.imgs * wp.per_img, *share = dU + wp.filt, *slabs = share + wp.filt;
    const dim3 blk(256);
    for (int img0 = 0; img0 < cs.N; img0 += wp.imgs) {
        ConvShape part = cs;
        part.N = std::min(wp.imgs, cs.N - img0);
        const WinoGeom gm = geom_of(part, m);
        if (gm.T * (std::max(cs.C, cs.K) / vec) / 256 >= 0x7fffffffll || gm.T >= (1 << 24)) throw KernelError("conv_winograd_wgrad: shape too large");
        float *V = VD, *D = V + (size_t)planes * gm.T * cs.C;
        const float *px = x + (size_t)img0 * cs.H * cs.W * cs.C, *pdy = dy + (size_t)img0 * cs.H * cs.W * cs.K;
        const int64_t ie = gm.T * (cs.C / vec), de = gm.T * (cs.K / vec);
        const dim3 ig((unsigned)(((ie + 255) / 256 + 7) / 8 * 8)), dg((unsigned)((de + 255) / 256));
        if (m == 2) {
            hipLaunchKernelGGL(wino_input_kernel<2>, ig, blk, 0, st, px, V, gm, cs.C);
            hipLaunchKernelGGL(wino_dy_kernel, dg, blk, 0, st, pdy, D, gm, cs.K);
        } else {
            hipLaunchKernelGGL(wino4_input_kernel<2>, ig, blk, 0, st, px, V, gm, cs.C);
            hipLaunchKernelGGL(wino4_dy_kernel, dg, blk, 0, st, pdy, D, gm, cs.K);
        }
        hip_check(hipGetLastError(), "winograd transform launch");
        const int sp = std::min(wp.ranges, wgrad_ranges(cs, gm.T, planes));      // the last chunk may be shorter
        gemm_tn_batched(st, D, V, img0 == 0 ? dU : share, planes, gm.T, cs.K, cs.C, sp, sp > 1 ? slabs : nullptr,
                        sp > 1 ? (size_t)sp * wp.filt * sizeof(float) : 0);
        if (img0 > 0) copy_or_accumulate(st, share, dU, (int64_t)wp.filt, true);
    }
    const int64_t fe = (int64_t)cs.K * cs.C;
    const dim3 fg((unsigned)((fe + 255) / 256));
    if (m == 2) hipLaunchKernelGGL(wino_filter_back_kernel, fg, blk, 0, st, (const float *)dU, dw, cs.K, cs.C);
    else hipLaunchKernelGGL(wino4_filter_back_kernel, fg, blk, 0, st, (const float *)dU, dw, cs.K, cs.C);
    hip_check(hipGetLastError(), "winograd filter gradient launch");
}

}  // namespace monet
