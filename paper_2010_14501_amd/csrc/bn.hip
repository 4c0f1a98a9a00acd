// BatchNorm (training mode, biased variance) over a rows x C matrix (rows = N*H*W, channel
// fastest): statistics, apply, and backward from the input or -- the output-activated variant
// of the paper's Appendix D -- from the operator's own output.
//
// Reductions are two-level and fixed-order (per-thread partials over a row slab, a shared-memory
// tree per block, then one pass over the slab partials), so results are bitwise reproducible:
// no floating-point atomics.  Variance is accumulated around a per-thread pivot and merged with
// the pairwise (Chan) update, never as E[x^2]-mean^2.
#include "kernels.hpp"

namespace monet {

namespace {

struct BnGeom {
    int C4;      // float4 column groups
    int TPR;     // threads that share a row
    int RPP;     // rows per pass of a 256-thread block
    int CB;      // column blocks (grid.y)
    int G;       // row slabs (grid.x)
    int64_t slab;
};

BnGeom bn_geom(int64_t rows, int C, int64_t scratch_floats, int per_slab_floats_per_channel) {
    if (C % 4) throw KernelError("BatchNorm: C must be a multiple of 4");
    BnGeom g;
    g.C4 = C / 4;
    g.TPR = 1;
    while (g.TPR * 2 <= g.C4 && g.TPR < 64) g.TPR *= 2;   // power of two <= min(C4, 64)
    g.RPP = 256 / g.TPR;
    g.CB = (g.C4 + g.TPR - 1) / g.TPR;
    int64_t want = (rows + (int64_t)g.RPP * 8 - 1) / ((int64_t)g.RPP * 8);
    int64_t cap = scratch_floats / ((int64_t)per_slab_floats_per_channel * C);
    if (cap < 1) throw KernelError("BatchNorm: reduction scratch too small");
    g.G = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, 1024), cap));
    g.slab = (rows + g.G - 1) / g.G;
    return g;
}

}  // namespace

// ------------------------------------------------------------------ statistics
// partial[(slab * C + c) * 2 + {0,1}] = {mean, M2} of the slab's rows for channel c
__global__ __launch_bounds__(256) void bn_stats_partial(const float *__restrict__ x, float *__restrict__ part, int64_t rows,
                                                        int C, int TPR, int64_t slab) {
    __shared__ float sh_mean[256 * 4];
    __shared__ float sh_m2[256 * 4];
    __shared__ float sh_n[256];
    const int C4 = C / 4;
    const int tc = threadIdx.x % TPR, tr = threadIdx.x / TPR, RPP = 256 / TPR;
    const int cg = blockIdx.y * TPR + tc;
    const int64_t r0 = (int64_t)blockIdx.x * slab;
    const int64_t r1 = r0 + slab < rows ? r0 + slab : rows;
    float pv[4] = {0, 0, 0, 0}, s1[4] = {0, 0, 0, 0}, s2[4] = {0, 0, 0, 0};
    float n = 0;
    if (cg < C4) {
        for (int64_t r = r0 + tr; r < r1; r += RPP) {
            float4 v = ((const float4 *)x)[r * C4 + cg];
            float vv[4] = {v.x, v.y, v.z, v.w};
            if (n == 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) pv[j] = vv[j];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float d = vv[j] - pv[j];
                s1[j] += d;
                s2[j] += d * d;
            }
            n += 1;
        }
    }
    // thread statistics: mean = pivot + s1/n, M2 = s2 - s1^2/n
    sh_n[threadIdx.x] = n;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float m = n > 0 ? pv[j] + s1[j] / n : 0.0f;
        float q = n > 0 ? s2[j] - s1[j] * s1[j] / n : 0.0f;
        sh_mean[threadIdx.x * 4 + j] = m;
        sh_m2[threadIdx.x * 4 + j] = q < 0 ? 0.0f : q;
    }
    __syncthreads();
    // tree over the RPP threads that share a column group (thread index = tr*TPR + tc)
    for (int half = RPP / 2; half > 0; half >>= 1) {
        if (tr < half) {
            int a = threadIdx.x, b = (tr + half) * TPR + tc;
            float na = sh_n[a], nb = sh_n[b], nt = na + nb;
            if (nb > 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float ma = sh_mean[a * 4 + j], mb = sh_mean[b * 4 + j];
                    float d = mb - ma;
                    sh_mean[a * 4 + j] = na > 0 ? ma + d * (nb / nt) : mb;
                    sh_m2[a * 4 + j] = sh_m2[a * 4 + j] + sh_m2[b * 4 + j] + (na > 0 ? d * d * (na * nb / nt) : 0.0f);
                }
                sh_n[a] = nt;
            }
        }
        __syncthreads();
    }
    if (tr == 0 && cg < C4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = cg * 4 + j;
            part[((int64_t)blockIdx.x * C + c) * 2 + 0] = sh_mean[tc * 4 + j];
            part[((int64_t)blockIdx.x * C + c) * 2 + 1] = sh_m2[tc * 4 + j];
        }
    }
}

// Block = 16 channels x 16 slab lanes.  Lane sl merges slabs sl, sl+16, ... in order, then the 16
// lanes of a channel are merged by a fixed tree.
__global__ __launch_bounds__(256) void bn_stats_final(const float *__restrict__ part, float *__restrict__ stats, int64_t rows,
                                                      int C, int G, int64_t slab, float eps) {
    __shared__ float sh_n[256], sh_mean[256], sh_m2[256];
    const int cl = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + cl;
    float n = 0, mean = 0, m2 = 0;
    if (c < C) {
        for (int g = sl; g < G; g += 16) {
            int64_t r0 = (int64_t)g * slab;
            int64_t cnt = r0 + slab < rows ? slab : rows - r0;
            if (cnt <= 0) break;
            float nb = (float)cnt;
            float mb = part[((int64_t)g * C + c) * 2 + 0], qb = part[((int64_t)g * C + c) * 2 + 1];
            float nt = n + nb, d = mb - mean;
            mean = n > 0 ? mean + d * (nb / nt) : mb;
            m2 = m2 + qb + (n > 0 ? d * d * (n * nb / nt) : 0.0f);
            n = nt;
        }
    }
    sh_n[threadIdx.x] = n; sh_mean[threadIdx.x] = mean; sh_m2[threadIdx.x] = m2;
    __syncthreads();
    for (int half = 8; half > 0; half >>= 1) {
        if (sl < half) {
            int a = threadIdx.x, b = (sl + half) * 16 + cl;
            float na = sh_n[a], nb = sh_n[b], nt = na + nb;
            if (nb > 0) {
                float ma = sh_mean[a], mb = sh_mean[b], d = mb - ma;
                sh_mean[a] = na > 0 ? ma + d * (nb / nt) : mb;
                sh_m2[a] = sh_m2[a] + sh_m2[b] + (na > 0 ? d * d * (na * nb / nt) : 0.0f);
                sh_n[a] = nt;
            }
        }
        __syncthreads();
    }
    if (sl == 0 && c < C) {
        float var = sh_m2[cl] / sh_n[cl];
        stats[c] = sh_mean[cl];
        stats[C + c] = 1.0f / sqrtf(var + eps);
    }
}

void bn_stats(hipStream_t st, const float *x, float *stats, int64_t rows, int C, float eps, float *scratch, size_t scratch_bytes) {
    if (rows <= 0) throw KernelError("BatchNorm: no rows");
    BnGeom g = bn_geom(rows, C, (int64_t)(scratch_bytes / 4), 2);
    hipLaunchKernelGGL(bn_stats_partial, dim3(g.G, g.CB), dim3(256), 0, st, x, scratch, rows, C, g.TPR, g.slab);
    hipLaunchKernelGGL(bn_stats_final, dim3((C + 15) / 16), dim3(256), 0, st, (const float *)scratch, stats, rows, C, g.G, g.slab, eps);
    hip_check(hipGetLastError(), "bn_stats launch");
}

// ------------------------------------------------------------------ apply: y = gamma*(x-mean)*invstd + beta.  y may alias x.
__global__ __launch_bounds__(256) void bn_apply_kernel(const float *x, float *y, const float *__restrict__ gamma,
                                                       const float *__restrict__ beta, const float *__restrict__ stats,
                                                       int64_t total4, int C) {
    const int C4 = C / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool fixed = (stride % C4) == 0;     // then every element this thread visits has the same channels
    float a[4], b[4];
    int cg = (int)(i % C4);
    auto load_ab = [&](int g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = g * 4 + j;
            float s = gamma[c] * stats[C + c];
            a[j] = s;
            b[j] = beta[c] - stats[c] * s;
        }
    };
    if (fixed) load_ab(cg);
    for (; i < total4; i += stride) {
        if (!fixed) load_ab((int)(i % C4));
        float4 v = ((const float4 *)x)[i];
        ((float4 *)y)[i] = make_float4(v.x * a[0] + b[0], v.y * a[1] + b[1], v.z * a[2] + b[2], v.w * a[3] + b[3]);
    }
}

void bn_apply(hipStream_t st, const float *x, float *y, const float *gamma, const float *beta, const float *stats, int64_t rows, int C) {
    if (C % 4) throw KernelError("BatchNorm: C must be a multiple of 4");
    int64_t total4 = rows * (C / 4);
    if (total4 <= 0) return;
    int64_t want = (total4 + 256 * 4 - 1) / (256 * 4);
    int grid = (int)std::max<int64_t>(1, std::min<int64_t>(want, 8192));
    if (grid > 2) grid &= ~1;   // keep the thread count a multiple of the usual power-of-two channel groups
    hipLaunchKernelGGL(bn_apply_kernel, dim3(grid), dim3(256), 0, st, x, y, gamma, beta, stats, total4, C);
    hip_check(hipGetLastError(), "bn_apply launch");
}

// ------------------------------------------------------------------ backward
// xhat = (x - mean)*invstd            (from the input)
//      = (y - beta)/gamma             (from the output; gamma must be non-zero)
// dbeta = sum dy, dgamma = sum dy*xhat, dx = gamma*invstd*(dy - dbeta/m - xhat*dgamma/m)
template <bool FROM_OUT>
__global__ __launch_bounds__(256) void bn_bwd_partial(const float *__restrict__ dy, const uint64_t *__restrict__ mask,
                                                      const float *__restrict__ t, const float *__restrict__ gamma, const float *__restrict__ beta,
                                                      const float *__restrict__ stats, float *__restrict__ part, int64_t rows,
                                                      int C, int TPR, int64_t slab) {
    __shared__ float sh_b[256 * 4];
    __shared__ float sh_g[256 * 4];
    const int C4 = C / 4;
    const int tc = threadIdx.x % TPR, tr = threadIdx.x / TPR, RPP = 256 / TPR;
    const int cg = blockIdx.y * TPR + tc;
    const int64_t r0 = (int64_t)blockIdx.x * slab;
    const int64_t r1 = r0 + slab < rows ? r0 + slab : rows;
    float sb[4] = {0, 0, 0, 0}, sg[4] = {0, 0, 0, 0};
    if (cg < C4) {
        float sc[4], sh[4];   // xhat = t*sc + sh
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = cg * 4 + j;
            if (FROM_OUT) { sc[j] = 1.0f / gamma[c]; sh[j] = -beta[c] * sc[j]; }
            else { sc[j] = stats[C + c]; sh[j] = -stats[c] * sc[j]; }
        }
        for (int64_t r = r0 + tr; r < r1; r += RPP) {
            const int64_t i4 = r * C4 + cg;
            float4 g = ((const float4 *)dy)[i4];
            float4 v = ((const float4 *)t)[i4];
            float gg[4] = {g.x, g.y, g.z, g.w}, vv[4] = {v.x, v.y, v.z, v.w};
            if (mask) {     // the incoming gradient still has to pass a ReLU: keep it where the sign bit is set
                unsigned bits = (unsigned)(mask[i4 >> 4] >> ((i4 & 15) * 4)) & 15u;
#pragma unroll
                for (int j = 0; j < 4; ++j) gg[j] = (bits >> j) & 1 ? gg[j] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sb[j] += gg[j];
                sg[j] += gg[j] * (vv[j] * sc[j] + sh[j]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        sh_b[threadIdx.x * 4 + j] = sb[j];
        sh_g[threadIdx.x * 4 + j] = sg[j];
    }
    __syncthreads();
    for (int half = RPP / 2; half > 0; half >>= 1) {
        if (tr < half) {
            int a = threadIdx.x, b = (tr + half) * TPR + tc;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sh_b[a * 4 + j] += sh_b[b * 4 + j];
                sh_g[a * 4 + j] += sh_g[b * 4 + j];
            }
        }
        __syncthreads();
    }
    if (tr == 0 && cg < C4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = cg * 4 + j;
            part[((int64_t)blockIdx.x * C + c) * 2 + 0] = sh_b[tc * 4 + j];
            part[((int64_t)blockIdx.x * C + c) * 2 + 1] = sh_g[tc * 4 + j];
        }
    }
}

// Block = 16 channels x 16 slab lanes (lane sl adds slabs sl, sl+16, ... in order, then a fixed
// tree); writes dbeta, dgamma and, for the apply pass, coef[c] = dbeta/m, coef[C+c] = dgamma/m
__global__ __launch_bounds__(256) void bn_bwd_final(const float *__restrict__ part, float *__restrict__ dgamma,
                                                    float *__restrict__ dbeta, float *__restrict__ coef, int64_t rows, int C, int G) {
    __shared__ float sh_b[256], sh_g[256];
    const int cl = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + cl;
    float b = 0, g = 0;
    if (c < C)
        for (int s = sl; s < G; s += 16) {
            b += part[((int64_t)s * C + c) * 2 + 0];
            g += part[((int64_t)s * C + c) * 2 + 1];
        }
    sh_b[threadIdx.x] = b; sh_g[threadIdx.x] = g;
    __syncthreads();
    for (int half = 8; half > 0; half >>= 1) {
        if (sl < half) {
            sh_b[threadIdx.x] += sh_b[(sl + half) * 16 + cl];
            sh_g[threadIdx.x] += sh_g[(sl + half) * 16 + cl];
        }
        __syncthreads();
    }
    if (sl == 0 && c < C) {
        b = sh_b[cl]; g = sh_g[cl];
        dbeta[c] = b;
        dgamma[c] = g;
        coef[c] = b / (float)rows;
        coef[C + c] = g / (float)rows;
    }
}

template <bool FROM_OUT, bool ACC>
__global__ __launch_bounds__(256) void bn_bwd_apply(const float *__restrict__ dy, const uint64_t *__restrict__ mask,
                                                    const float *__restrict__ t,
                                                    const float *__restrict__ gamma, const float *__restrict__ beta,
                                                    const float *__restrict__ stats, const float *__restrict__ coef, float *dx,
                                                    int64_t total4, int C) {
    const int C4 = C / 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool fixed = (stride % C4) == 0;
    float sc[4], sh[4], a[4], mb[4], mg[4];
    auto load = [&](int g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = g * 4 + j;
            if (FROM_OUT) { sc[j] = 1.0f / gamma[c]; sh[j] = -beta[c] * sc[j]; }
            else { sc[j] = stats[C + c]; sh[j] = -stats[c] * sc[j]; }
            a[j] = gamma[c] * stats[C + c];
            mb[j] = coef[c];
            mg[j] = coef[C + c];
        }
    };
    if (fixed) load((int)(i % C4));
    for (; i < total4; i += stride) {
        if (!fixed) load((int)(i % C4));
        float4 g = ((const float4 *)dy)[i];
        float4 v = ((const float4 *)t)[i];
        float gg[4] = {g.x, g.y, g.z, g.w}, vv[4] = {v.x, v.y, v.z, v.w}, r[4];
        if (mask) {
            unsigned bits = (unsigned)(mask[i >> 4] >> ((i & 15) * 4)) & 15u;
#pragma unroll
            for (int j = 0; j < 4; ++j) gg[j] = (bits >> j) & 1 ? gg[j] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float xh = vv[j] * sc[j] + sh[j];
            r[j] = a[j] * (gg[j] - mb[j] - xh * mg[j]);
        }
        if (ACC) { float4 o = ((float4 *)dx)[i]; r[0] += o.x; r[1] += o.y; r[2] += o.z; r[3] += o.w; }
        ((float4 *)dx)[i] = make_float4(r[0], r[1], r[2], r[3]);
    }
}

void bn_bwd(hipStream_t st, const float *dy, const float *t, bool from_output, const float *gamma, const float *beta,
            const float *stats, float *dx, float *dgamma, float *dbeta, int64_t rows, int C, bool accumulate, float *scratch,
            size_t scratch_bytes, const uint64_t *mask) {
    if (rows <= 0) throw KernelError("BatchNorm: no rows");
    int64_t floats = (int64_t)(scratch_bytes / 4) - 2 * C;    // tail of the scratch holds the two coefficient vectors
    BnGeom g = bn_geom(rows, C, floats, 2);
    float *coef = scratch + (int64_t)g.G * C * 2;
    if (from_output) hipLaunchKernelGGL((bn_bwd_partial<true>), dim3(g.G, g.CB), dim3(256), 0, st, dy, mask, t, gamma, beta, stats, scratch, rows, C, g.TPR, g.slab);
    else hipLaunchKernelGGL((bn_bwd_partial<false>), dim3(g.G, g.CB), dim3(256), 0, st, dy, mask, t, gamma, beta, stats, scratch, rows, C, g.TPR, g.slab);
    hipLaunchKernelGGL(bn_bwd_final, dim3((C + 15) / 16), dim3(256), 0, st, (const float *)scratch, dgamma, dbeta, coef, rows, C, g.G);
    int64_t total4 = rows * (C / 4);
    int64_t want = (total4 + 256 * 4 - 1) / (256 * 4);
    int grid = (int)std::max<int64_t>(1, std::min<int64_t>(want, 8192));
    if (grid > 2) grid &= ~1;
#define BA(F, A) hipLaunchKernelGGL((bn_bwd_apply<F, A>), dim3(grid), dim3(256), 0, st, dy, mask, t, gamma, beta, stats, (const float *)coef, dx, total4, C)
    if (from_output) { if (accumulate) BA(true, true); else BA(true, false); }
    else             { if (accumulate) BA(false, true); else BA(false, false); }
#undef BA
    hip_check(hipGetLastError(), "bn_bwd launch");
}

}  // namespace monet
