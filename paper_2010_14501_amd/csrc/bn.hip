// BatchNorm (training mode, biased variance) over a rows x C matrix (rows = N*H*W, channel
// fastest): statistics, apply, and backward from the input or -- the output-activated variant
// of the paper's Appendix D -- from the operator's own output.
//
// Reductions are two-level and fixed-order (per-thread partials over a row slab, a shared-memory
// tree per block, then one pass over the slab partials), so results are bitwise reproducible:
// no floating-point atomics.  Variance is accumulated around a per-thread pivot and merged with
// the pairwise (Chan) update, never as E[x^2]-mean^2.
#include "bn_affine.hpp"
#include "kernels.hpp"
#include "tile_stats.hpp"

#include <mutex>

namespace monet {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

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
    if (cg < C4 && r0 + tr < r1) {
        // pivot = the thread's first element; rows are then taken four at a time so that four loads are in flight
        const f4 *xp = (const f4 *)x + cg;
        const f4 p = __builtin_nontemporal_load(xp + (r0 + tr) * C4);
        pv[0] = p.x; pv[1] = p.y; pv[2] = p.z; pv[3] = p.w;
        int64_t r = r0 + tr;
        for (; r + 3 * RPP < r1; r += 4 * RPP) {
            f4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(xp + (r + u * RPP) * C4);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float d = vv[j] - pv[j];
                    s1[j] += d;
                    s2[j] += d * d;
                }
            }
            n += 4;
        }
        for (; r < r1; r += RPP) {
            const f4 v = __builtin_nontemporal_load(xp + r * C4);
            float vv[4] = {v.x, v.y, v.z, v.w};
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

// The same partial results in groups of 64 rows (see tile_stats.hpp): one wave per (row group, 64 columns),
// no LDS, sixteen 16-byte loads per lane in flight.  Wave u of the launch takes group u / chunks, columns
// 64 * (u % chunks).
__global__ __launch_bounds__(256) void bn_stats_rows64(const float *__restrict__ x, float *__restrict__ part, int64_t rows, int C,
                                                        int chunks, int64_t units) {
    const int lane = threadIdx.x & 63;
    const int64_t u = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (u >= units) return;
    const int64_t grp = u / chunks;
    const int col = (int)(u % chunks) * 64 + 4 * (lane & 15);
    const int64_t r0 = grp * STAT_ROWS + (lane >> 4);
    f4 v[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int64_t r = r0 + 16 * (t >> 2) + 4 * (t & 3);
        v[t] = f4{0, 0, 0, 0};
        if (r < rows && col < C) v[t] = __builtin_nontemporal_load((const f4 *)(x + r * C + col));
    }
    LaneStats ls;
    ls.init();
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int64_t r = r0 + 16 * (t >> 2) + 4 * (t & 3);
        if (r < rows && col < C) ls.add(v[t].x, v[t].y, v[t].z, v[t].w);
    }
    float n, mean[4], m2[4];
    merge_lane_stats(ls, lane, n, mean, m2);
    store_group_stats(part, grp, C, col, lane, mean, m2);
}

// Second level for tensors with many row groups: one wave per (64 consecutive groups, 64 channels) merges them in
// group order, lane = channel, so every load instruction reads 512 contiguous bytes; eight loads in flight.
constexpr int FOLD = 64;
__global__ __launch_bounds__(256) void bn_stats_fold(const float *__restrict__ part, float *__restrict__ folded, int64_t rows, int C,
                                                      int64_t groups, int chunks, int64_t units) {
#pragma clang fp contract(off)
    const int lane = threadIdx.x & 63;
    const int64_t u = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (u >= units) return;
    const int64_t sg = u / chunks;
    const int c = (int)(u % chunks) * 64 + lane;
    if (c >= C) return;
    const int64_t g0 = sg * FOLD, g1 = g0 + FOLD < groups ? g0 + FOLD : groups;
    float n = 0, mean = 0, m2 = 0;
    for (int64_t gb = g0; gb < g1; gb += 8) {
        float2 p[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) p[t] = gb + t < g1 ? *(const float2 *)(part + ((gb + t) * C + c) * 2) : make_float2(0, 0);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t g = gb + t;
            if (g >= g1) break;
            const int64_t r0 = g * STAT_ROWS;
            const float nb = (float)(r0 + STAT_ROWS < rows ? STAT_ROWS : rows - r0);
            const float nt = n + nb, d = p[t].x - mean;
            mean = n > 0 ? mean + d * (nb / nt) : p[t].x;
            m2 = m2 + p[t].y + (n > 0 ? d * d * (n * nb / nt) : 0.0f);
            n = nt;
        }
    }
    *(float2 *)(folded + (sg * C + c) * 2) = make_float2(mean, m2);
}

// Block = FIN_CH channels x FIN_LANES slab lanes.  Lane sl merges slabs sl, sl+FIN_LANES, ... in order,
// then the lanes of a channel are merged by a fixed tree.  Few channels per block and many lanes keep
// the dependent chain per thread short: these kernels are latency-bound, not bandwidth-bound.
constexpr int FIN_CH = 4, FIN_LANES = 64;
__global__ __launch_bounds__(256) void bn_stats_final(const float *__restrict__ part, float *__restrict__ stats, int64_t rows,
                                                      int C, int G, int64_t slab, float eps) {
    __shared__ float sh_n[256], sh_mean[256], sh_m2[256];
    const int cl = threadIdx.x & (FIN_CH - 1), sl = threadIdx.x / FIN_CH;
    const int c = blockIdx.x * FIN_CH + cl;
    float n = 0, mean = 0, m2 = 0;
    if (c < C) {
        // loads of four slabs are issued together, then merged in slab order
        for (int g0 = sl; g0 < G; g0 += 4 * FIN_LANES) {
            float mb[4], qb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = g0 + u * FIN_LANES;
                const float2 p = g < G ? *(const float2 *)(part + ((int64_t)g * C + c) * 2) : make_float2(0, 0);
                mb[u] = p.x; qb[u] = p.y;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = g0 + u * FIN_LANES;
                const int64_t r0 = (int64_t)g * slab;
                const int64_t cnt = g < G ? (r0 + slab < rows ? slab : rows - r0) : 0;
                if (cnt <= 0) continue;
                float nb = (float)cnt;
                float nt = n + nb, d = mb[u] - mean;
                mean = n > 0 ? mean + d * (nb / nt) : mb[u];
                m2 = m2 + qb[u] + (n > 0 ? d * d * (n * nb / nt) : 0.0f);
                n = nt;
            }
        }
    }
    sh_n[threadIdx.x] = n; sh_mean[threadIdx.x] = mean; sh_m2[threadIdx.x] = m2;
    __syncthreads();
    for (int half = FIN_LANES / 2; half > 0; half >>= 1) {
        if (sl < half) {
            int a = threadIdx.x, b = (sl + half) * FIN_CH + cl;
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

// more row groups than this are first merged 64 at a time (bn_stats_fold)
constexpr int64_t FOLD_ABOVE = 4096;   // measured: below this the extra launch costs more than the longer final merge

bool bn_stats_in_row_groups(int64_t rows, int C, size_t scratch_bytes) {
    if (rows <= 0 || C % 4) return false;
    const int64_t groups = (rows + STAT_ROWS - 1) / STAT_ROWS;
    const int64_t folded = groups > FOLD_ABOVE ? (groups + FOLD - 1) / FOLD : 0;
    return (size_t)(groups + folded) * C * 2 * sizeof(float) <= scratch_bytes;
}

void bn_stats(hipStream_t st, const float *x, float *stats, int64_t rows, int C, float eps, float *scratch, size_t scratch_bytes,
              bool partials_ready) {
    if (rows <= 0) throw KernelError("BatchNorm: no rows");
    if (bn_stats_in_row_groups(rows, C, scratch_bytes)) {
        const int64_t groups = (rows + STAT_ROWS - 1) / STAT_ROWS;
        if (!partials_ready) {
            const int chunks = (C + 63) / 64;
            const int64_t units = groups * chunks;
            hipLaunchKernelGGL(bn_stats_rows64, dim3((unsigned)((units + 3) / 4)), dim3(256), 0, st, x, scratch, rows, C, chunks, units);
        }
        if (groups > FOLD_ABOVE) {
            const int64_t folded = (groups + FOLD - 1) / FOLD;
            float *second = scratch + groups * C * 2;
            const int chunks = (C + 63) / 64;
            const int64_t units = folded * chunks;
            hipLaunchKernelGGL(bn_stats_fold, dim3((unsigned)((units + 3) / 4)), dim3(256), 0, st, (const float *)scratch, second, rows, C,
                               groups, chunks, units);
            hipLaunchKernelGGL(bn_stats_final, dim3((C + FIN_CH - 1) / FIN_CH), dim3(256), 0, st, (const float *)second, stats, rows, C,
                               (int)folded, (int64_t)STAT_ROWS * FOLD, eps);
        } else {
            hipLaunchKernelGGL(bn_stats_final, dim3((C + FIN_CH - 1) / FIN_CH), dim3(256), 0, st, (const float *)scratch, stats, rows, C,
                               (int)groups, (int64_t)STAT_ROWS, eps);
        }
        hip_check(hipGetLastError(), "bn_stats launch");
        return;
    }
    if (partials_ready) throw KernelError("BatchNorm: partial statistics announced for a tensor that does not use row groups");
    BnGeom g = bn_geom(rows, C, (int64_t)(scratch_bytes / 4), 2);
    hipLaunchKernelGGL(bn_stats_partial, dim3(g.G, g.CB), dim3(256), 0, st, x, scratch, rows, C, g.TPR, g.slab);
    hipLaunchKernelGGL(bn_stats_final, dim3((C + FIN_CH - 1) / FIN_CH), dim3(256), 0, st, (const float *)scratch, stats, rows, C, g.G, g.slab, eps);
    hip_check(hipGetLastError(), "bn_stats launch");
}

// ------------------------------------------------------------------ statistics without caller scratch
// For callers that cannot allocate device memory: the slab / row-group partial results go to a file-scope device
// array instead of a scratch argument.  In host code the array's name is only a stand-in: its device address is looked
// up once per device (each GPU holds its own copy) and only that address is handed to kernels.
constexpr size_t kStaticScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char static_scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex static_scratch_mutex;
float *static_scratch_ptr[kMaxDevices] = {};

float *static_scratch_on_current_device() {
    int dev = -1;
    hip_check(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) throw KernelError("BatchNorm statistics: device index out of range");
    std::lock_guard<std::mutex> lock(static_scratch_mutex);
    if (!static_scratch_ptr[dev]) {
        void *ptr = nullptr;
        hip_check(hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch)), "hipGetSymbolAddress(static_scratch)");
        if (!ptr) throw KernelError("BatchNorm statistics: no address for the static scratch");
        static_scratch_ptr[dev] = (float *)ptr;
    }
    return static_scratch_ptr[dev];
}
}  // namespace

void bn_stats_static(hipStream_t st, const float *x, float *stats, int64_t rows, int C, float eps) {
    if (rows <= 0) throw KernelError("BatchNorm: no rows");
    if (C <= 0 || C % 4 || C > kBnStaticMaxC)
        throw KernelError("BatchNorm statistics without scratch: C must be a multiple of 4, at most " + std::to_string(kBnStaticMaxC));
    if (rows > kBnStaticMaxRows)
        throw KernelError("BatchNorm statistics without scratch: at most " + std::to_string(kBnStaticMaxRows) + " rows");
    // every partial result the merge kernels read is written by the first kernel of the same call: nothing to clear
    bn_stats(st, x, stats, rows, C, eps, static_scratch_on_current_device(), kStaticScratchBytes);
}

// ------------------------------------------------------------------ apply: y = gamma*(x-mean)*invstd + beta.  y may alias x.
__global__ __launch_bounds__(256) void bn_apply_kernel(const float *x, float *y, const float *__restrict__ gamma,
                                                       const float *__restrict__ beta, const float *__restrict__ stats,
                                                       int64_t total4, int C) {
    // One contiguous range per workgroup (a multiple of 256 float4, so a thread keeps its channel group
    // whenever C/4 divides 256), four float4 per thread in flight, streaming loads and stores.
    constexpr int U = 4;
    const int C4 = C / 4;
    const bool fixed = (256 % C4) == 0;
    float a[4], b[4];
    auto load_ab = [&](int g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bn_affine_coeffs(gamma, beta, stats, C, g * 4 + j, a[j], b[j]);
        }
    };
    const int64_t per = ((total4 + gridDim.x - 1) / gridDim.x + 255) / 256 * 256;
    const int64_t r0 = (int64_t)blockIdx.x * per;
    const int64_t r1 = r0 + per < total4 ? r0 + per : total4;
    if (fixed) load_ab((int)(threadIdx.x % C4));
    for (int64_t base = r0 + threadIdx.x; base < r1; base += U * 256) {
        f4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u * 256 < r1) v[u] = __builtin_nontemporal_load((const f4 *)x + base + u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            if (i >= r1) continue;
            if (!fixed) load_ab((int)(i % C4));
            __builtin_nontemporal_store(f4{bn_affine(v[u].x, a[0], b[0]), bn_affine(v[u].y, a[1], b[1]), bn_affine(v[u].z, a[2], b[2]), bn_affine(v[u].w, a[3], b[3])}, (f4 *)y + i);
        }
    }
}

// one workgroup per 2048 float4 (32 KiB), up to 64 Ki workgroups
static int stream_grid(int64_t total4) {
    int64_t want = (total4 + 2047) / 2048;
    return (int)std::max<int64_t>(1, std::min<int64_t>(want, 65536));
}

void bn_apply(hipStream_t st, const float *x, float *y, const float *gamma, const float *beta, const float *stats, int64_t rows, int C) {
    if (C % 4) throw KernelError("BatchNorm: C must be a multiple of 4");
    int64_t total4 = rows * (C / 4);
    if (total4 <= 0) return;
    int grid = stream_grid(total4);
    hipLaunchKernelGGL(bn_apply_kernel, dim3(grid), dim3(256), 0, st, x, y, gamma, beta, stats, total4, C);
    hip_check(hipGetLastError(), "bn_apply launch");
}

// ------------------------------------------------------------------ backward
// xhat = (x - mean)*invstd            (from the input)
//      = (y - beta)/gamma             (from the output; gamma must be non-zero)
// dbeta = sum dy, dgamma = sum dy*xhat, dx = gamma*invstd*(dy - dbeta/m - xhat*dgamma/m)
// RM: how the incoming gradient is gated before use (a ReLU backward folded in): 0 not at all, 1 by the 1-bit
// sign code in rt, 2 by rt > 0, 3 by 0 < rt < 6 (rt = the ReLU's float input or output).
template <int RM>
__device__ inline void relu_gate(float (&gg)[4], unsigned bits, const f4 &rv) {
    if (RM == 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) gg[j] = (bits >> j) & 1 ? gg[j] : 0.0f;
    } else if (RM >= 2) {
        const float rr[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool pass = RM == 3 ? (rr[j] > 0.0f && rr[j] < 6.0f) : (rr[j] > 0.0f);
            gg[j] = pass ? gg[j] : 0.0f;
        }
    }
}

template <bool FROM_OUT, int RM>
__global__ __launch_bounds__(256) void bn_bwd_partial(const float *__restrict__ dy, const void *__restrict__ rt,
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
        const uint64_t *mask = (const uint64_t *)rt;
        auto accumulate = [&](const f4 &g, const f4 &v, const f4 &rv, int64_t i4) {
            float gg[4] = {g.x, g.y, g.z, g.w}, vv[4] = {v.x, v.y, v.z, v.w};
            // the incoming gradient may still have to pass a ReLU
            unsigned bits = 0;
            if (RM == 1) bits = (unsigned)(mask[i4 >> 4] >> ((i4 & 15) * 4)) & 15u;
            relu_gate<RM>(gg, bits, rv);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sb[j] += gg[j];
                sg[j] += gg[j] * (vv[j] * sc[j] + sh[j]);
            }
        };
        // rows two at a time: four 16-byte loads in flight per thread
        int64_t r = r0 + tr;
        for (; r + RPP < r1; r += 2 * RPP) {
            const int64_t ia = r * C4 + cg, ib = (r + RPP) * C4 + cg;
            const f4 ga = (*((const f4 *)dy + ia)), va = (*((const f4 *)t + ia));
            const f4 gb = (*((const f4 *)dy + ib)), vb = (*((const f4 *)t + ib));
            f4 ra = f4{0, 0, 0, 0}, rb = f4{0, 0, 0, 0};
            if (RM >= 2) { ra = __builtin_nontemporal_load((const f4 *)rt + ia); rb = __builtin_nontemporal_load((const f4 *)rt + ib); }
            accumulate(ga, va, ra, ia);
            accumulate(gb, vb, rb, ib);
        }
        for (; r < r1; r += RPP) {
            const int64_t ia = r * C4 + cg;
            f4 ra = f4{0, 0, 0, 0};
            if (RM >= 2) ra = __builtin_nontemporal_load((const f4 *)rt + ia);
            accumulate((*((const f4 *)dy + ia)), (*((const f4 *)t + ia)), ra, ia);
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

// The same partial sums for channel counts whose groups of four are no power of two (24, 36, 48, 96, 144, 240, 320 ...
// groups): there the kernel above leaves up to half of the lanes of its last column block without work.  Here a workgroup
// has T threads, a multiple of the number of channel groups, and streams one contiguous range of float4 elements
// (a multiple of T, so that thread t meets channel group t % C4 only); the T / C4 threads of a group are added in thread
// order.  Same layout of `part`, one row per workgroup.
template <bool FROM_OUT, int RM>
__global__ __launch_bounds__(512) void bn_bwd_partial_flat(const float *__restrict__ dy, const void *__restrict__ rt,
                                                           const float *__restrict__ t, const float *__restrict__ gamma,
                                                           const float *__restrict__ beta, const float *__restrict__ stats,
                                                           float *__restrict__ part, int64_t total4, int C, int64_t slab4) {
    __shared__ float sh_b[512 * 4];
    __shared__ float sh_g[512 * 4];
    const int C4 = C / 4, T = blockDim.x, tid = threadIdx.x;
    const int cg = tid % C4;
    const int64_t r0 = (int64_t)blockIdx.x * slab4;
    const int64_t r1 = r0 + slab4 < total4 ? r0 + slab4 : total4;
    float sb[4] = {0, 0, 0, 0}, sg[4] = {0, 0, 0, 0};
    float sc[4], sh[4];   // xhat = t*sc + sh
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = cg * 4 + j;
        if (FROM_OUT) { sc[j] = 1.0f / gamma[c]; sh[j] = -beta[c] * sc[j]; }
        else { sc[j] = stats[C + c]; sh[j] = -stats[c] * sc[j]; }
    }
    const uint64_t *mask = (const uint64_t *)rt;
    auto accumulate = [&](const f4 &g, const f4 &v, const f4 &rv, int64_t i4) {
        float gg[4] = {g.x, g.y, g.z, g.w}, vv[4] = {v.x, v.y, v.z, v.w};
        unsigned bits = 0;
        if (RM == 1) bits = (unsigned)(mask[i4 >> 4] >> ((i4 & 15) * 4)) & 15u;
        relu_gate<RM>(gg, bits, rv);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sb[j] += gg[j];
            sg[j] += gg[j] * (vv[j] * sc[j] + sh[j]);
        }
    };
    // two elements at a time: four 16-byte loads in flight per thread
    int64_t i = r0 + tid;
    for (; i + T < r1; i += 2 * (int64_t)T) {
        const int64_t ia = i, ib = i + T;
        const f4 ga = (*((const f4 *)dy + ia)), va = (*((const f4 *)t + ia));
        const f4 gb = (*((const f4 *)dy + ib)), vb = (*((const f4 *)t + ib));
        f4 ra = f4{0, 0, 0, 0}, rb = f4{0, 0, 0, 0};
        if (RM >= 2) { ra = __builtin_nontemporal_load((const f4 *)rt + ia); rb = __builtin_nontemporal_load((const f4 *)rt + ib); }
        accumulate(ga, va, ra, ia);
        accumulate(gb, vb, rb, ib);
    }
    if (i < r1) {
        f4 ra = f4{0, 0, 0, 0};
        if (RM >= 2) ra = __builtin_nontemporal_load((const f4 *)rt + i);
        accumulate((*((const f4 *)dy + i)), (*((const f4 *)t + i)), ra, i);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        sh_b[tid * 4 + j] = sb[j];
        sh_g[tid * 4 + j] = sg[j];
    }
    __syncthreads();
    if (tid < C4) {
        float b[4] = {0, 0, 0, 0}, g[4] = {0, 0, 0, 0};
        for (int k = tid; k < T; k += C4)
#pragma unroll
            for (int j = 0; j < 4; ++j) { b[j] += sh_b[k * 4 + j]; g[j] += sh_g[k * 4 + j]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = tid * 4 + j;
            part[((int64_t)blockIdx.x * C + c) * 2 + 0] = b[j];
            part[((int64_t)blockIdx.x * C + c) * 2 + 1] = g[j];
        }
    }
}

// Block = FIN_CH channels x FIN_LANES slab lanes (lane sl adds slabs sl, sl+FIN_LANES, ... in order, then a fixed
// tree); writes dbeta, dgamma and, for the apply pass, coef[c] = dbeta/m, coef[C+c] = dgamma/m
__global__ __launch_bounds__(256) void bn_bwd_final(const float *__restrict__ part, float *__restrict__ dgamma,
                                                    float *__restrict__ dbeta, float *__restrict__ coef, int64_t rows, int C, int G) {
    __shared__ float sh_b[256], sh_g[256];
    const int cl = threadIdx.x & (FIN_CH - 1), sl = threadIdx.x / FIN_CH;
    const int c = blockIdx.x * FIN_CH + cl;
    float b = 0, g = 0;
    if (c < C)
        for (int s0 = sl; s0 < G; s0 += 4 * FIN_LANES) {
            float2 p[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + u * FIN_LANES;
                p[u] = s < G ? *(const float2 *)(part + ((int64_t)s * C + c) * 2) : make_float2(0, 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (s0 + u * FIN_LANES < G) { b += p[u].x; g += p[u].y; }
        }
    sh_b[threadIdx.x] = b; sh_g[threadIdx.x] = g;
    __syncthreads();
    for (int half = FIN_LANES / 2; half > 0; half >>= 1) {
        if (sl < half) {
            sh_b[threadIdx.x] += sh_b[(sl + half) * FIN_CH + cl];
            sh_g[threadIdx.x] += sh_g[(sl + half) * FIN_CH + cl];
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

// side (may be null): a second tensor that receives (or accumulates) the gated incoming gradient itself -- the
// other branch of a residual add whose backward is folded in.
template <bool FROM_OUT, int RM>
__global__ __launch_bounds__(512) void bn_bwd_apply(const float *__restrict__ dy, const void *__restrict__ rt,
                                                    const float *__restrict__ t,
                                                    const float *__restrict__ gamma, const float *__restrict__ beta,
                                                    const float *__restrict__ stats, const float *__restrict__ coef, float *dx,
                                                    int acc, float *side, int side_acc, int64_t total4, int C) {
    const uint64_t *mask = (const uint64_t *)rt;
    // same streaming pattern as bn_apply_kernel
    constexpr int U = 4;
    const int C4 = C / 4;
    // The workgroup has T threads, a multiple of the number of channel groups whenever the host finds one (240 threads for
    // 24, 40, 48, 80 or 240 groups, 252 for 36, ...): a thread then meets the same four channels in every element it visits
    // and loads their coefficients once.  Otherwise (more than 512 groups) it looks them up element by element.
    const int T = blockDim.x;
    const bool fixed = (T % C4) == 0;
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
    const int64_t per = ((total4 + gridDim.x - 1) / gridDim.x + T - 1) / T * T;
    // The ranges are taken from the end of the tensor backwards and dy / t are read with ordinary (cached) loads: the
    // partial-sum pass has just read both tensors front to back, so what it read last is what the memory-side cache
    // still holds (measured: 2-3 % on the ResNet-50 layers against front-to-back streaming loads).
    const int64_t r0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * per;
    const int64_t r1 = r0 + per < total4 ? r0 + per : total4;
    if (fixed) load((int)(threadIdx.x % C4));
    for (int64_t base = r0 + threadIdx.x; base < r1; base += U * T) {
        f4 g[U], v[U], o[U], rv[U], so[U];
        unsigned bits[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * T;
            bits[u] = 0;
            rv[u] = f4{0, 0, 0, 0};
            if (i >= r1) continue;
            g[u] = (*((const f4 *)dy + i));
            v[u] = (*((const f4 *)t + i));
            if (acc) o[u] = __builtin_nontemporal_load((const f4 *)dx + i);
            if (RM == 1) bits[u] = (unsigned)(mask[i >> 4] >> ((i & 15) * 4)) & 15u;
            if (RM >= 2) rv[u] = __builtin_nontemporal_load((const f4 *)rt + i);
            if (side && side_acc) so[u] = __builtin_nontemporal_load((const f4 *)side + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * T;
            if (i >= r1) continue;
            if (!fixed) load((int)(i % C4));
            float gg[4] = {g[u].x, g[u].y, g[u].z, g[u].w}, vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w}, r[4];
            relu_gate<RM>(gg, bits[u], rv[u]);
            if (side) {
                const f4 sg = f4{gg[0], gg[1], gg[2], gg[3]};
                __builtin_nontemporal_store(side_acc ? sg + so[u] : sg, (f4 *)side + i);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float xh = vv[j] * sc[j] + sh[j];
                r[j] = a[j] * (gg[j] - mb[j] - xh * mg[j]);
            }
            if (acc) { r[0] += o[u].x; r[1] += o[u].y; r[2] += o[u].z; r[3] += o[u].w; }
            __builtin_nontemporal_store(f4{r[0], r[1], r[2], r[3]}, (f4 *)dx + i);
        }
    }
}

void bn_bwd(hipStream_t st, const float *dy, const float *t, bool from_output, const float *gamma, const float *beta,
            const float *stats, float *dx, float *dgamma, float *dbeta, int64_t rows, int C, bool accumulate, float *scratch,
            size_t scratch_bytes, const void *relu_t, int relu_mode, bool six, float *side, bool side_acc) {
    if (rows <= 0) throw KernelError("BatchNorm: no rows");
    int rm = 0;
    if (relu_t) {
        if (relu_mode == RELU_FROM_MASK) rm = 1;
        else if (relu_mode == RELU_FROM_INPUT || relu_mode == RELU_FROM_OUTPUT) rm = six ? 3 : 2;
        else throw KernelError("BatchNorm backward: unknown ReLU mode");
    }
    int64_t floats = (int64_t)(scratch_bytes / 4) - 2 * C;    // tail of the scratch holds the two coefficient vectors
    BnGeom g = bn_geom(rows, C, floats, 2);
    float *coef = scratch + (int64_t)g.G * C * 2;
    const int64_t total4 = rows * (C / 4);
    const int grid = stream_grid(total4);
    const int acc = accumulate ? 1 : 0, sacc = side_acc ? 1 : 0;
#define BP(F, RM) hipLaunchKernelGGL((bn_bwd_partial<F, RM>), dim3(g.G, g.CB), dim3(256), 0, st, dy, relu_t, t, gamma, beta, stats, scratch, rows, C, g.TPR, g.slab)
    // threads of an apply workgroup: a multiple of the channel groups (so that a thread keeps its channels), at most 256
    // where one exists, the group count itself up to 512
    const int C4 = C / 4;
    const int apply_threads = 256 % C4 == 0 ? 256 : C4 <= 256 ? C4 * (256 / C4) : C4 <= 512 ? C4 : 256;
#define BA(F, RM) hipLaunchKernelGGL((bn_bwd_apply<F, RM>), dim3(grid), dim3(apply_threads), 0, st, dy, relu_t, t, gamma, beta, stats, (const float *)coef, dx, acc, side, sacc, total4, C)
#define BOTH(STEP)                                                                 \
    do {                                                                           \
        if (from_output) { switch (rm) { case 0: STEP(true, 0); break; case 1: STEP(true, 1); break; case 2: STEP(true, 2); break; default: STEP(true, 3); } } \
        else             { switch (rm) { case 0: STEP(false, 0); break; case 1: STEP(false, 1); break; case 2: STEP(false, 2); break; default: STEP(false, 3); } } \
    } while (0)
    // channel groups that leave lanes of the row-shared mapping idle take the flat mapping (same thread count as the apply pass)
    int slabs = g.G;
    if (g.C4 % g.TPR != 0 && apply_threads % C4 == 0) {
        const int m = apply_threads / C4;                                        // rows per sweep of a workgroup
        const int64_t slab_rows = (g.slab + m - 1) / m * m;
        slabs = (int)((rows + slab_rows - 1) / slab_rows);
        const int64_t slab4 = slab_rows * C4;
#define BF(F, RM) hipLaunchKernelGGL((bn_bwd_partial_flat<F, RM>), dim3(slabs), dim3(apply_threads), 0, st, dy, relu_t, t, gamma, beta, stats, scratch, total4, C, slab4)
        BOTH(BF);
#undef BF
    } else {
        BOTH(BP);
    }
    hipLaunchKernelGGL(bn_bwd_final, dim3((C + FIN_CH - 1) / FIN_CH), dim3(256), 0, st, (const float *)scratch, dgamma, dbeta, coef, rows, C, slabs);
    BOTH(BA);
#undef BOTH
#undef BA
#undef BP
    hip_check(hipGetLastError(), "bn_bwd launch");
}

}  // namespace monet
