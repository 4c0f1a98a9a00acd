// Filter gradient of 1x1 convolutions with few channels on one side (MobileNetV2's expansion and projection layers on
// its large maps): dW[k][c] = sum over the N*H*W positions m of dy[m][k] * x[m][c] is a reduction of 1.5 GB of
// activations into a 96 x 16 matrix, i.e. bound by HBM; on the tile kernel of conv.hip its 16-32 channel side is
// padded to 64 columns and the padding, not the traffic, sets the time.  Here both operands go from memory straight
// into the lane layout of the matrix instruction, no LDS, and a wave streams a contiguous range of positions:
//
//   mfma_f32_32x32x2f32: D[32 x 32] += A[32 x 2] B[2 x 32]; lane l holds A[l % 32][l / 32] and B[l / 32][l % 32].
//   The reduction index is the position: the two halves of a wave take two consecutive positions m, m + 1.
//   "Wide" operand (the side with up to 192 channels) = A: lane (r, h) loads the 16 bytes wide[m + h][4 r .. 4 r + 3];
//   its four floats feed four accumulator blocks, block b holding the channels 4 r + b of rows r = 0 .. 31 -- one
//   coalesced 512-byte row segment per half wave covers 128 channels.  Channels beyond 128 come in blocks of 32 through
//   4-byte loads (lane (r, h): wide[m + h][128 + 32 j + r]).  "Narrow" operand (up to 32 channels) = B: lane (c, h)
//   loads narrow[m + h][c].
//   Lanes whose channel does not exist load channel 0 instead (a fixed per-lane offset, no select in the loop): what
//   they accumulate lands in rows / columns of D that are never written out.
//
// Every wave leaves its partial K x C result in the workspace; the fixed-order reduction of conv.hip adds them, so the
// result does not depend on timing and two runs agree bit for bit.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "kernels.hpp"

namespace monet {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// NF4: 0 / 1 groups of 128 wide channels through 16-byte loads; ND: further blocks of 32 wide channels through 4-byte loads.
// A workgroup of four waves streams one contiguous range of positions, group g of 16 positions going to wave g % 4 (so
// the workgroup, not the wave, is the unit that walks through memory: measured, 1024 independent per-wave streams ran
// at 4.7 TB/s and 4096 of them at 3 TB/s); the four accumulators meet through LDS in wave order.
template <int NF4, int ND>
__global__ __launch_bounds__(256) void pw_wgrad_kernel(const float *__restrict__ wide, const float *__restrict__ narrow, float *__restrict__ part,
                                                      int64_t M, int w, int n, int wide_is_k, int64_t rows_per_wg) {
    constexpr int NB = 4 * NF4 + ND;     // accumulator blocks
    constexpr int U = 8;                 // row pairs per group (two groups in flight per wave)
    __shared__ float red[NB * 16][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int r = lane & 31, h = lane >> 5;
    const int64_t m0 = std::min<int64_t>((int64_t)blockIdx.x * rows_per_wg, M);
    const int64_t m1 = std::min<int64_t>(m0 + rows_per_wg, M);
    floatx16 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
    // per-lane channel offsets (floats); an absent channel reads channel 0
    const int f4off = NF4 && 4 * r < w ? 4 * r : 0;
    int doff[ND > 0 ? ND : 1];
#pragma unroll
    for (int j = 0; j < ND; ++j) {
        const int ch = 128 * NF4 + 32 * j + r;
        doff[j] = ch < w ? ch : 0;
    }
    const int noff = r < n ? r : 0;
    const int64_t groups = (m1 - m0) / (2 * U);                              // whole groups of the workgroup's range
    const int64_t mine_groups = groups > wave ? (groups - wave + 3) / 4 : 0; // ... of which this wave takes wave, wave + 4, ...
    {
        const float *wp = wide + (m0 + 2 * U * wave + h) * (int64_t)w;
        const float *np = narrow + (m0 + 2 * U * wave + h) * (int64_t)n;
        // two register sets: the loads of the wave's next group are issued before the matrix instructions of the current one
        struct Set { float4 a4[U]; float ad[U][ND > 0 ? ND : 1], b[U]; };
        auto load = [&](Set &t) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (NF4) t.a4[u] = *(const float4 *)(wp + (int64_t)(2 * u) * w + f4off);
#pragma unroll
                for (int j = 0; j < ND; ++j) t.ad[u][j] = wp[(int64_t)(2 * u) * w + doff[j]];
                t.b[u] = np[(int64_t)(2 * u) * n + noff];
            }
            wp += (int64_t)(8 * U) * w;
            np += (int64_t)(8 * U) * n;
        };
        auto compute = [&](const Set &t) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (NF4) {
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(t.a4[u].x, t.b[u], acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(t.a4[u].y, t.b[u], acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(t.a4[u].z, t.b[u], acc[2], 0, 0, 0);
                    acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(t.a4[u].w, t.b[u], acc[3], 0, 0, 0);
                }
#pragma unroll
                for (int j = 0; j < ND; ++j) acc[4 * NF4 + j] = __builtin_amdgcn_mfma_f32_32x32x2f32(t.ad[u][j], t.b[u], acc[4 * NF4 + j], 0, 0, 0);
            }
        };
        Set s0, s1;
        if (mine_groups > 0) load(s0);
        for (int64_t g = 0; g < mine_groups; g += 2) {
            if (g + 1 < mine_groups) load(s1);
            __builtin_amdgcn_sched_barrier(0);
            compute(s0);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 2 < mine_groups) load(s0);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 1 < mine_groups) compute(s1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // the rows after the last whole group (fewer than 16), pair by pair on the last wave: a half wave whose row lies beyond
    // the range reads the range's last row and contributes zero
    if (wave == 3) {
        for (int64_t m = m0 + groups * 2 * U; m < m1; m += 2) {
            const bool ok = m + h < m1;
            const int64_t row = ok ? m + h : m1 - 1;
            const float *wp = wide + row * (int64_t)w, *np = narrow + row * (int64_t)n;
            const float bv = ok ? np[noff] : 0.0f;
            if (NF4) {
                const float4 a = *(const float4 *)(wp + f4off);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bv, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bv, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bv, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bv, acc[3], 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < ND; ++j) acc[4 * NF4 + j] = __builtin_amdgcn_mfma_f32_32x32x2f32(wp[doff[j]], bv, acc[4 * NF4 + j], 0, 0, 0);
        }
    }
    // waves 1, 2, 3 hand their accumulators to wave 0 in that order (one buffer, reused): ((w0 + w1) + w2) + w3
    for (int v = 1; v < 4; ++v) {
        if (wave == v) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) red[b * 16 + i][lane] = acc[b][i];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[b][i] += red[b * 16 + i][lane];
        }
        __syncthreads();
    }
    // the workgroup's partial result, laid out as dW[k][c]: lane holds column l % 32 (narrow channel) of rows
    // 8 (i / 4) + 4 (l / 32) + i % 4 of every block
    float *mine = part + (int64_t)blockIdx.x * w * n;
    const int col = r;
    if (wave == 0 && col < n) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 8 * (i / 4) + 4 * h + (i % 4);
                const int ch = b < 4 * NF4 ? 4 * row + b : 128 * NF4 + 32 * (b - 4 * NF4) + row;
                if (ch < w) mine[wide_is_k ? ch * n + col : col * w + ch] = acc[b][i];
            }
    }
}

// workgroups of a launch: one per CU, i.e. one wave per SIMD (measured on 272 x 112 x 112, 16 -> 96 channels: 329 us with
// 256 workgroups, 358 with 512, 423 with 1024; the other layers alike)
constexpr int PW_MAX_WG = 256;
struct PwPlan { bool ok; bool wide_is_k; int w, n, nf4, nd; };
PwPlan pw_plan(const ConvShape &cs) {
    PwPlan p{};
    if (cs.R != 1 || cs.S != 1 || cs.stride != 1 || cs.pad != 0 || cs.C % 4 || cs.K % 4) return p;
    p.wide_is_k = cs.K >= cs.C;
    p.w = p.wide_is_k ? cs.K : cs.C;
    p.n = p.wide_is_k ? cs.C : cs.K;
    if (p.n > 32 || p.w > 192) return p;
    p.nf4 = p.w > 64 ? 1 : 0;
    p.nd = p.nf4 ? (p.w > 128 ? (p.w - 128 + 31) / 32 : 0) : (p.w + 31) / 32;
    p.ok = true;
    return p;
}

}  // namespace

// the layers this form is for: 1x1, stride 1, one side at most 32 channels, the other at most 192, reduced over enough
// positions that streaming matters; the caller's `splits` >= 2 says how many partial results the workspace may hold, of
// which min(splits, 256) are used
bool pointwise_wgrad_applies(const ConvShape &cs, int splits, size_t ws_bytes) {
    const PwPlan p = pw_plan(cs);
    return p.ok && splits >= 2 && cs.M() >= (int64_t)64 * std::min(splits, PW_MAX_WG) &&
           ws_bytes >= (size_t)std::min(splits, PW_MAX_WG) * cs.K * cs.C * sizeof(float);
}

int pw_groups(int splits) { return std::min(splits, PW_MAX_WG); }

void pointwise_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws, size_t ws_bytes) {
    if (!pointwise_wgrad_applies(cs, splits, ws_bytes)) throw KernelError("pointwise_wgrad: shape, split count or workspace not supported");
    const PwPlan p = pw_plan(cs);
    const int64_t M = cs.M();
    const int wgs = pw_groups(splits);
    const int64_t rows_per_wg = 2 * ((M + 2 * (int64_t)wgs - 1) / (2 * (int64_t)wgs));      // even: a pair of rows per instruction
    const float *wide = p.wide_is_k ? dy : x, *narrow = p.wide_is_k ? x : dy;
    const dim3 grid((unsigned)wgs), block(256);
    const int wk = p.wide_is_k ? 1 : 0;
#define PW(F, D) hipLaunchKernelGGL((pw_wgrad_kernel<F, D>), grid, block, 0, st, wide, narrow, ws, M, p.w, p.n, wk, rows_per_wg)
    if (!p.nf4 && p.nd == 1) PW(0, 1);
    else if (!p.nf4) PW(0, 2);
    else if (p.nd == 0) PW(1, 0);
    else if (p.nd == 1) PW(1, 1);
    else PW(1, 2);
#undef PW
    hip_check(hipGetLastError(), "pointwise_wgrad launch");
    split_reduce(st, ws, dw, (int64_t)cs.K * cs.C, wgs, false);
}

}  // namespace monet
