// Fused forms of adjacent bandwidth-bound operators.  The schedule still lists the operators
// one by one (and the allocation trace is unchanged); when two of them run back to back the
// executor launches one kernel that does both, so the tensor between them is read or written
// once less.  Arithmetic per element is the same as in the separate kernels, so results are
// bit-identical to the unfused path.
//
//   forward : [BatchNorm apply | add] -> ReLU(6) (+ 1-bit mask), pre-activation kept if asked for
//   backward: ReLU(6) backward (mask / output / input) feeding up to two gradient tensors
//             (the residual add's backward is a fan-out), each written or accumulated
// The BatchNorm backward that takes its incoming gradient through a ReLU mask lives in bn.hip.
#include "kernels.hpp"

namespace monet {

namespace {

// spreads the low 16 bits of x to bit positions 0, 4, 8, ..., 60
__device__ inline uint64_t spread16(uint64_t x) {
    x &= 0xFFFFull;
    x = (x | (x << 24)) & 0x000000FF000000FFull;
    x = (x | (x << 12)) & 0x000F000F000F000Full;
    x = (x | (x << 6)) & 0x0303030303030303ull;
    x = (x | (x << 3)) & 0x1111111111111111ull;
    return x;
}

// Each thread owns four consecutive elements (one float4); a wave owns 256 consecutive elements,
// i.e. four mask words.  Word w of the wave collects, from lanes 16w..16w+15, bit 4*(l-16w)+j of
// element j of lane l: four ballots (one per j), each cut to the 16 lanes of the word and spread.
template <bool BN, bool ADD, bool PRE_OUT, bool SIX, bool MASK>
__global__ __launch_bounds__(256) void fwd_chain_kernel(const float *x, const float *x2, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, const float *__restrict__ stats, int C,
                                                        float *out_pre, float *out, uint64_t *__restrict__ mask, int64_t total4) {
    const int lane = threadIdx.x & 63;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int C4 = BN ? C / 4 : 1;
    const bool fixed = BN && (stride % C4) == 0;
    float a[4] = {1, 1, 1, 1}, b[4] = {0, 0, 0, 0};
    auto load_ab = [&](int g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = g * 4 + j;
            float s = gamma[c] * stats[C + c];
            a[j] = s;
            b[j] = beta[c] - stats[c] * s;
        }
    };
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (BN && fixed) load_ab((int)(i % C4));
    for (; i - lane < total4; i += stride) {      // i - lane is the wave's first index: the trip count is wave-uniform
        const bool valid = i < total4;
        float4 v = make_float4(0, 0, 0, 0);
        if (valid) {
            v = ((const float4 *)x)[i];
            if (ADD) { float4 w = ((const float4 *)x2)[i]; v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w; }
            if (BN) {
                if (!fixed) load_ab((int)(i % C4));
                v.x = v.x * a[0] + b[0]; v.y = v.y * a[1] + b[1]; v.z = v.z * a[2] + b[2]; v.w = v.w * a[3] + b[3];
            }
            if (PRE_OUT) ((float4 *)out_pre)[i] = v;
        }
        float e[4] = {v.x, v.y, v.z, v.w}, r[4];
        bool pass[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pass[j] = valid && (SIX ? (e[j] > 0.0f && e[j] < 6.0f) : (e[j] > 0.0f));
            r[j] = e[j] > 0.0f ? e[j] : 0.0f;
            if (SIX) r[j] = r[j] < 6.0f ? r[j] : 6.0f;
        }
        if (valid) ((float4 *)out)[i] = make_float4(r[0], r[1], r[2], r[3]);
        if (MASK) {
            uint64_t b0 = __ballot(pass[0]), b1 = __ballot(pass[1]), b2 = __ballot(pass[2]), b3 = __ballot(pass[3]);
            if (lane < 4) {
                int sh = 16 * lane;
                uint64_t word = spread16(b0 >> sh) | (spread16(b1 >> sh) << 1) | (spread16(b2 >> sh) << 2) | (spread16(b3 >> sh) << 3);
                int64_t first4 = i - lane + 16 * lane;          // first float4 index covered by this word
                if (first4 < total4) mask[(i - lane) / 16 + lane] = word;
            }
        }
    }
}

int chain_grid(int64_t total4) {
    int64_t want = (total4 + 256 * 4 - 1) / (256 * 4);
    int grid = (int)std::max<int64_t>(1, std::min<int64_t>(want, 8192));
    if (grid > 2) grid &= ~1;
    return grid;
}

}  // namespace

void fwd_chain(hipStream_t st, const float *x, const float *x2, const float *gamma, const float *beta, const float *stats, int C,
               float *out_pre, float *out, uint64_t *mask, int64_t n, bool six) {
    if (n <= 0) return;
    if (n % 4) throw KernelError("fused forward: element count must be a multiple of 4");
    const bool bn = gamma != nullptr, add = x2 != nullptr, pre = out_pre != nullptr, mk = mask != nullptr;
    if (bn && add) throw KernelError("fused forward: BatchNorm and add cannot be combined");
    if (bn && C % 4) throw KernelError("fused forward: C must be a multiple of 4");
    const int64_t total4 = n / 4;
    const int grid = chain_grid(total4);
#define FC(BN, ADD, PRE, SIX, MK) \
    hipLaunchKernelGGL((fwd_chain_kernel<BN, ADD, PRE, SIX, MK>), dim3(grid), dim3(256), 0, st, x, x2, gamma, beta, stats, C, out_pre, out, mask, total4)
#define FC_MK(BN, ADD, PRE, SIX) do { if (mk) FC(BN, ADD, PRE, SIX, true); else FC(BN, ADD, PRE, SIX, false); } while (0)
#define FC_SIX(BN, ADD, PRE) do { if (six) FC_MK(BN, ADD, PRE, true); else FC_MK(BN, ADD, PRE, false); } while (0)
#define FC_PRE(BN, ADD) do { if (pre) FC_SIX(BN, ADD, true); else FC_SIX(BN, ADD, false); } while (0)
    if (bn) FC_PRE(true, false);
    else if (add) FC_PRE(false, true);
    else FC_PRE(false, false);
#undef FC_PRE
#undef FC_SIX
#undef FC_MK
#undef FC
    hip_check(hipGetLastError(), "fused forward launch");
}

// ------------------------------------------------------------------ ReLU backward with fan-out
namespace {

template <int MODE, bool SIX>
__global__ __launch_bounds__(256) void relu_bwd_fanout_kernel(const float *__restrict__ dz, const void *__restrict__ t, float *d0, int acc0,
                                                              float *d1, int acc1, int64_t total4) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total4; i += stride) {
        float4 g = ((const float4 *)dz)[i];
        float gg[4] = {g.x, g.y, g.z, g.w}, r[4];
        if (MODE == RELU_FROM_MASK) {
            uint64_t word = ((const uint64_t *)t)[i >> 4];
            unsigned bits = (unsigned)(word >> ((i & 15) * 4)) & 15u;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = (bits >> j) & 1 ? gg[j] : 0.0f;
        } else {
            float4 f = ((const float4 *)t)[i];
            float ff[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bool pass = SIX ? (ff[j] > 0.0f && ff[j] < 6.0f) : (ff[j] > 0.0f);
                r[j] = pass ? gg[j] : 0.0f;
            }
        }
        if (d0) {
            float4 o = make_float4(r[0], r[1], r[2], r[3]);
            if (acc0) { float4 p = ((float4 *)d0)[i]; o.x += p.x; o.y += p.y; o.z += p.z; o.w += p.w; }
            ((float4 *)d0)[i] = o;
        }
        if (d1) {
            float4 o = make_float4(r[0], r[1], r[2], r[3]);
            if (acc1) { float4 p = ((float4 *)d1)[i]; o.x += p.x; o.y += p.y; o.z += p.z; o.w += p.w; }
            ((float4 *)d1)[i] = o;
        }
    }
}

}  // namespace

void relu_bwd_fanout(hipStream_t st, const float *dz, const void *t, int mode, float *d0, bool acc0, float *d1, bool acc1, int64_t n,
                     bool six) {
    if (n <= 0) return;
    if (n % 4) throw KernelError("fused ReLU backward: element count must be a multiple of 4");
    const int64_t total4 = n / 4;
    const int grid = chain_grid(total4);
#define RF(MODE, SIX) hipLaunchKernelGGL((relu_bwd_fanout_kernel<MODE, SIX>), dim3(grid), dim3(256), 0, st, dz, t, d0, acc0 ? 1 : 0, d1, acc1 ? 1 : 0, total4)
    if (mode == RELU_FROM_MASK) RF(RELU_FROM_MASK, false);
    else if (mode == RELU_FROM_INPUT || mode == RELU_FROM_OUTPUT) { if (six) RF(RELU_FROM_INPUT, true); else RF(RELU_FROM_INPUT, false); }
    else throw KernelError("fused ReLU backward: unknown mode");
#undef RF
    hip_check(hipGetLastError(), "fused ReLU backward launch");
}

}  // namespace monet
