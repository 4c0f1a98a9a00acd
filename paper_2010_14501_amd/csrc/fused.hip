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
#include "bn_affine.hpp"
#include "kernels.hpp"

namespace monet {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

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
//
// v = x; BN: v = a*v + b, kept in out_bn if that tensor has to exist; ADD: v += x2, kept in out_pre if
// that tensor has to exist; out = relu(v); mask bits.  BN and ADD together are the tail of a residual
// block (BatchNorm -> add -> ReLU) in one pass.
template <bool BN, bool ADD, bool SIX, bool MASK>
__global__ __launch_bounds__(256) void fwd_chain_kernel(const float *x, const float *x2, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, const float *__restrict__ stats, int C,
                                                        float *out_bn, float *out_pre, float *out, uint64_t *__restrict__ mask,
                                                        int64_t total4) {
    // Each workgroup streams one contiguous range (a multiple of 256 float4, so that wave boundaries fall
    // on mask words and a thread's channel group stays fixed whenever C/4 divides 256), four float4 per
    // thread in flight, streaming (non-temporal) loads and stores: tensors here are far larger than any cache.
    constexpr int U = 4;
    const int lane = threadIdx.x & 63;
    const int C4 = BN ? C / 4 : 1;
    const bool fixed = BN && (256 % C4) == 0;
    float a[4] = {1, 1, 1, 1}, b[4] = {0, 0, 0, 0};
    auto load_ab = [&](int g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bn_affine_coeffs(gamma, beta, stats, C, g * 4 + j, a[j], b[j]);
        }
    };
    const int64_t per = ((total4 + gridDim.x - 1) / gridDim.x + 255) / 256 * 256;
    const int64_t r0 = (int64_t)blockIdx.x * per;
    const int64_t r1 = r0 + per < total4 ? r0 + per : total4;
    if (BN && fixed) load_ab((int)(threadIdx.x % C4));
    for (int64_t base = r0 + threadIdx.x; base - lane < r1; base += U * 256) {      // base - lane: wave-uniform trip count
        f4 v[U], w[U];
        bool valid[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            valid[u] = i < r1;
            v[u] = f4{0, 0, 0, 0};
            w[u] = f4{0, 0, 0, 0};
            if (valid[u]) {
                v[u] = __builtin_nontemporal_load((const f4 *)x + i);
                if (ADD) w[u] = __builtin_nontemporal_load((const f4 *)x2 + i);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            if (i - lane >= r1) break;                                                // whole wave beyond the range
            if (valid[u] && BN) {
                if (!fixed) load_ab((int)(i % C4));
                v[u] = f4{bn_affine(v[u].x, a[0], b[0]), bn_affine(v[u].y, a[1], b[1]), bn_affine(v[u].z, a[2], b[2]), bn_affine(v[u].w, a[3], b[3])};
                if (out_bn) __builtin_nontemporal_store(v[u], (f4 *)out_bn + i);
            }
            if (ADD) v[u] += w[u];
            if (valid[u] && out_pre) __builtin_nontemporal_store(v[u], (f4 *)out_pre + i);
            float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w}, r[4];
            bool pass[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pass[j] = valid[u] && (SIX ? (e[j] > 0.0f && e[j] < 6.0f) : (e[j] > 0.0f));
                r[j] = e[j] > 0.0f ? e[j] : 0.0f;
                if (SIX) r[j] = r[j] < 6.0f ? r[j] : 6.0f;
            }
            if (valid[u]) __builtin_nontemporal_store(f4{r[0], r[1], r[2], r[3]}, (f4 *)out + i);
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
}

// one workgroup per 2048 float4 (32 KiB) up to 64 Ki workgroups: many short contiguous streams measured
// fastest for a plain copy on this chip
int chain_grid(int64_t total4) {
    int64_t want = (total4 + 2047) / 2048;
    return (int)std::max<int64_t>(1, std::min<int64_t>(want, 65536));
}

}  // namespace

void fwd_chain(hipStream_t st, const float *x, const float *x2, const float *gamma, const float *beta, const float *stats, int C,
               float *out_bn, float *out_pre, float *out, uint64_t *mask, int64_t n, bool six) {
    if (n <= 0) return;
    if (n % 4) throw KernelError("fused forward: element count must be a multiple of 4");
    const bool bn = gamma != nullptr, add = x2 != nullptr, mk = mask != nullptr;
    if (bn && C % 4) throw KernelError("fused forward: C must be a multiple of 4");
    if (!bn && out_bn) throw KernelError("fused forward: BatchNorm output requested without BatchNorm");
    const int64_t total4 = n / 4;
    const int grid = chain_grid(total4);
#define FC(BN, ADD, SIX, MK) \
    hipLaunchKernelGGL((fwd_chain_kernel<BN, ADD, SIX, MK>), dim3(grid), dim3(256), 0, st, x, x2, gamma, beta, stats, C, out_bn, out_pre, out, mask, total4)
#define FC_MK(BN, ADD, SIX) do { if (mk) FC(BN, ADD, SIX, true); else FC(BN, ADD, SIX, false); } while (0)
#define FC_SIX(BN, ADD) do { if (six) FC_MK(BN, ADD, true); else FC_MK(BN, ADD, false); } while (0)
    if (bn && add) FC_SIX(true, true);
    else if (bn) FC_SIX(true, false);
    else if (add) FC_SIX(false, true);
    else FC_SIX(false, false);
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
    // contiguous range per workgroup, four float4 per thread in flight, streaming loads and stores
    constexpr int U = 4;
    const int64_t per = ((total4 + gridDim.x - 1) / gridDim.x + 255) / 256 * 256;
    const int64_t r0 = (int64_t)blockIdx.x * per;
    const int64_t r1 = r0 + per < total4 ? r0 + per : total4;
    for (int64_t base = r0 + threadIdx.x; base < r1; base += U * 256) {
        f4 g[U], f[U], p0[U], p1[U];
        unsigned bits[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            if (i >= r1) continue;
            g[u] = __builtin_nontemporal_load((const f4 *)dz + i);
            if (MODE == RELU_FROM_MASK) {
                uint64_t word = ((const uint64_t *)t)[i >> 4];
                bits[u] = (unsigned)(word >> ((i & 15) * 4)) & 15u;
            } else {
                f[u] = __builtin_nontemporal_load((const f4 *)t + i);
            }
            if (d0 && acc0) p0[u] = __builtin_nontemporal_load((const f4 *)d0 + i);
            if (d1 && acc1) p1[u] = __builtin_nontemporal_load((const f4 *)d1 + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + u * 256;
            if (i >= r1) continue;
            float gg[4] = {g[u].x, g[u].y, g[u].z, g[u].w}, r[4];
            if (MODE == RELU_FROM_MASK) {
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = (bits[u] >> j) & 1 ? gg[j] : 0.0f;
            } else {
                float ff[4] = {f[u].x, f[u].y, f[u].z, f[u].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bool pass = SIX ? (ff[j] > 0.0f && ff[j] < 6.0f) : (ff[j] > 0.0f);
                    r[j] = pass ? gg[j] : 0.0f;
                }
            }
            const f4 o = f4{r[0], r[1], r[2], r[3]};
            if (d0) __builtin_nontemporal_store(acc0 ? o + p0[u] : o, (f4 *)d0 + i);
            if (d1) __builtin_nontemporal_store(acc1 ? o + p1[u] : o, (f4 *)d1 + i);
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
