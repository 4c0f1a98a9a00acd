// Winograd F(4x4, 3x3) in one kernel: input transform, the 36 products on the matrix cores and the output transform
// without the transformed input and the products ever reaching memory (Section 4 lists Winograd among the implementations
// an operator chooses from; Appendix D: workspace against time -- this is the small-workspace end: the workspace holds the
// transformed filters only).
//
//   Y = A^T [ (G g G^T) .* (B^T d B) ] A     per 6x6 input tile d, 3x3 filter g, 4x4 output tile Y (matrices: winograd.hip)
//
// A workgroup (four waves, one per SIMD) owns 32 tiles x 64 output channels for all 36 positions z of the transformed
// tile: wave w keeps the nine products z = 9w .. 9w+8 as 9 x 2 accumulator blocks of 32x32 (288 registers per lane).  The
// reduction runs over the input channels in chunks of 8:
//   * every thread loads the 6x6 patch of one (tile, channel) of the next chunk straight from the activation tensor
//     (neighbouring tiles overlap by two rows / columns; the overlap is served by the caches), transforms it in registers
//     and leaves V[z][tile][c] in one of two LDS buffers;
//   * the A operand of v_mfma_f32_32x32x2_f32 (lane -> tile l % 32, channel l / 32) is one LDS word per lane; the B
//     operand comes from the transformed filters, which the filter kernel below stores in exactly the order the lanes
//     read them (one 16-byte load per lane covers the four steps of a chunk), three positions ahead of their use.
// After the last chunk the accumulators go through LDS in two halves of 32 channels (36 x 32 x 32 floats each), and one
// thread per (tile, channel) applies A^T . A and writes the 4x4 outputs, optionally added to what is there (a second
// consumer's gradient) or followed by a BatchNorm apply step (recomputation).
//
// Traffic: the input once per block of 64 output channels (plus the tile overlap where the caches miss), the output once,
// the transformed filters from L2.  With many channels the input passes and the filter stream (36 x 64 floats per input
// channel and workgroup) cost more than the workspace form's large GEMM tiles save; the graph offers this form where it
// was measured to be faster.
#include "bn_affine.hpp"
#include "kernels.hpp"

namespace monet {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int FT = 32;            // tiles per workgroup
constexpr int FK = 64;            // output channels per workgroup
constexpr int FC = 8;             // reduction channels per chunk
constexpr int VROW = FC + 1;      // row of V[z][tile][.] in LDS, padded: 32 tiles x 9 words hit 32 different banks
constexpr int MROW = 33;          // row of M[z][tile][.] in LDS
constexpr int LDS_FLOATS = 36 * FT * MROW;               // 152 064 bytes; the two V buffers take the first 82 944
static_assert(2 * 36 * FT * VROW <= LDS_FLOATS, "V buffers must fit");

// the one-dimensional maps of F(4, 3) (the same arithmetic as the workspace form)
__device__ inline void f4_bt(float v0, float v1, float v2, float v3, float v4, float v5, float (&o)[6]) {
    o[0] = 4.0f * v0 - 5.0f * v2 + v4;
    o[1] = (v3 + v4) - 4.0f * (v1 + v2);
    o[2] = 4.0f * (v1 - v2) + (v4 - v3);
    o[3] = 2.0f * (v3 - v1) + (v4 - v2);
    o[4] = 2.0f * (v1 - v3) + (v4 - v2);
    o[5] = 4.0f * v1 - 5.0f * v3 + v5;
}
__device__ inline void f4_g(float g0, float g1, float g2, float (&o)[6]) {
    o[0] = 0.25f * g0;
    o[1] = (-1.0f / 6.0f) * (g0 + g1 + g2);
    o[2] = (-1.0f / 6.0f) * (g0 - g1 + g2);
    o[3] = (1.0f / 24.0f) * g0 + (1.0f / 12.0f) * g1 + (1.0f / 6.0f) * g2;
    o[4] = (1.0f / 24.0f) * g0 - (1.0f / 12.0f) * g1 + (1.0f / 6.0f) * g2;
    o[5] = g2;
}
__device__ inline void f4_at(float m0, float m1, float m2, float m3, float m4, float m5, float (&o)[4]) {
    const float p = m1 + m2, q = m1 - m2, r = m3 + m4, t = m3 - m4;
    o[0] = m0 + p + r;
    o[1] = q + 2.0f * t;
    o[2] = p + 4.0f * r;
    o[3] = q + 8.0f * t + m5;
}

// Transformed filters in the order the matrix-core lanes read them:
//   Up[z][out / 32][red / 8][lane][j],  lane = 32 * (red % 2) + out % 32,  j = (red % 8) / 2
// `out` runs over the output channels padded to a multiple of 64 (zeros), `red` over the reduction channels.
// ADJ: forward pass (out = K, red = C) or input gradient (out = C, red = K, filter turned by 180 degrees).
template <bool ADJ>
__global__ __launch_bounds__(256) void wino4_filter_fused_kernel(const float *__restrict__ w, float *__restrict__ Up, int K, int C, int out_pad) {
    const int outc = ADJ ? C : K, red = ADJ ? K : C;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)out_pad * red) return;
    const int o = (int)(idx / red), c = (int)(idx % red);
    float g[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s)
            g[r][s] = o >= outc ? 0.0f : (ADJ ? w[((int64_t)c * 9 + (2 - r) * 3 + (2 - s)) * C + o] : w[((int64_t)o * 9 + r * 3 + s) * C + c]);
    float t[3][6];      // t[s][a] = (G g)[a][s]
#pragma unroll
    for (int s = 0; s < 3; ++s) f4_g(g[0][s], g[1][s], g[2][s], t[s]);
    const int nch = red / FC, o32 = out_pad / 32;
    const int lane = 32 * (c & 1) + (o & 31), j = (c & 7) >> 1;
#pragma unroll
    for (int a = 0; a < 6; ++a) {
        float u[6];
        f4_g(t[0][a], t[1][a], t[2][a], u);
#pragma unroll
        for (int b = 0; b < 6; ++b) {
            const int z = 6 * a + b;
            Up[((((int64_t)z * o32 + (o >> 5)) * nch + (c >> 3)) * 64 + lane) * 4 + j] = u[b];
        }
    }
}


struct FusedGeom {
    int N, H, W, th, tw;
    int64_t T;          // tiles
    int red, outc;      // reduction / output channels
    int nch;            // red / 8
    int kblocks;        // ceil(outc / 64)
    int64_t items;      // ceil(T / 32) * kblocks
};

// The reduction loop of one wave: NZ positions z0 .. z0 + NZ - 1 of the 32 x 64 tile; PATCH: this wave also loads and
// transforms the input patches (one (tile, channel) per lane and chunk).
template <int NZ, bool PATCH>
__device__ __forceinline__ void fused_reduce(const float *__restrict__ x, const float *__restrict__ Up, float *lds, const FusedGeom &gm, int kb,
                                             int64_t tb, int z0, int ptid, int lane, floatx16 (&acc)[5][2]) {
    const int l32 = lane & 31, g = lane >> 5;
    const int H = gm.H, W = gm.W, red = gm.red, nch = gm.nch;
    // ---- the (tile, channel) whose patch this lane transforms
    // Patch element (a, b) of chunk ch sits at byte x + coff[b] + roff[a] + 32 * ch: coff / roff are the lane's own 32-bit
    // byte offsets of (image, row 0, column 4 * tj + b - 1, pc) and of row 4 * ti + a - 1, with row and column clamped into
    // the map, so that every load is in bounds; what lies outside the map is then replaced by zero (a wave whose 8 tiles
    // are all interior skips that).  The host checks that the tensor has fewer than 2^32 bytes.
    const int pc = ptid & 7, pt = ptid >> 3;
    unsigned rowok = 0, colok = 0;
    unsigned coff[6] = {0, 0, 0, 0, 0, 0}, roff[6] = {0, 0, 0, 0, 0, 0};
    if (PATCH) {
        const int64_t t = tb * FT + pt;
        if (t < gm.T) {
            const int tj = (int)(t % gm.tw);
            const int64_t r = t / gm.tw;
            const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
            const int h0 = 4 * ti - 1, w0 = 4 * tj - 1;
            const int64_t e = ((int64_t)n * H * W) * red + pc;
#pragma unroll
            for (int a = 0; a < 6; ++a) {
                if ((unsigned)(h0 + a) < (unsigned)H) rowok |= 1u << a;
                if ((unsigned)(w0 + a) < (unsigned)W) colok |= 1u << a;
                const int hc = min(max(h0 + a, 0), H - 1), wc = min(max(w0 + a, 0), W - 1);
                roff[a] = (unsigned)((int64_t)hc * W * red * 4);
                coff[a] = (unsigned)((e + (int64_t)wc * red) * 4);
            }
        }
    }
    const bool interior = PATCH && __all(rowok == 0x3fu && colok == 0x3fu);      // uniform over the wave
    float d[36];
    auto load_patch = [&](int ch) {
        const unsigned cbytes = (unsigned)ch * (FC * 4);
#pragma unroll
        for (int a = 0; a < 6; ++a)
#pragma unroll
            for (int b = 0; b < 6; ++b) d[a * 6 + b] = *(const float *)((const char *)x + (coff[b] + roff[a] + cbytes));
    };
    auto transform_store = [&](float *V) {
        if (!interior) {
#pragma unroll
            for (int a = 0; a < 6; ++a)
#pragma unroll
                for (int b = 0; b < 6; ++b)
                    if (!((rowok >> a) & (colok >> b) & 1u)) d[a * 6 + b] = 0.0f;
        }
        float m[6][6];      // m[b][a] = (B^T d)[a][b]
#pragma unroll
        for (int b = 0; b < 6; ++b) f4_bt(d[b], d[6 + b], d[12 + b], d[18 + b], d[24 + b], d[30 + b], m[b]);
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            float o[6];
            f4_bt(m[0][a], m[1][a], m[2][a], m[3][a], m[4][a], m[5][a], o);
#pragma unroll
            for (int b = 0; b < 6; ++b) V[((6 * a + b) * FT + pt) * VROW + pc] = o[b];
        }
    };

    // ---- B operands: position z0 + zi, channel blocks 2 * kb and 2 * kb + 1, chunk ch.  Loads return in the order they
    // were issued, so they are issued in the order of their use: the positions of chunk ch + 1 are requested while chunk ch
    // is multiplied (each into the registers its predecessor just left), after the patch of chunk ch + 1, which is
    // requested first and used last.
    const int o32 = gm.kblocks * 2;
    const f4 *bbase = (const f4 *)Up + ((int64_t)z0 * o32 + 2 * kb) * nch * 64 + lane;
    const int64_t zstride = (int64_t)o32 * nch * 64, hstride = (int64_t)nch * 64;
    f4 bq[NZ][2];
    auto load_b = [&](int zi, int ch) {
        const f4 *p = bbase + zi * zstride + (int64_t)ch * 64;
        bq[zi][0] = p[0];
        bq[zi][1] = p[hstride];
    };

    if (PATCH) load_patch(0);
#pragma unroll
    for (int zi = 0; zi < NZ; ++zi) load_b(zi, 0);
    if (PATCH) transform_store(lds);
    __syncthreads();

    for (int ch = 0; ch < nch; ++ch) {
        const float *Vcur = lds + (ch & 1) * (36 * FT * VROW);
        float *Vnext = lds + ((ch + 1) & 1) * (36 * FT * VROW);
        // the last chunk requests its own operands once more instead of branching around the requests (nothing reads them)
        const int nx = ch + 1 < nch ? ch + 1 : ch;
        if (PATCH) load_patch(nx);
        // The scheduler must not sink the requests towards their use (it would, to save registers): the order of the
        // sections below is the order of issue.
        __builtin_amdgcn_sched_barrier(0);
        const float *vp = Vcur + (z0 * FT + l32) * VROW + g;
        float a0 = vp[0], a1 = vp[2], a2 = vp[4], a3 = vp[6];
#pragma unroll
        for (int zi = 0; zi < NZ; ++zi) {
            const float c0 = a0, c1 = a1, c2 = a2, c3 = a3;
            if (zi + 1 < NZ) {      // A operands of the next position, read while this one multiplies
                const float *vn = vp + (zi + 1) * (FT * VROW);
                a0 = vn[0]; a1 = vn[2]; a2 = vn[4]; a3 = vn[6];
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0, bq[zi][0].x, acc[zi][0], 0, 0, 0);
            acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0, bq[zi][1].x, acc[zi][1], 0, 0, 0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1, bq[zi][0].y, acc[zi][0], 0, 0, 0);
            acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1, bq[zi][1].y, acc[zi][1], 0, 0, 0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c2, bq[zi][0].z, acc[zi][0], 0, 0, 0);
            acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c2, bq[zi][1].z, acc[zi][1], 0, 0, 0);
            acc[zi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(c3, bq[zi][0].w, acc[zi][0], 0, 0, 0);
            acc[zi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c3, bq[zi][1].w, acc[zi][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            load_b(zi, nx);      // into the registers the products above have just read
            __builtin_amdgcn_sched_barrier(0);
        }
        if (PATCH) transform_store(Vnext);
        __syncthreads();      // V[next] complete; every wave is done reading V[cur]
    }
}

// Eight waves, two per SIMD: waves 0-3 multiply five positions each (z = 5w ..), waves 4-7 four positions each
// (z = 20 + 4(w - 4) ..) and transform the input patches, so that on every SIMD the transform arithmetic of one wave runs
// beside the matrix-core work of the other.
template <bool ADJ>
__global__ __launch_bounds__(512) void wino4_fused_kernel(const float *__restrict__ x, const float *__restrict__ Up, float *y, FusedGeom gm,
                                                          int accumulate, BnAffine bn) {
    __shared__ float lds[LDS_FLOATS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    // Work item: hardware deals workgroups to the 8 XCDs in turn; item = (id mod 8) * (grid / 8) + id / 8 gives each XCD a
    // contiguous share, so that neighbouring tile rows (shared halo) and the channel blocks of one tile range (same input)
    // meet in one L2.  The grid is a multiple of 8; items beyond the last one do nothing.
    const int64_t grid = gridDim.x, id = blockIdx.x;
    const int64_t item = (id & 7) * (grid >> 3) + (id >> 3);
    if (item >= gm.items) return;
    const int kb = (int)(item % gm.kblocks);
    const int64_t tb = item / gm.kblocks;
    const int H = gm.H, W = gm.W;

    floatx16 acc[5][2];
#pragma unroll
    for (int zi = 0; zi < 5; ++zi)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[zi][h][i] = 0.0f;
    const bool heavy = wave < 4;
    const int z0 = heavy ? 5 * wave : 20 + 4 * (wave - 4), nz = heavy ? 5 : 4;
    if (heavy) fused_reduce<5, false>(x, Up, lds, gm, kb, tb, z0, 0, lane, acc);
    else fused_reduce<4, true>(x, Up, lds, gm, kb, tb, z0, tid - 256, lane, acc);

    // ---- output transform, 32 channels at a time
    const int ok_ = tid & 31, oq = tid >> 5;      // channel within the half, first of two tiles (oq, oq + 16)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int kout = kb * FK + h * 32 + ok_;
        if (kb * FK + h * 32 >= gm.outc) break;       // uniform over the workgroup
        if (h) __syncthreads();                        // the first half has been read
#pragma unroll
        for (int zi = 0; zi < 5; ++zi)
            if (zi < nz) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    lds[((z0 + zi) * FT + 8 * (i >> 2) + 4 * g + (i & 3)) * MROW + l32] = acc[zi][h][i];
            }
        __syncthreads();
        float bn_a = 1.0f, bn_b = 0.0f;
        if (!ADJ && bn.gamma && kout < gm.outc) bn_affine_coeffs(bn.gamma, bn.beta, bn.stats, gm.outc, kout, bn_a, bn_b);
        for (int q = 0; q < 2; ++q) {
            const int tl = oq + 16 * q;
            const int64_t t = tb * FT + tl;
            if (t >= gm.T || kout >= gm.outc) continue;
            const int tj = (int)(t % gm.tw);
            const int64_t r = t / gm.tw;
            const int ti = (int)(r % gm.th), n = (int)(r / gm.th);
            float s[6][4];      // s[b][a] = (A^T m)[a][b]
#pragma unroll
            for (int b = 0; b < 6; ++b) {
                float m[6];
#pragma unroll
                for (int a = 0; a < 6; ++a) m[a] = lds[((6 * a + b) * FT + tl) * MROW + ok_];
                f4_at(m[0], m[1], m[2], m[3], m[4], m[5], s[b]);
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int hh = 4 * ti + a;
                if (hh >= H) continue;
                float o[4];
                f4_at(s[0][a], s[1][a], s[2][a], s[3][a], s[4][a], s[5][a], o);
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int ww = 4 * tj + b;
                    if (ww >= W) continue;
                    float *dst = y + (((int64_t)n * H + hh) * W + ww) * gm.outc + kout;
                    float v = accumulate ? *dst + o[b] : o[b];
                    if (!ADJ && bn.gamma) v = bn_affine(v, bn_a, bn_b);
                    *dst = v;
                }
            }
        }
    }
}

}  // namespace

bool winograd_fused_applies(const ConvShape &cs, bool adjoint) {
    if (cs.R != 3 || cs.S != 3 || cs.stride != 1 || cs.pad != 1) return false;
    const int red = adjoint ? cs.K : cs.C, out = adjoint ? cs.C : cs.K;
    return red % FC == 0 && out >= 1;
}

size_t winograd_fused_workspace_bytes(const ConvShape &cs, bool adjoint) {
    const int red = adjoint ? cs.K : cs.C, out = adjoint ? cs.C : cs.K;
    return (size_t)36 * ((out + FK - 1) / FK * FK) * red * sizeof(float);
}

void conv_winograd_fused(hipStream_t st, const float *in, const float *w, float *out, const ConvShape &cs, bool adjoint, bool accumulate,
                         float *ws, size_t ws_bytes, const BnAffine *affine) {
    if (affine && (adjoint || accumulate || !affine->gamma || !affine->beta || !affine->stats))
        throw KernelError("conv_winograd_fused: a BatchNorm apply step goes with the forward form, without accumulation, and needs all coefficients");
    if (!winograd_fused_applies(cs, adjoint))
        throw KernelError("conv_winograd_fused: needs a 3x3 / stride 1 / pad 1 layer whose reduction channels are a multiple of 8");
    if (!ws || ws_bytes < winograd_fused_workspace_bytes(cs, adjoint))
        throw KernelError("conv_winograd_fused: workspace too small for the transformed filters");
    FusedGeom gm;
    gm.N = cs.N; gm.H = cs.H; gm.W = cs.W;
    gm.th = (cs.H + 3) / 4; gm.tw = (cs.W + 3) / 4;
    gm.T = (int64_t)cs.N * gm.th * gm.tw;
    gm.red = adjoint ? cs.K : cs.C;
    gm.outc = adjoint ? cs.C : cs.K;
    gm.nch = gm.red / FC;
    gm.kblocks = (gm.outc + FK - 1) / FK;
    gm.items = (gm.T + FT - 1) / FT * gm.kblocks;
    const int64_t grid = (gm.items + 7) / 8 * 8;
    if (gm.T < 1 || grid >= 0x7fffffffll || (int64_t)cs.N * cs.H * cs.W * gm.red >= ((int64_t)1 << 30))
        throw KernelError("conv_winograd_fused: shape out of range (the input must have fewer than 2^32 bytes)");
    const int out_pad = gm.kblocks * FK;
    const int64_t fe = (int64_t)out_pad * gm.red;
    const dim3 fg((unsigned)((fe + 255) / 256)), blk(256), wg(512);
    const BnAffine bn = affine ? *affine : BnAffine{};
    const int acc = accumulate ? 1 : 0;
    if (adjoint) {
        hipLaunchKernelGGL(wino4_filter_fused_kernel<true>, fg, blk, 0, st, w, ws, cs.K, cs.C, out_pad);
        hipLaunchKernelGGL(wino4_fused_kernel<true>, dim3((unsigned)grid), wg, 0, st, in, (const float *)ws, out, gm, acc, bn);
    } else {
        hipLaunchKernelGGL(wino4_filter_fused_kernel<false>, fg, blk, 0, st, w, ws, cs.K, cs.C, out_pad);
        hipLaunchKernelGGL(wino4_fused_kernel<false>, dim3((unsigned)grid), wg, 0, st, in, (const float *)ws, out, gm, acc, bn);
    }
    hip_check(hipGetLastError(), "fused winograd launch");
}

}  // namespace monet
