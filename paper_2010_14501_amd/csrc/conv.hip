// Convolution forward, input-gradient and weight-gradient as implicit GEMMs on the fp32
// matrix cores of gfx950 (v_mfma_f32_32x32x2_f32), NHWC activations, KRSC filters.
//
//   forward : Y[m, k]   = sum_{r,s,c} X[n, p*st+r-pad, q*st+s-pad, c] * W[k, r, s, c]     m = (n,p,q)
//   dgrad   : dX[m, c]  = sum_{r,s,k} dY[n, (h+pad-r)/st, (w+pad-s)/st, k] * W[k, r, s, c] m = (n,h,w)
//   wgrad   : dW[k, j]  = sum_{m}     dY[m, k] * X[n, p*st+r-pad, q*st+s-pad, c]           j = (r,s,c)
//
// These are the convolution operator and the two backward operators it is split into in the
// paper's Appendix D (parameter-gradient, then input-gradient).  wgrad with splits > 1 writes
// one partial result per split into a workspace and sums them in split order: the workspace /
// time trade-off the schedule chooses between (Section 4, "Forward/Backward Operator
// Optimization").
//
// One workgroup computes a (64*WM) x (64*WN) tile with WM*WN waves, each wave a 64x64 sub-tile
// as 2x2 MFMA blocks.  The reduction runs in steps of 16, double-buffered through LDS: global
// loads for step t+1 are issued into registers before step t's MFMAs and written to the other
// LDS buffer afterwards.  An operand whose reduction index is contiguous in memory is kept
// [row][16+4] in LDS and read as one 128-bit load per lane (lane group g = lane/32 takes
// reduction indices 8h+4g..8h+4g+3); the MFMA pairs index 8h+4g+j of both operands, so the
// order of the sum inside a step is permuted but complete.  An operand contiguous along its
// row/column index is kept [16][cols+4] and read with 32-bit loads under the same pairing.
#include "kernels.hpp"

namespace monet {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BK = 16;        // reduction step
constexpr int KC_LD = BK + 4; // row stride of a reduction-contiguous operand in LDS (floats)

enum ConvMode { FWD = 0, DGRAD = 1, WGRAD = 2 };

struct TileArgs {
    const float *a;   // FWD: x, DGRAD: dy, WGRAD: dy
    const float *b;   // FWD: w, DGRAD: w,  WGRAD: x
    float *out;       // FWD: y, DGRAD: dx, WGRAD: dw or workspace
    ConvShape cs;
    int64_t Mg;       // GEMM rows
    int Ng;           // GEMM columns
    int64_t Kg;       // reduction length
    int tiles_n;
    int64_t steps_per_split;   // WGRAD: reduction steps (of BK) handled by one blockIdx.z
    int accumulate;            // DGRAD: add into dx
};

__device__ inline float4 ld4(const float *p) { return *(const float4 *)p; }

template <int MODE, int WM, int WN, bool FAST>
__global__ __launch_bounds__(64 * WM * WN) void conv_tile_kernel(TileArgs ta) {
    constexpr int BM = 64 * WM, BN = 64 * WN, NT = 64 * WM * WN;
    constexpr bool A_KC = (MODE != WGRAD);          // A operand reduction-contiguous?
    constexpr bool B_KC = (MODE == FWD);
    constexpr int A_LD = A_KC ? KC_LD : BM + 4;
    constexpr int B_LD = B_KC ? KC_LD : BN + 4;
    constexpr int A_SZ = A_KC ? BM * KC_LD : BK * (BM + 4);
    constexpr int B_SZ = B_KC ? BN * KC_LD : BK * (BN + 4);
    constexpr int LA = BM * 4 / NT;                 // float4 slots per thread, A tile
    constexpr int LB = BN * 4 / NT;
    __shared__ float As[2][A_SZ];
    __shared__ float Bs[2][B_SZ];

    const ConvShape &cs = ta.cs;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g = lane >> 5;
    const int tile_n = blockIdx.x % ta.tiles_n;
    const int64_t tile_m = blockIdx.x / ta.tiles_n;
    const int64_t row0 = tile_m * BM;
    const int col0 = tile_n * BN;
    const int64_t RSC = cs.RSC();

    // reduction range of this workgroup
    int64_t kt0 = 0, kt1 = (ta.Kg + BK - 1) / BK;
    if (MODE == WGRAD) {
        kt0 = (int64_t)blockIdx.z * ta.steps_per_split;
        int64_t e = kt0 + ta.steps_per_split;
        kt1 = e < kt1 ? e : kt1;
    }

    // ---------------- per-slot constants of the A loader
    // reduction-contiguous A (FWD / DGRAD): slot = (row, float4 j): idx = tid + s*NT, row = idx/4, j = idx%4
    // row-contiguous A (WGRAD)            : slot = (red row, float4 along k): red = idx/(BM/4), k4 = idx%(BM/4)
    int64_t a_base[LA];
    int a_h0[LA], a_w0[LA];
    bool a_ok[LA];
#pragma unroll
    for (int s = 0; s < LA; ++s) {
        int idx = tid + s * NT;
        if (A_KC) {
            int64_t m = row0 + idx / 4;
            a_ok[s] = m < ta.Mg;
            int64_t mm = a_ok[s] ? m : 0;
            if (MODE == FWD) {
                int q = (int)(mm % cs.Q);
                int64_t t = mm / cs.Q;
                int p = (int)(t % cs.P);
                int n = (int)(t / cs.P);
                a_h0[s] = p * cs.stride - cs.pad;
                a_w0[s] = q * cs.stride - cs.pad;
                a_base[s] = (int64_t)n * cs.H * cs.W * cs.C;
            } else {   // DGRAD: m = (n,h,w) of dx
                int w = (int)(mm % cs.W);
                int64_t t = mm / cs.W;
                int h = (int)(t % cs.H);
                int n = (int)(t / cs.H);
                a_h0[s] = h + cs.pad;
                a_w0[s] = w + cs.pad;
                a_base[s] = (int64_t)n * cs.P * cs.Q * cs.K;
            }
        } else {
            int k4 = idx % (BM / 4);
            a_h0[s] = idx / (BM / 4);                       // red row within the step
            a_w0[s] = (int)(row0 + k4 * 4);                 // first out-channel of the float4
            a_ok[s] = a_w0[s] < cs.K;
            a_base[s] = 0;
        }
    }
    // ---------------- per-slot constants of the B loader
    int b_i0[LB], b_i1[LB], b_i2[LB];
    bool b_ok[LB];
#pragma unroll
    for (int s = 0; s < LB; ++s) {
        int idx = tid + s * NT;
        if (B_KC) {          // FWD: slot = (filter k, float4 j)
            b_i0[s] = col0 + idx / 4;
            b_ok[s] = b_i0[s] < cs.K;
            b_i1[s] = b_i2[s] = 0;
        } else {             // slot = (red row, float4 along the column index)
            int c4 = idx % (BN / 4);
            int col = col0 + c4 * 4;
            b_i0[s] = idx / (BN / 4);                       // red row within the step
            if (MODE == DGRAD) {
                b_i1[s] = col;                              // input channel c
                b_ok[s] = col < cs.C;
                b_i2[s] = 0;
            } else {         // WGRAD: column = (r,s,c)
                b_ok[s] = col < RSC;
                int cc = b_ok[s] ? col : 0;
                b_i1[s] = cc / cs.C;                        // r*S + s
                b_i2[s] = cc % cs.C;                        // c
            }
        }
    }

    float4 a_reg[LA], b_reg[LB];

    auto load_tiles = [&](int64_t kt) {
        const int64_t kk0 = kt * BK;
        // ======== A
#pragma unroll
        for (int s = 0; s < LA; ++s) {
            int idx = tid + s * NT;
            float4 v = make_float4(0, 0, 0, 0);
            if (MODE == FWD) {
                const int j4 = (idx % 4) * 4;
                if (FAST) {
                    int rs = (int)(kk0 / cs.C), c0 = (int)(kk0 % cs.C);
                    int r = rs / cs.S, ss = rs % cs.S;
                    int h = a_h0[s] + r, w = a_w0[s] + ss;
                    if (a_ok[s] && (unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                        v = ld4(ta.a + a_base[s] + ((int64_t)h * cs.W + w) * cs.C + c0 + j4);
                } else {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        int64_t kk = kk0 + j4 + u;
                        if (a_ok[s] && kk < ta.Kg) {
                            int rs = (int)(kk / cs.C), c = (int)(kk % cs.C);
                            int r = rs / cs.S, ss = rs % cs.S;
                            int h = a_h0[s] + r, w = a_w0[s] + ss;
                            if ((unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                                e[u] = ta.a[a_base[s] + ((int64_t)h * cs.W + w) * cs.C + c];
                        }
                    }
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else if (MODE == DGRAD) {
                const int j4 = (idx % 4) * 4;
                // reduction index = (r, s, k); FAST: K % 16 == 0 so a step stays inside one (r,s)
                if (FAST) {
                    int rs = (int)(kk0 / cs.K), k0 = (int)(kk0 % cs.K);
                    int r = rs / cs.S, ss = rs % cs.S;
                    int hn = a_h0[s] - r, wn_ = a_w0[s] - ss;
                    if (a_ok[s] && hn >= 0 && wn_ >= 0 && hn % cs.stride == 0 && wn_ % cs.stride == 0) {
                        int p = hn / cs.stride, q = wn_ / cs.stride;
                        if (p < cs.P && q < cs.Q) v = ld4(ta.a + a_base[s] + ((int64_t)p * cs.Q + q) * cs.K + k0 + j4);
                    }
                } else {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        int64_t kk = kk0 + j4 + u;
                        if (a_ok[s] && kk < ta.Kg) {
                            int rs = (int)(kk / cs.K), k = (int)(kk % cs.K);
                            int r = rs / cs.S, ss = rs % cs.S;
                            int hn = a_h0[s] - r, wn_ = a_w0[s] - ss;
                            if (hn >= 0 && wn_ >= 0 && hn % cs.stride == 0 && wn_ % cs.stride == 0) {
                                int p = hn / cs.stride, q = wn_ / cs.stride;
                                if (p < cs.P && q < cs.Q) e[u] = ta.a[a_base[s] + ((int64_t)p * cs.Q + q) * cs.K + k];
                            }
                        }
                    }
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else {   // WGRAD: A[red = m][row = k] = dy[m][k]
                int64_t m = kk0 + a_h0[s];
                if (m < ta.Kg) {
                    if (FAST) {
                        if (a_ok[s]) v = ld4(ta.a + m * cs.K + a_w0[s]);
                    } else {
                        float e[4] = {0, 0, 0, 0};
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (a_w0[s] + u < cs.K) e[u] = ta.a[m * cs.K + a_w0[s] + u];
                        v = make_float4(e[0], e[1], e[2], e[3]);
                    }
                }
            }
            a_reg[s] = v;
        }
        // ======== B
#pragma unroll
        for (int s = 0; s < LB; ++s) {
            int idx = tid + s * NT;
            float4 v = make_float4(0, 0, 0, 0);
            if (MODE == FWD) {
                const int j4 = (idx % 4) * 4;
                if (FAST) {
                    if (b_ok[s]) v = ld4(ta.b + (int64_t)b_i0[s] * RSC + kk0 + j4);
                } else {
                    float e[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (b_ok[s] && kk0 + j4 + u < ta.Kg) e[u] = ta.b[(int64_t)b_i0[s] * RSC + kk0 + j4 + u];
                    v = make_float4(e[0], e[1], e[2], e[3]);
                }
            } else if (MODE == DGRAD) {
                // B[red = (r,s,k)][col = c] = W[k][r][s][c]
                int64_t kk = kk0 + b_i0[s];
                if (kk < ta.Kg) {
                    int rs = (int)(kk / cs.K), k = (int)(kk % cs.K);
                    const float *src = ta.b + (int64_t)k * RSC + (int64_t)rs * cs.C + b_i1[s];
                    if (FAST) {
                        if (b_ok[s]) v = ld4(src);
                    } else {
                        float e[4] = {0, 0, 0, 0};
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (b_i1[s] + u < cs.C) e[u] = src[u];
                        v = make_float4(e[0], e[1], e[2], e[3]);
                    }
                }
            } else {   // WGRAD: B[red = m][col = (r,s,c)] = x[n, p*st+r-pad, q*st+s-pad, c]
                int64_t m = kk0 + b_i0[s];
                if (m < ta.Kg) {
                    int q = (int)(m % cs.Q);
                    int64_t t = m / cs.Q;
                    int p = (int)(t % cs.P);
                    int n = (int)(t / cs.P);
                    int h0 = p * cs.stride - cs.pad, w0 = q * cs.stride - cs.pad;
                    const float *img = ta.b + (int64_t)n * cs.H * cs.W * cs.C;
                    if (FAST) {
                        int r = b_i1[s] / cs.S, ss = b_i1[s] % cs.S;
                        int h = h0 + r, w = w0 + ss;
                        if (b_ok[s] && (unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                            v = ld4(img + ((int64_t)h * cs.W + w) * cs.C + b_i2[s]);
                    } else {
                        float e[4] = {0, 0, 0, 0};
                        int col = col0 + (idx % (BN / 4)) * 4;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            int cc = col + u;
                            if (cc < RSC) {
                                int rs = cc / cs.C, c = cc % cs.C;
                                int r = rs / cs.S, ss = rs % cs.S;
                                int h = h0 + r, w = w0 + ss;
                                if ((unsigned)h < (unsigned)cs.H && (unsigned)w < (unsigned)cs.W)
                                    e[u] = img[((int64_t)h * cs.W + w) * cs.C + c];
                            }
                        }
                        v = make_float4(e[0], e[1], e[2], e[3]);
                    }
                }
            }
            b_reg[s] = v;
        }
    };

    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int s = 0; s < LA; ++s) {
            int idx = tid + s * NT;
            if (A_KC) *(float4 *)&As[buf][(idx / 4) * KC_LD + (idx % 4) * 4] = a_reg[s];
            else *(float4 *)&As[buf][(idx / (BM / 4)) * A_LD + (idx % (BM / 4)) * 4] = a_reg[s];
        }
#pragma unroll
        for (int s = 0; s < LB; ++s) {
            int idx = tid + s * NT;
            if (B_KC) *(float4 *)&Bs[buf][(idx / 4) * KC_LD + (idx % 4) * 4] = b_reg[s];
            else *(float4 *)&Bs[buf][(idx / (BN / 4)) * B_LD + (idx % (BN / 4)) * 4] = b_reg[s];
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto compute = [&](int buf) {
        const float *A = As[buf], *B = Bs[buf];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float af[2][4], bf[2][4];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                int r = wm * 64 + mi * 32 + l32;
                if (A_KC) {
                    float4 v = *(const float4 *)&A[r * KC_LD + 8 * h + 4 * g];
                    af[mi][0] = v.x; af[mi][1] = v.y; af[mi][2] = v.z; af[mi][3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) af[mi][j] = A[(8 * h + 4 * g + j) * A_LD + r];
                }
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                int c = wn * 64 + ni * 32 + l32;
                if (B_KC) {
                    float4 v = *(const float4 *)&B[c * KC_LD + 8 * h + 4 * g];
                    bf[ni][0] = v.x; bf[ni][1] = v.y; bf[ni][2] = v.z; bf[ni][3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) bf[ni][j] = B[(8 * h + 4 * g + j) * B_LD + c];
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi][j], bf[ni][j], acc[mi][ni], 0, 0, 0);
        }
    };

    if (kt0 < kt1) {
        load_tiles(kt0);
        store_tiles(0);
        __syncthreads();
        int buf = 0;
        for (int64_t kt = kt0; kt < kt1; ++kt) {
            const bool more = kt + 1 < kt1;
            if (more) load_tiles(kt + 1);
            compute(buf);
            if (more) store_tiles(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }

    // ---------------- epilogue: lane holds column l32 of rows 8*(v/4) + 4*g + v%4 of each 32x32 block
    float *out = ta.out;
    if (MODE == WGRAD) out += (int64_t)blockIdx.z * ta.Mg * ta.Ng;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            int col = col0 + wn * 64 + ni * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int64_t row = row0 + wm * 64 + mi * 32 + 8 * (v / 4) + 4 * g + (v % 4);
                if (row < ta.Mg && col < ta.Ng) {
                    float *dst = out + row * ta.Ng + col;
                    float r = acc[mi][ni][v];
                    if (MODE == DGRAD && ta.accumulate) r += *dst;
                    *dst = r;
                }
            }
        }
}

// sums `splits` partial results in split order
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ ws, float *__restrict__ dw, int64_t n, int splits) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float s = 0;
        for (int z = 0; z < splits; ++z) s += ws[(int64_t)z * n + i];
        dw[i] = s;
    }
}

void check_shape(const ConvShape &cs) {
    if (cs.N <= 0 || cs.H <= 0 || cs.W <= 0 || cs.C <= 0 || cs.K <= 0 || cs.R <= 0 || cs.S <= 0 || cs.stride <= 0 || cs.pad < 0)
        throw KernelError("conv: bad shape");
    if (cs.P != (cs.H + 2 * cs.pad - cs.R) / cs.stride + 1 || cs.Q != (cs.W + 2 * cs.pad - cs.S) / cs.stride + 1 || cs.P <= 0 || cs.Q <= 0)
        throw KernelError("conv: output size does not match input, filter, stride and padding");
    if ((int64_t)cs.R * cs.S * cs.C > (1ll << 30) || cs.M() > (1ll << 40)) throw KernelError("conv: shape too large");
}

template <int MODE, int WM, int WN>
void launch_tile(hipStream_t st, TileArgs ta, bool fast, int splits) {
    constexpr int BM = 64 * WM, BN = 64 * WN, NT = 64 * WM * WN;
    int64_t tiles_m = (ta.Mg + BM - 1) / BM;
    ta.tiles_n = (ta.Ng + BN - 1) / BN;
    int64_t blocks = tiles_m * ta.tiles_n;
    if (blocks > 0x7fffffffll) throw KernelError("conv: too many tiles");
    dim3 grid((unsigned)blocks, 1, (unsigned)splits);
    if (fast) hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, true>), grid, dim3(NT), 0, st, ta);
    else hipLaunchKernelGGL((conv_tile_kernel<MODE, WM, WN, false>), grid, dim3(NT), 0, st, ta);
    hip_check(hipGetLastError(), "conv launch");
}

}  // namespace

void conv_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs) {
    check_shape(cs);
    TileArgs ta{};
    ta.a = x; ta.b = w; ta.out = y; ta.cs = cs;
    ta.Mg = cs.M(); ta.Ng = cs.K; ta.Kg = cs.RSC();
    bool fast = cs.C % BK == 0;
    if (cs.K <= 64) launch_tile<FWD, 4, 1>(st, ta, fast, 1);
    else launch_tile<FWD, 2, 2>(st, ta, fast, 1);
}

void conv_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, const ConvShape &cs, bool accumulate) {
    check_shape(cs);
    TileArgs ta{};
    ta.a = dy; ta.b = w; ta.out = dx; ta.cs = cs;
    ta.Mg = (int64_t)cs.N * cs.H * cs.W; ta.Ng = cs.C; ta.Kg = (int64_t)cs.R * cs.S * cs.K;
    ta.accumulate = accumulate ? 1 : 0;
    bool fast = cs.K % BK == 0 && cs.C % 4 == 0;
    if (cs.C <= 64) launch_tile<DGRAD, 4, 1>(st, ta, fast, 1);
    else launch_tile<DGRAD, 2, 2>(st, ta, fast, 1);
}

void conv_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws, size_t ws_bytes) {
    check_shape(cs);
    if (splits < 1) throw KernelError("conv_wgrad: splits must be >= 1");
    TileArgs ta{};
    ta.a = dy; ta.b = x; ta.cs = cs;
    ta.Mg = cs.K; ta.Ng = (int)cs.RSC(); ta.Kg = cs.M();
    int64_t steps = (ta.Kg + BK - 1) / BK;
    if (splits > steps) splits = (int)steps;
    ta.steps_per_split = (steps + splits - 1) / splits;
    splits = (int)((steps + ta.steps_per_split - 1) / ta.steps_per_split);   // no empty split
    int64_t n = (int64_t)cs.K * cs.RSC();
    if (splits > 1) {
        if (!ws || ws_bytes < (size_t)splits * n * 4) throw KernelError("conv_wgrad: workspace too small for the requested splits");
        ta.out = ws;
    } else {
        ta.out = dw;
    }
    bool fast = cs.K % 4 == 0 && cs.C % 4 == 0;
    if (cs.K <= 64) launch_tile<WGRAD, 1, 2>(st, ta, fast, splits);
    else launch_tile<WGRAD, 2, 2>(st, ta, fast, splits);
    if (splits > 1) {
        int grid = (int)std::min<int64_t>((n + 255) / 256, 4096);
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(grid), dim3(256), 0, st, (const float *)ws, dw, n, splits);
        hip_check(hipGetLastError(), "wgrad reduce launch");
    }
}

}  // namespace monet
