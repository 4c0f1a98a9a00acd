// Launchers of the gfx950 kernels.  Plain device pointers and sizes; every launch goes to
// the given stream and returns without synchronising.  Host-side shape checks throw
// KernelError before anything is enqueued.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <stdexcept>
#include <string>

namespace monet {

struct KernelError : std::runtime_error {
    using std::runtime_error::runtime_error;
};

inline void hip_check(hipError_t e, const char *what) {
    if (e != hipSuccess) throw KernelError(std::string(what) + ": " + hipGetErrorString(e));
}

struct ConvShape {
    int N, H, W, C;      // input  N,H,W,C
    int K, R, S;         // filter K,R,S,C
    int stride, pad;
    int P, Q;            // output N,P,Q,K
    __host__ __device__ int64_t M() const { return (int64_t)N * P * Q; }
    __host__ __device__ int64_t RSC() const { return (int64_t)R * S * C; }
};

// A BatchNorm apply step folded into the kernel that produces its input (a recomputed convolution, whose
// statistics are known): device pointers gamma[K], beta[K], stats = mean[K] followed by invstd[K]; the kernel then
// writes gamma * (y - mean) * invstd + beta, with the bits bn_apply() would produce from y.
struct BnAffine {
    const float *gamma = nullptr, *beta = nullptr, *stats = nullptr;
    // a ReLU (1) or ReLU6 (2) that follows the BatchNorm, applied in the same epilogue: its result replaces the BatchNorm's
    // (relu_out == null: both in place) or goes to relu_out, a tensor of the output's shape, beside it
    int relu = 0;
    float *relu_out = nullptr;
    // ... and that ReLU's sign code, written as relu_fwd writes it (bit (e & 63) of word (e >> 6), e the element's linear
    // index, set where the value passes); needs a multiple of 64 output channels.  The implicit GEMM and the one-kernel
    // Winograd form take it, the other kernels refuse it.
    unsigned long long *mask = nullptr;
};
// which convolution kernels can write the sign code from their epilogue
bool conv_epilogue_writes_mask(const ConvShape &cs, bool winograd_fused);

// ---- convolution (implicit GEMM on fp32 MFMA)
// Every variant can cut its reduction into `splits` ranges: partial results go to ws (splits * |output|
// floats) and are added in range order.  splits == 1 needs no workspace.
// y (+)= conv(x, w)
// stats_part: if given, the epilogue also leaves BatchNorm's partial statistics of y (groups of 64 rows, the
// layout bn_stats() reads with partials_ready) there; needs conv_fwd_aligned(cs), K % 4 == 0, splits == 1, no accumulation.
// affine: if given, the BatchNorm apply step of y in the epilogue (same conditions as stats_part; not both).
// whether the forward pass takes its aligned loader: C % 16 == 0, or a 1x1 layer with C % 4 == 0
bool conv_fwd_aligned(const ConvShape &cs);
void conv_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs, int splits = 1, float *ws = nullptr,
              size_t ws_bytes = 0, bool accumulate = false, float *stats_part = nullptr, const BnAffine *affine = nullptr);
// dx (+)= transpose-conv of dy with w
void conv_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, const ConvShape &cs, bool accumulate, int splits = 1,
                float *ws = nullptr, size_t ws_bytes = 0);
// dw = sum over N,P,Q
void conv_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws,
                size_t ws_bytes);

// `batch` independent GEMMs out[z][rows][cols] = a[z][rows][red] b[z][cols][red]^T in one launch (red % 16 == 0, cols % 4 == 0)
// (adjoint_use only picks the kernel's name in profiles: the GEMMs of an input gradient are listed apart from a forward pass's)
void gemm_batched(hipStream_t st, const float *a, const float *b, float *out, int batch, int64_t rows, int cols, int red,
                  bool adjoint_use = false);
void gemm_tn_batched(hipStream_t st, const float *a, const float *b, float *out, int batch, int64_t red, int m, int n, int splits,
                     float *ws, size_t ws_bytes);
// Winograd F(4x4, 3x3) in one kernel (transformed input and products stay on chip): workspace = the transformed filters
// only, 36 * round_up(out channels, 64) * reduction channels floats.  Needs reduction channels % 8 == 0.
bool winograd_fused_applies(const ConvShape &cs, bool adjoint);
size_t winograd_fused_workspace_bytes(const ConvShape &cs, bool adjoint);
void conv_winograd_fused(hipStream_t st, const float *in, const float *w, float *out, const ConvShape &cs, bool adjoint, bool accumulate,
                         float *ws, size_t ws_bytes, const BnAffine *affine = nullptr);
// Winograd F(m x m, 3x3), m = 2 or 4, for 3x3 / stride 1 / pad 1 layers.  adjoint = false: out = y[N,H,W,K] from in = x[N,H,W,C]
// (C % 16 == 0, K % 4 == 0); adjoint = true: out = dx[N,H,W,C] from in = dy[N,H,W,K] (K % 16 == 0, C % 4 == 0).  Workspace:
// (m+2)^2 transformed filters and (m+2)^2 / m^2 times the input and the output of one chunk of whole images; the layer
// goes through in as many chunks as the workspace asks for (winograd_workspace_bytes: chunks of about half a GiB).
bool winograd_applies(const ConvShape &cs, bool adjoint);
size_t winograd_workspace_bytes(const ConvShape &cs, int m);
// affine (forward only, no accumulation): the BatchNorm apply step of y in the output transform
void conv_winograd(hipStream_t st, const float *in, const float *w, float *out, const ConvShape &cs, int m, bool adjoint, bool accumulate,
                   float *ws, size_t ws_bytes, const BnAffine *affine = nullptr);
// filter gradient in the same transformed domain: dw[K,3,3,C] = G^T [ sum over tiles (A dy A^T) .* (B^T d B) ] G
// (C % 4 == 0, K % 4 == 0); workspace winograd_wgrad_workspace_bytes
size_t winograd_wgrad_workspace_bytes(const ConvShape &cs, int m);
void conv_winograd_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int m, float *ws, size_t ws_bytes);

// ---- depthwise convolution (K == C, filters C,R,S; at most 9 taps); HBM-bound, no matrix cores
// affine: the BatchNorm apply step of y in the same kernel (only where dwconv_fwd_takes_affine)
void dwconv_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs, const BnAffine *affine = nullptr);
bool dwconv_fwd_takes_affine(const ConvShape &cs);
void dwconv_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, const ConvShape &cs, bool accumulate);
// two-level fixed-order reduction; scratch holds slabs * R*S*C floats
void dwconv_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, float *scratch, size_t scratch_bytes);

// Convolution through an explicit patch matrix of a chunk of whole images (im2col.hip): workspace decides the chunk.
bool conv_im2col_applies(const ConvShape &cs);
size_t conv_im2col_workspace_bytes(const ConvShape &cs, bool wgrad);      // recommended (patches of about 256 MiB per chunk)
void conv_im2col_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs, float *ws, size_t ws_bytes,
                     bool accumulate);
void conv_im2col_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, float *ws, size_t ws_bytes);

// First layers (three input channels; 7x7 / stride 2, 3x3 / stride 1 or 2; 32 .. 128 output channels): the input rows
// under a tile of output positions are staged in LDS as they lie in memory and read from there by the matrix instruction
// (stem.hip).  conv_fwd takes this path by itself where it applies.
bool stem_applies(const ConvShape &cs);
void stem_fwd(hipStream_t st, const float *x, const float *w, float *y, const ConvShape &cs);
// ... and their filter gradient: min(splits, 1024, tiles) workgroups leave partial results in ws (that many times
// K * R * S * 3 floats), added in a fixed order.  conv_wgrad takes this path by itself where it applies.
bool stem_wgrad_applies(const ConvShape &cs, int splits, size_t ws_bytes);
void stem_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws, size_t ws_bytes);

// out[i] (+)= sum over z < splits of ws[z * n + i], in a fixed order
void split_reduce(hipStream_t st, const float *ws, float *out, int64_t n, int splits, bool accumulate);
// Filter gradient of a 1x1 / stride-1 convolution with at most 32 channels on one side and at most 192 on the other
// (pointwise.hip): min(splits, 256) workgroups stream contiguous ranges of positions, their partial results (that many
// times K * C floats of workspace) are added in a fixed order.  conv_wgrad takes this path by itself where it applies.
bool pointwise_wgrad_applies(const ConvShape &cs, int splits, size_t ws_bytes);
void pointwise_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, const ConvShape &cs, int splits, float *ws, size_t ws_bytes);

// tuning aid: cfg 0..5 forces tile shape (2x2, 4x1, 1x4, 2x1, 1x2, 1x1 waves of 64x64); -1 restores the heuristic
void conv_force_tile(int cfg);
// workspace bytes of conv_fwd (which = 0) / conv_dgrad (which = 1) for `splits` ranges; for splits = 1 the bytes
// with which the ragged last round of tiles is cut as far as it pays (0 if there is nothing to gain)
size_t conv_workspace_bytes(int which, const ConvShape &cs, int splits);
// Zeroes the table in which the cut tiles of forward / input-gradient launches count their arrivals.  The kernels put
// every entry back themselves; this is for a stream on which an earlier sequence of launches ended in an error.
void conv_reset_arrivals(hipStream_t st);

// ---- BatchNorm over rows x C (rows = N*H*W), training mode, biased variance
constexpr int64_t kBnScratchFloats = 1 << 20;
// stats = mean[C] followed by invstd[C]; scratch holds per-slab partials
// partials_ready: the producer of x (a forward convolution given `stats_part`) has already left the per-group
// partial results in `scratch`; only the final merge runs.  Allowed only where bn_stats_in_row_groups() holds.
void bn_stats(hipStream_t st, const float *x, float *stats, int64_t rows, int C, float eps, float *scratch,
              size_t scratch_bytes, bool partials_ready = false);
// The same with the partial results in a 4 MiB array inside the library (no scratch argument, no allocation); result
// bit-identical to bn_stats() with a 4 MiB scratch.  Calls that overlap in time on one GPU share the array and race.
constexpr int kBnStaticMaxC = 8192;
constexpr int64_t kBnStaticMaxRows = (int64_t)1 << 31;
void bn_stats_static(hipStream_t st, const float *x, float *stats, int64_t rows, int C, float eps);
// true if the statistics of a rows x C tensor are built from groups of 64 rows (scratch: 2 floats per group and channel)
bool bn_stats_in_row_groups(int64_t rows, int C, size_t scratch_bytes);
void bn_apply(hipStream_t st, const float *x, float *y, const float *gamma, const float *beta, const float *stats,
              int64_t rows, int C);
// t is the BatchNorm input (from_output = false) or its own output (true).  With relu_t, dy is first passed through
// a ReLU backward (relu_mode: a ReluBwdMode; relu_t = that ReLU's input, output or 1-bit sign code) -- fused
// ReLU-backward + BatchNorm-backward; `side` (may be null) then also receives, or accumulates, the gated dy
// itself: the other branch of a residual add between the two.
void bn_bwd(hipStream_t st, const float *dy, const float *t, bool from_output, const float *gamma, const float *beta,
            const float *stats, float *dx, float *dgamma, float *dbeta, int64_t rows, int C, bool accumulate,
            float *scratch, size_t scratch_bytes, const void *relu_t = nullptr, int relu_mode = -1, bool six = false,
            float *side = nullptr, bool side_acc = false);

// ---- fused neighbours (same arithmetic as the separate kernels)
// v = x; if gamma: v = BatchNorm apply of v (kept in out_bn unless null); if x2: v += x2; out_pre (may be null)
// receives v; out = relu(v); mask (may be null) the sign code.  Outputs may alias an input at the same index.
void fwd_chain(hipStream_t st, const float *x, const float *x2, const float *gamma, const float *beta, const float *stats, int C,
               float *out_bn, float *out_pre, float *out, uint64_t *mask, int64_t n, bool six);
// ReLU backward written (or accumulated) into up to two gradient tensors
void relu_bwd_fanout(hipStream_t st, const float *dz, const void *t, int mode, float *d0, bool acc0, float *d1, bool acc1, int64_t n,
                     bool six);

// ---- ReLU / ReLU6; mask may be null; y may alias x
void relu_fwd(hipStream_t st, const float *x, float *y, uint64_t *mask, int64_t n, bool six);
enum ReluBwdMode { RELU_FROM_INPUT = 0, RELU_FROM_OUTPUT = 1, RELU_FROM_MASK = 2 };
void relu_bwd(hipStream_t st, const float *dz, const void *t, int mode, float *dx, int64_t n, bool six, bool accumulate);

// ---- pooling
struct PoolShape {
    int N, H, W, C, k, stride, pad, P, Q;
};
void maxpool_fwd(hipStream_t st, const float *x, float *y, uint8_t *idx, const PoolShape &ps);
// from x (idx == null) or from the stored window index
void maxpool_bwd(hipStream_t st, const float *dy, const float *x, const uint8_t *idx, float *dx, const PoolShape &ps,
                 bool accumulate);
void avgpool_fwd(hipStream_t st, const float *x, float *y, int N, int HW, int C);
void avgpool_bwd(hipStream_t st, const float *dy, float *dx, int N, int HW, int C, bool accumulate);

// ---- elementwise
void add_fwd(hipStream_t st, const float *a, const float *b, float *y, int64_t n);
void copy_or_accumulate(hipStream_t st, const float *src, float *dst, int64_t n, bool accumulate);
void fill_f32(hipStream_t st, float *dst, int64_t n, float v);
void fill_u32(hipStream_t st, uint32_t *dst, int64_t n, uint32_t v);

// dst[row][0..cols) (+)= src[row][0..cols); consecutive rows are src_ld / dst_ld floats apart
void column_copy(hipStream_t st, const float *src, int64_t src_ld, float *dst, int64_t dst_ld, int cols, int64_t rows, bool accumulate);

// ---- linear layer: y[N,out] = x[N,in] w[out,in]^T + b
// scratch (may be null): device memory for partial results of a split reduction
void linear_fwd(hipStream_t st, const float *x, const float *w, const float *b, float *y, int N, int in, int out, float *scratch = nullptr,
                size_t scratch_bytes = 0);
void linear_wgrad(hipStream_t st, const float *x, const float *dy, float *dw, float *db, int N, int in, int out);
void linear_dgrad(hipStream_t st, const float *dy, const float *w, float *dx, int N, int in, int out, bool accumulate,
                  float *scratch = nullptr, size_t scratch_bytes = 0);

// ---- losses; scratch >= N floats
void softmaxce_fwd(hipStream_t st, const float *logits, const int32_t *labels, float *loss, int N, int classes,
                   float *scratch);
void softmaxce_bwd(hipStream_t st, const float *logits, const int32_t *labels, float *dlogits, int N, int classes,
                   bool accumulate);
// the same loss for many rows of few classes (per-pixel scores): one thread per row; scratch >= 1024 floats
void softmaxce_rows_fwd(hipStream_t st, const float *logits, const int32_t *labels, float *loss, int64_t rows, int classes, float *scratch,
                        size_t scratch_bytes);
void softmaxce_rows_bwd(hipStream_t st, const float *logits, const int32_t *labels, float *dlogits, int64_t rows, int classes, bool accumulate);
void sumloss_fwd(hipStream_t st, const float *x, float *loss, int64_t n, float *scratch, size_t scratch_bytes);

}  // namespace monet
