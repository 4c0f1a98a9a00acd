/*
 * monet_kernels.h -- C ABI of the individual gfx950 operator kernels that monet_step runs.
 *
 * These are the operator implementations the schedule selects between (the paper's
 * Appendix D, "Operator optimizations": output-activated BatchNorm / ReLU backward,
 * ReLU backward from a 1-bit sign code, max-pool backward from an 8-bit window index,
 * convolution with selectable workspace, in-place activations; Appendix D also splits
 * the convolution backward into a parameter-gradient and an input-gradient operator).
 * Exported so that each kernel can be checked and timed on its own.
 *
 * All pointers are device pointers owned by the caller; activations N,H,W,C fp32,
 * filters K,R,S,C.  `stream` is a hipStream_t (NULL = default stream).  Calls only
 * enqueue work.  Return 0, or a negative monet_status with monet_last_error() set.
 */
#ifndef MONET_KERNELS_H
#define MONET_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* All three convolution kernels take `splits`: > 1 cuts the reduction into that many ranges -- more workgroups
 * for layers whose result is small, at the price of workspace (device memory, contents irrelevant before and
 * after the call).  The partial results are always added in range order, so a result depends on `splits` and
 * the workspace size only.
 *   splits > 1: ws >= splits * |result| floats; a second kernel adds the partial results.
 *   fwd, dgrad with splits == 1 and a workspace: only the tiles of the ragged last round (beyond a multiple of
 *     the 256 CUs) are cut, as far as the workspace allows (monet_conv_workspace_bytes gives the useful size);
 *     their partial tiles wait in ws and the workgroup that finishes a tile last adds them.  Arrival counts live
 *     in a table inside the library: convolution calls that overlap in time on one GPU (different streams) must
 *     not both pass such a workspace.  With ws == NULL nothing is cut.
 * Appendix D's workspace / speed trade-off of convolution algorithms is this choice.
 *
 * y[N,P,Q,K] = cross-correlation of x[N,H,W,C] with w[K,R,S,C], zero padding, no bias. */
int monet_conv_fwd(void *stream, const float *x, const float *w, float *y,
                   int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                   int splits, float *ws, size_t ws_bytes);
/* Puts the arrival table of the cut tiles back to zero (one small kernel on `stream`).  The convolution kernels leave
 * every entry at zero when they finish; a caller whose sequence of launches was broken off by an error (or by a reset of
 * the stream) calls this before the next monet_conv_fwd / monet_conv_dgrad that passes a workspace with splits == 1.
 * monet_step does it at the start of every step. */
int monet_conv_reset_arrivals(void *stream);
/* monet_conv_fwd followed by monet_bn_stats of its output, with the statistics' first level computed in the
 * convolution's epilogue instead of a pass over y (the largest of the fusions the executor applies between a
 * convolution and the BatchNorm behind it).  Needs C % 16 == 0 (a 1x1 layer: C % 4 == 0) and K % 4 == 0; ws / ws_bytes as for monet_conv_fwd
 * with splits == 1; scratch >= 8 * (G + ceil(G / 64)) * K bytes with G = ceil(N*P*Q / 64).  `stats` is bit-identical to monet_bn_stats(y)
 * called with the same scratch size. */
int monet_conv_fwd_bn_stats(void *stream, const float *x, const float *w, float *y,
                            int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                            float *ws, size_t ws_bytes, float *stats, float eps, float *scratch, size_t scratch_bytes);
/* monet_conv_fwd followed by monet_bn_apply of its output in place, with the apply step (one multiply-add per
 * element) done in the convolution's epilogue: the form a recomputed convolution takes when the BatchNorm behind it
 * is recomputed in place, because then the statistics are the forward pass's (Section 3: recomputation repeats the
 * forward operator; Appendix D: in-place operators).  `stats` = mean[K] then 1/sqrt(var+eps)[K] as monet_bn_stats
 * leaves them, `gamma`, `beta` [K].  winograd_m = 0: implicit GEMM (needs C % 16 == 0, or C % 4 == 0 for a 1x1 layer, and K % 4 == 0; ws / ws_bytes as for
 * monet_conv_fwd with splits == 1); winograd_m = 2 or 4: the Winograd form below (3x3 / stride 1 / pad 1 only, its
 * workspace); winograd_m = 5: the one-kernel F(4x4) form (monet_conv_winograd_fused, its workspace).  y is bit-identical
 * to the two separate calls. */
int monet_conv_fwd_bn_apply(void *stream, const float *x, const float *w, float *y,
                            int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int winograd_m,
                            float *ws, size_t ws_bytes, const float *gamma, const float *beta, const float *stats);
/* The same with the ReLU (six == 0) or ReLU6 (six != 0) behind the BatchNorm applied in the epilogue as well: the form
 * of a recomputed convolution -> BatchNorm -> ReLU chain whose sign mask was kept from the forward pass (Section 3:
 * recomputation repeats the forward operators; Appendix D: in-place operators).  relu_out == null: y holds the ReLU's
 * result, bit-identical to monet_conv_fwd_bn_apply followed by monet_relu_fwd in place.  relu_out != null (device,
 * shape of y, must not overlap x, y or ws): y holds the BatchNorm's output as monet_conv_fwd_bn_apply leaves it and
 * relu_out the ReLU's, as monet_relu_fwd(y -> relu_out) would write it.  mask == null: no sign code is written (the code
 * of a lean schedule was kept from the forward pass).  mask != null (device, ceil(N*P*Q*K / 64) words, must not overlap x,
 * y, relu_out or ws): the ReLU's 1-bit sign code, the words monet_relu_fwd would write; needs K % 64 == 0 and
 * winograd_m == 0 or 5 (the other forms return an error). */
int monet_conv_fwd_bn_relu(void *stream, const float *x, const float *w, float *y,
                           int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int winograd_m,
                           float *ws, size_t ws_bytes, const float *gamma, const float *beta, const float *stats, int six,
                           float *relu_out, uint64_t *mask);
/* Winograd F(m x m, 3x3) form of a 3x3 / stride 1 / pad 1 convolution, m = 2 or 4 (Section 4 lists Winograd among the
 * implementations an operator chooses from; Appendix D: workspace against time).  adjoint == 0: out = y[N,H,W,K] from
 * in = x[N,H,W,C] (needs C % 16 == 0, K % 4 == 0).  adjoint != 0: out = dx[N,H,W,C] (+)= from in = dy[N,H,W,K]
 * (K % 16 == 0, C % 4 == 0).  Workspace (device memory): P = (m+2)^2 transformed filters (P*K*C floats) plus, per image
 * of a chunk, P * ceil(H/m) * ceil(W/m) * (C + K) floats of transformed input and products (4 x the image's input and
 * output for m = 2, 2.25 x for m = 4).  The layer is worked through in chunks of as many whole images as ws holds: any
 * ws_bytes from the filters plus one image up is accepted, the result does not depend on it, and
 * monet_conv_winograd_workspace_bytes returns the size for chunks of about half a GiB (or the whole batch if smaller),
 * below which the launches get too small to run at full rate.  Smaller: error.  m = 4 needs 4 x fewer
 * multiplications than the direct form (m = 2: 2.25 x) and rounds about five times more coarsely (normwise error of
 * one layer about 2e-6). */
int monet_conv_winograd(void *stream, const float *in, const float *w, float *out, int N, int H, int W, int C, int K,
                        int m, int adjoint, int accumulate, float *ws, size_t ws_bytes);
int64_t monet_conv_winograd_workspace_bytes(int N, int H, int W, int C, int K, int m);
/* The same convolution (m = 4) in one kernel: input transform, the 36 products and the output transform without the
 * transformed tensors ever reaching memory -- the small-workspace end of Appendix D's trade-off.  Workspace: the
 * transformed filters only, 36 * round_up(out channels, 64) * reduction channels floats
 * (monet_conv_winograd_fused_workspace_bytes; out = K, reduction = C for the forward pass, exchanged for adjoint != 0).
 * Needs reduction channels % 8 == 0.  Reads the input once per 64 output channels, so it is the faster form for layers
 * with few channels on large maps and the slower one for many channels.  Same arithmetic as monet_conv_winograd with
 * m = 4 (results agree to rounding; the sums over channels run in the same order). */
int monet_conv_winograd_fused(void *stream, const float *in, const float *w, float *out, int N, int H, int W, int C, int K,
                              int adjoint, int accumulate, float *ws, size_t ws_bytes);
int64_t monet_conv_winograd_fused_workspace_bytes(int N, int H, int W, int C, int K, int adjoint);
/* Convolution through an explicit patch matrix (Section 4 "Forward Operator Optimization" / Appendix I: the
 * matrix-multiplication form of a convolution, one of the implementations whose workspace the solver trades against
 * time).  The patches of a chunk of whole images are written to the workspace as rows of R*S*C floats (padded with
 * zeros to a multiple of 16), then the chunk is one GEMM: y = col W^T (forward; accumulate != 0 adds into y), or
 * dW = sum over chunks of dy^T col (filter gradient, chunks added in image order).  Same tensors and layouts as
 * monet_conv_fwd / monet_conv_wgrad (device pointers, NHWC, filters K x R x S x C); needs K % 4 == 0.  ws / ws_bytes:
 * device workspace owned by the caller; its size decides the chunk (at least the patches of one image, the padded
 * filters and, for the filter gradient, the chunk's K x round_up(R*S*C, 16) result with its split-reduction parts;
 * a negative status otherwise).  monet_conv_im2col_workspace_bytes gives the recommended size (chunks of about
 * 256 MiB of patches; wgrad != 0 for the filter gradient).  Results agree with the implicit GEMM to rounding. */
int monet_conv_im2col_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int C, int K, int R, int S,
                          int stride, int pad, int accumulate, float *ws, size_t ws_bytes);
int monet_conv_im2col_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K, int R, int S,
                            int stride, int pad, float *ws, size_t ws_bytes);
int64_t monet_conv_im2col_workspace_bytes(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int wgrad);
/* First layers: forward pass and filter gradient of a convolution over a three-channel image (the networks of Section 5
 * all start with one; same definitions and layouts as monet_conv_fwd / monet_conv_wgrad with C = 3, same results to
 * rounding).  The input rows under a tile of output positions are staged in LDS as they lie in memory and read from
 * there by the matrix instruction, so no patch matrix is formed and no load goes element by element.  Needs R == S,
 * (R, stride) one of (7, 2), (3, 1), (3, 2), K one of 32, 64, 96, 128 and an output row of any width (rows wider than 224
 * positions are worked through in segments); a negative status otherwise, also where the input rows under a tile exceed
 * what the forward kernel stages per workgroup (the 7x7 filter with 32 output channels, or on rows wider than about 380
 * pixels).  Filter gradient: splits >= 2 and a device
 * workspace of min(splits, 1024, tiles) * K * R * S * 3 floats, tiles = N * ceil(P / rows per tile) * segments (partial
 * results of the workgroups, added in a fixed order: two calls agree bit for bit).  monet_conv_fwd (splits == 1, no
 * accumulation) and monet_conv_wgrad take these forms by themselves where they apply. */
int monet_conv_stem_fwd(void *stream, const float *x, const float *w, float *y, int N, int H, int W, int K, int R, int S, int stride, int pad);
int monet_conv_stem_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int K, int R, int S, int stride,
                          int pad, int splits, float *ws, size_t ws_bytes);
/* Filter gradient of a 1x1 / stride 1 / unpadded convolution with few channels on one side (the expansion and projection
 * layers of an inverted-residual block on its large maps): dw[K,1,1,C] = sum over the N*H*W positions of dy[.,k] x[.,c],
 * a reduction of the two activation tensors into a small matrix and so bound by reading them once (one more
 * implementation of an operator in the sense of Section 4; same result as monet_conv_wgrad to rounding).  Needs
 * C % 4 == 0, K % 4 == 0, min(C, K) <= 32, max(C, K) <= 192, splits >= 2, N*H*W >= 64 * min(splits, 256) and a device
 * workspace of at least min(splits, 256) * K * C floats (partial results of the workgroups, added in a fixed order: two
 * calls agree bit for bit); a negative status otherwise.  monet_conv_wgrad takes this form by itself where it applies. */
int monet_conv_pointwise_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K, int splits,
                               float *ws, size_t ws_bytes);
/* Filter gradient of such a layer in the same transformed domain: dw[K,3,3,C] = G^T [ sum over tiles (A dy A^T) .* (B^T d B) ] G
 * (C % 4 == 0, K % 4 == 0).  Workspace: the transformed input and output gradient of one chunk of images (as above),
 * two buffers of P*K*C floats (the transformed filter gradient and one chunk's share of it, added chunk after chunk)
 * and up to 1024 / (P * ceil(K/128) * ceil(C/128)) more of them for the partial sums of a chunk's reduction ranges;
 * monet_conv_winograd_wgrad_workspace_bytes returns the size for chunks of about half a GiB, smaller sizes down to one
 * image per chunk are accepted (the result then differs by rounding: another order of the sum over images). */
int monet_conv_winograd_wgrad(void *stream, const float *x, const float *dy, float *dw, int N, int H, int W, int C, int K,
                              int m, float *ws, size_t ws_bytes);
int64_t monet_conv_winograd_wgrad_workspace_bytes(int N, int H, int W, int C, int K, int m);
/* Workspace bytes for monet_conv_fwd (which = 0) / monet_conv_dgrad (which = 1) of this shape with `splits` ranges;
 * for splits == 1 the size that lets the ragged last round be cut as far as it pays (0: nothing to gain).
 * Negative: error code. */
int64_t monet_conv_workspace_bytes(int which, int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int splits);
/* dx[N,H,W,C] (+)= gradient of the above wrt x, from dy[N,P,Q,K]. */
int monet_conv_dgrad(void *stream, const float *dy, const float *w, float *dx,
                     int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int accumulate,
                     int splits, float *ws, size_t ws_bytes);
/* dw[K,R,S,C] = gradient wrt w (reduction over N,P,Q). */
int monet_conv_wgrad(void *stream, const float *x, const float *dy, float *dw,
                     int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                     int splits, float *ws, size_t ws_bytes);

/* BatchNorm over rows x C (rows = N*H*W): stats = mean[C] then 1/sqrt(var+eps)[C], biased variance.
 * scratch: >= 4 MiB of device memory for slab partials. */
int monet_bn_stats(void *stream, const float *x, float *stats, int64_t rows, int C, float eps,
                   float *scratch, size_t scratch_bytes);
/* monet_bn_stats for callers that cannot allocate device memory or pass a scratch buffer (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the partial results live in a 4 MiB array inside the library,
 * one copy per GPU, held until the process ends.  Allocates nothing.  `stats` is bit-identical to monet_bn_stats called
 * with a 4 MiB scratch.  Limits: C a multiple of 4 and at most 8192, rows at most 2^31; beyond them the call returns an
 * error and enqueues nothing.  All calls on one GPU share the array (it keeps the last call's contents; every value a
 * call reads it has written itself, so nothing needs clearing): calls that overlap in time on one GPU, e.g. on two
 * streams, race and must be serialised by the caller. */
int monet_bn_stats_static(void *stream, const float *x, float *stats, int64_t rows, int C, float eps);
/* y = gamma*(x-mean)*invstd + beta; y may alias x (in-place variant). */
int monet_bn_apply(void *stream, const float *x, float *y, const float *gamma, const float *beta,
                   const float *stats, int64_t rows, int C);
/* t = BatchNorm input (from_output = 0) or its own output (from_output = 1, needs gamma != 0). */
int monet_bn_bwd(void *stream, const float *dy, const float *t, int from_output,
                 const float *gamma, const float *beta, const float *stats,
                 float *dx, float *dgamma, float *dbeta, int64_t rows, int C, int accumulate,
                 float *scratch, size_t scratch_bytes);

/* y = max(x,0) (six: min(.,6)); mask (may be NULL) gets one bit per element, ceil(n/64) words. y may alias x. */
int monet_relu_fwd(void *stream, const float *x, float *y, uint64_t *mask, int64_t n, int six);
/* mode 0: t = forward input, 1: t = forward output, 2: t = packed mask. */
int monet_relu_bwd(void *stream, const float *dz, const void *t, int mode, float *dx, int64_t n, int six, int accumulate);

/* k x k max pool; idx (may be NULL) gets r*k+s of the first maximum per output element. */
int monet_maxpool_fwd(void *stream, const float *x, float *y, uint8_t *idx,
                      int N, int H, int W, int C, int k, int stride, int pad);
/* from idx if non-NULL, else from x. */
int monet_maxpool_bwd(void *stream, const float *dy, const float *x, const uint8_t *idx, float *dx,
                      int N, int H, int W, int C, int k, int stride, int pad, int accumulate);

/* Transposed convolution without padding (the up-sampling layer of encoder-decoder networks):
 * y[N,(H-1)*stride+R,(W-1)*stride+S,K] = sum_c x[n,h,v,c] * w[c,r,s,k] scattered to (h*stride+r, v*stride+s).
 * w is C,R,S,K.  Runs on the convolution kernels above with the roles of the operands exchanged. */
int monet_tconv_fwd(void *stream, const float *x, const float *w, float *y,
                    int N, int H, int W, int C, int K, int R, int S, int stride);
int monet_tconv_dgrad(void *stream, const float *dy, const float *w, float *dx,
                      int N, int H, int W, int C, int K, int R, int S, int stride, int accumulate);
int monet_tconv_wgrad(void *stream, const float *x, const float *dy, float *dw,
                      int N, int H, int W, int C, int K, int R, int S, int stride,
                      int splits, float *ws, size_t ws_bytes);

/* Depthwise convolution: one R x S filter per channel (R*S <= 9), w is C,R,S; zero padding.
 * wgrad needs scratch of at least R*S*C floats (more lets more workgroups share the reduction). */
int monet_dwconv_fwd(void *stream, const float *x, const float *w, float *y,
                     int N, int H, int W, int C, int R, int S, int stride, int pad);
int monet_dwconv_dgrad(void *stream, const float *dy, const float *w, float *dx,
                       int N, int H, int W, int C, int R, int S, int stride, int pad, int accumulate);
int monet_dwconv_wgrad(void *stream, const float *x, const float *dy, float *dw,
                       int N, int H, int W, int C, int R, int S, int stride, int pad,
                       float *scratch, size_t scratch_bytes);

/* dst[row][0..cols) (+)= src[row][0..cols) for `rows` rows that are src_ld / dst_ld floats apart
 * (channel concatenation and its backward; base pointers already offset to the first column). */
int monet_column_copy(void *stream, const float *src, int64_t src_ld, float *dst, int64_t dst_ld,
                      int cols, int64_t rows, int accumulate);

/* Mean over rows of -log softmax(logits[row])[labels[row]] for rows of few classes (per-pixel scores),
 * and its gradient; scratch >= 4 KiB. */
int monet_softmaxce_rows_fwd(void *stream, const float *logits, const int32_t *labels, float *loss,
                             int64_t rows, int classes, float *scratch, size_t scratch_bytes);
int monet_softmaxce_rows_bwd(void *stream, const float *logits, const int32_t *labels, float *dlogits,
                             int64_t rows, int classes, int accumulate);

/* Tuning aid: force the workgroup tile of the three convolution kernels (0: 128x128, 1: 256x64,
 * 2: 64x256, 3: 128x64, 4: 64x128, 5: 64x64 as rows x columns of the implicit GEMM); -1 restores
 * the built-in choice.  Process-wide, not thread-safe. */
int monet_conv_force_tile(int cfg);

/* plain device copy, for bandwidth calibration */
int monet_copy(void *stream, const float *src, float *dst, int64_t n);

#ifdef __cplusplus
}
#endif
#endif /* MONET_KERNELS_H */
