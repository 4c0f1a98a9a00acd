"""Operator definitions of the oracle: fp64, NCHW, textbook forms (test infrastructure).

The training step the paper schedules is exact: any schedule reaches the
gradients of plain back-propagation (Section 3, Algorithms 1 and 2), so each
operator here is the plain definition written out.  Convolution is
cross-correlation with zero padding and no bias; BatchNorm is training-mode
with biased variance; the operator variants of Appendix D ("Operator
optimizations": output-activated BatchNorm/ReLU backward, ReLU backward from
a 1-bit sign code, max-pool backward from an 8-bit window index) are written
next to the input-activated forms they must agree with.

Layout note: arrays are N,C,H,W and weights K,C,R,S here.  The packed sign
mask is the only place where a storage order matters; it is packed in N,H,W,C
order (the order the graph text declares for activations).
"""
import numpy as np

F64 = np.float64


# ---------------------------------------------------------------- convolution
def _pad(x, pad):
    if pad == 0:
        return x
    return np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))


def conv_out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv2d_fwd(x, w, stride, pad):
    """y[n,k,p,q] = sum_{c,r,s} xpad[n,c,p*stride+r,q*stride+s] * w[k,c,r,s]."""
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    xp = _pad(x, pad)
    y = np.zeros((N, K, P, Q), F64)
    for r in range(R):
        for s in range(S):
            win = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            y += np.einsum("ncpq,kc->nkpq", win, w[:, :, r, s], optimize=True)
    return y


def conv2d_wgrad(x, dy, R, S, stride, pad):
    """dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * xpad[n,c,p*stride+r,q*stride+s]."""
    N, C, H, W = x.shape
    _, K, P, Q = dy.shape
    xp = _pad(x, pad)
    dw = np.zeros((K, C, R, S), F64)
    for r in range(R):
        for s in range(S):
            win = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            for n in range(N):      # sum over p,q as one matrix product per image: (K x PQ) (PQ x C)
                dw[:, :, r, s] += dy[n].reshape(K, P * Q) @ np.ascontiguousarray(win[n]).reshape(C, P * Q).T
    return dw


def conv2d_dgrad(dy, w, x_shape, stride, pad):
    """dx = transpose of conv2d_fwd in x: scatter dy*w back onto the padded input."""
    N, C, H, W = x_shape
    K, _, R, S = w.shape
    _, _, P, Q = dy.shape
    dxp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), F64)
    for r in range(R):
        for s in range(S):
            dxp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride] += np.einsum(
                "nkpq,kc->ncpq", dy, w[:, :, r, s], optimize=True)
    return dxp[:, :, pad:pad + H, pad:pad + W].copy()


# ---------------------------------------------------------------- transposed convolution
def tconv2d_fwd(x, w, stride):
    """y[n,k,h*stride+r,v*stride+s] += x[n,c,h,v] * w[c,k,r,s]  (no padding; w is C,K,R,S)."""
    N, C, H, W = x.shape
    C2, K, R, S = w.shape
    assert C == C2
    y = np.zeros((N, K, (H - 1) * stride + R, (W - 1) * stride + S), F64)
    for r in range(R):
        for s in range(S):
            y[:, :, r:r + stride * (H - 1) + 1:stride, s:s + stride * (W - 1) + 1:stride] += np.einsum(
                "nchv,ck->nkhv", x, w[:, :, r, s], optimize=True)
    return y


def tconv2d_dgrad(dy, w, stride):
    """dx[n,c,h,v] = sum_{k,r,s} dy[n,k,h*stride+r,v*stride+s] * w[c,k,r,s]."""
    C, K, R, S = w.shape
    N, _, HO, WO = dy.shape
    H, W = (HO - R) // stride + 1, (WO - S) // stride + 1
    dx = np.zeros((N, C, H, W), F64)
    for r in range(R):
        for s in range(S):
            win = dy[:, :, r:r + stride * (H - 1) + 1:stride, s:s + stride * (W - 1) + 1:stride]
            dx += np.einsum("nkhv,ck->nchv", win, w[:, :, r, s], optimize=True)
    return dx


def tconv2d_wgrad(x, dy, R, S, stride):
    """dw[c,k,r,s] = sum_{n,h,v} x[n,c,h,v] * dy[n,k,h*stride+r,v*stride+s]."""
    N, C, H, W = x.shape
    K = dy.shape[1]
    dw = np.zeros((C, K, R, S), F64)
    for r in range(R):
        for s in range(S):
            win = dy[:, :, r:r + stride * (H - 1) + 1:stride, s:s + stride * (W - 1) + 1:stride]
            for n in range(N):      # sum over h,v as one matrix product per image: (C x HW) (HW x K)
                dw[:, :, r, s] += x[n].reshape(C, H * W) @ np.ascontiguousarray(win[n]).reshape(K, H * W).T
    return dw


# ---------------------------------------------------------------- depthwise convolution
def dwconv2d_fwd(x, w, stride, pad):
    """y[n,c,p,q] = sum_{r,s} xpad[n,c,p*stride+r,q*stride+s] * w[c,0,r,s]  (one filter per channel)."""
    N, C, H, W = x.shape
    C2, one, R, S = w.shape
    assert C == C2 and one == 1
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    xp = _pad(x, pad)
    y = np.zeros((N, C, P, Q), F64)
    for r in range(R):
        for s in range(S):
            win = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            y += win * w[None, :, 0, r, s, None, None]
    return y


def dwconv2d_wgrad(x, dy, R, S, stride, pad):
    """dw[c,0,r,s] = sum_{n,p,q} dy[n,c,p,q] * xpad[n,c,p*stride+r,q*stride+s]."""
    N, C, H, W = x.shape
    _, _, P, Q = dy.shape
    xp = _pad(x, pad)
    dw = np.zeros((C, 1, R, S), F64)
    for r in range(R):
        for s in range(S):
            win = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            dw[:, 0, r, s] = (dy * win).sum(axis=(0, 2, 3))
    return dw


def dwconv2d_dgrad(dy, w, x_shape, stride, pad):
    """Transpose of dwconv2d_fwd in x."""
    N, C, H, W = x_shape
    _, _, R, S = w.shape
    _, _, P, Q = dy.shape
    dxp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), F64)
    for r in range(R):
        for s in range(S):
            dxp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride] += dy * w[None, :, 0, r, s, None, None]
    return dxp[:, :, pad:pad + H, pad:pad + W].copy()


# ---------------------------------------------------------------- channel concatenation
def concat_fwd(a, b):
    return np.concatenate([a, b], axis=1)


def concat_bwd(dy, channels_a):
    return dy[:, :channels_a].copy(), dy[:, channels_a:].copy()


# ---------------------------------------------------------------- batch norm
def bn_stats(x, eps):
    mean = x.mean(axis=(0, 2, 3))
    var = ((x - mean[None, :, None, None]) ** 2).mean(axis=(0, 2, 3))   # biased
    return mean, 1.0 / np.sqrt(var + eps)


def bn_apply(x, gamma, beta, mean, invstd):
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    return gamma[None, :, None, None] * xhat + beta[None, :, None, None]


def bn_fwd(x, gamma, beta, eps):
    mean, invstd = bn_stats(x, eps)
    return bn_apply(x, gamma, beta, mean, invstd), mean, invstd


def _bn_bwd_core(dy, xhat, gamma, invstd):
    m = dy.shape[0] * dy.shape[2] * dy.shape[3]
    dbeta = dy.sum(axis=(0, 2, 3))
    dgamma = (dy * xhat).sum(axis=(0, 2, 3))
    b = lambda v: v[None, :, None, None]
    dx = b(gamma * invstd) / m * (m * dy - b(dbeta) - xhat * b(dgamma))
    return dx, dgamma, dbeta


def bn_bwd_from_input(dy, x, gamma, mean, invstd):
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    return _bn_bwd_core(dy, xhat, gamma, invstd)


def bn_bwd_from_output(dy, y, gamma, beta, invstd):
    """Output-activated form: xhat is recovered from y (needs gamma != 0)."""
    xhat = (y - beta[None, :, None, None]) / gamma[None, :, None, None]
    return _bn_bwd_core(dy, xhat, gamma, invstd)


# ---------------------------------------------------------------- ReLU family
def relu_fwd(x):
    """x where x > 0, else 0 (so 0, -0.0 and NaN all give 0: the same strict predicate as the sign code)."""
    return np.where(x > 0, x, 0.0)


def relu6_fwd(x):
    return np.where(x > 0, np.minimum(x, 6.0), 0.0)


def relu_pass(x):
    """Elements through which ReLU passes gradient (strict: 0, -0.0 and NaN do not)."""
    return x > 0


def relu6_pass(x):
    return (x > 0) & (x < 6)


def pack_mask(pass_nchw):
    """1-bit code: bit (e & 63) of little-endian 64-bit word (e >> 6), e = N,H,W,C linear index."""
    stored = np.transpose(pass_nchw, (0, 2, 3, 1)) if pass_nchw.ndim == 4 else pass_nchw
    bits = np.ascontiguousarray(stored).ravel().astype(np.uint8)
    words = (bits.size + 63) // 64
    padded = np.zeros(words * 64, np.uint8)
    padded[:bits.size] = bits
    return np.packbits(padded, bitorder="little").view("<u8").copy()


def unpack_mask(words, nchw_shape):
    count = int(np.prod(nchw_shape))
    bits = np.unpackbits(np.ascontiguousarray(words).view(np.uint8), bitorder="little")[:count]
    if len(nchw_shape) != 4:
        return bits.reshape(nchw_shape).astype(bool)
    N, C, H, W = nchw_shape
    return np.transpose(bits.reshape(N, H, W, C), (0, 3, 1, 2)).astype(bool)


def relu_bwd_from_input(dz, x):
    return dz * relu_pass(x)


def relu_bwd_from_output(dz, z):
    return dz * (z > 0)


def relu_bwd_from_mask(dz, words):
    return dz * unpack_mask(words, dz.shape)


def relu6_bwd_from_input(dz, x):
    return dz * relu6_pass(x)


def relu6_bwd_from_output(dz, z):
    return dz * ((z > 0) & (z < 6))


# ---------------------------------------------------------------- pooling
def maxpool_fwd(x, k, stride, pad):
    """Max over k x k windows; index = r*k+s of the first maximum under a strict '>' scan,
    padded positions never selected."""
    N, C, H, W = x.shape
    P, Q = conv_out_hw(H, W, k, k, stride, pad)
    xp = np.full((N, C, H + 2 * pad, W + 2 * pad), -np.inf, F64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    best = np.full((N, C, P, Q), -np.inf, F64)
    idx = np.zeros((N, C, P, Q), np.uint8)
    for r in range(k):
        for s in range(k):
            win = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            take = win > best      # the scan starts at -inf, so the first in-bounds tap always wins once
            best = np.where(take, win, best)
            idx = np.where(take, np.uint8(r * k + s), idx)
    return best, idx


def maxpool_bwd_from_index(dy, idx, x_shape, k, stride, pad):
    N, C, H, W = x_shape
    _, _, P, Q = dy.shape
    dxp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), F64)
    for r in range(k):
        for s in range(k):
            sel = idx == (r * k + s)
            dxp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride] += dy * sel
    return dxp[:, :, pad:pad + H, pad:pad + W].copy()


def maxpool_bwd_from_input(dy, x, k, stride, pad):
    _, idx = maxpool_fwd(x, k, stride, pad)
    return maxpool_bwd_from_index(dy, idx, x.shape, k, stride, pad)


def avgpool_fwd(x):
    return x.mean(axis=(2, 3))


def avgpool_bwd(dy, x_shape):
    N, C, H, W = x_shape
    return np.broadcast_to(dy[:, :, None, None] / (H * W), x_shape).copy()


# ---------------------------------------------------------------- linear, losses
def linear_fwd(x, w, b):
    """y = flatten(x) w^T + b; a 4-D x (N,C,H,W) is flattened per image, w is then out,C,H,W."""
    n = x.shape[0]
    return x.reshape(n, -1) @ w.reshape(w.shape[0], -1).T + b[None, :]


def linear_wgrad(x, dy):
    n = x.shape[0]
    return (dy.T @ x.reshape(n, -1)).reshape((dy.shape[1],) + x.shape[1:]), dy.sum(axis=0)


def linear_dgrad(dy, w, x_shape=None):
    dx = dy @ w.reshape(w.shape[0], -1)
    return dx if x_shape is None else dx.reshape(x_shape)


def _rows(logits, labels):
    """Class scores as rows: a 4-D score map N,K,H,W (one label per pixel) becomes N*H*W rows of K."""
    if logits.ndim == 4:
        k = logits.shape[1]
        return np.transpose(logits, (0, 2, 3, 1)).reshape(-1, k), np.asarray(labels).reshape(-1)
    return logits, np.asarray(labels)



def softmaxce_fwd(logits, labels):
    """Mean over the batch (for a score map: over batch and pixels) of -log softmax(logits)[label]."""
    logits, labels = _rows(logits, labels)
    z = logits - logits.max(axis=1, keepdims=True)
    lse = np.log(np.exp(z).sum(axis=1))
    n = logits.shape[0]
    return float(np.mean(lse - z[np.arange(n), labels]))


def softmaxce_bwd(logits, labels):
    shape = logits.shape
    logits, labels = _rows(logits, labels)
    z = logits - logits.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    n = logits.shape[0]
    p[np.arange(n), labels] -= 1.0
    p /= n
    if len(shape) == 4:
        N, K, H, W = shape
        return np.transpose(p.reshape(N, H, W, K), (0, 3, 1, 2)).copy()
    return p


def sumloss_fwd(x):
    return float(x.sum())


def sumloss_bwd(x_shape):
    return np.ones(x_shape, F64)
