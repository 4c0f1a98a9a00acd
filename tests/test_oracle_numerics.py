"""Pins for the oracle's operators: brute force on tiny inputs, closed forms, library special
cases, finite differences.  None of these re-types an oracle formula."""
import numpy as np
import pytest

from oracle import numerics as nm
from oracle import network as onet
from workloads import graphs, tensors

RNG = np.random.default_rng(1234)


# ------------------------------------------------------------------ helpers
def conv_loops(x, w, stride, pad):
    """7-loop cross-correlation straight from the index definition (tiny inputs only)."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, K, P, Q))
    for n in range(N):
        for k in range(K):
            for p in range(P):
                for q in range(Q):
                    acc = 0.0
                    for c in range(C):
                        for r in range(R):
                            for s in range(S):
                                h, v = p * stride + r - pad, q * stride + s - pad
                                if 0 <= h < H and 0 <= v < W:
                                    acc += x[n, c, h, v] * w[k, c, r, s]
                    y[n, k, p, q] = acc
    return y


def fd_grad(f, x, h=1e-6):
    """Central finite differences of scalar f at x."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = f()
        x[i] = old - h
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ------------------------------------------------------------------ convolution
@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (2, 3, 7), (1, 0, 1), (2, 0, 1)])
def test_conv_fwd_matches_index_definition(stride, pad, R):
    x = RNG.standard_normal((2, 3, 9, 8))
    w = RNG.standard_normal((4, 3, R, R))
    assert rel(nm.conv2d_fwd(x, w, stride, pad), conv_loops(x, w, stride, pad)) < 1e-14


def test_conv_1x1_is_matmul():
    x = RNG.standard_normal((2, 5, 4, 6))
    w = RNG.standard_normal((7, 5, 1, 1))
    y = nm.conv2d_fwd(x, w, 1, 0)
    ref = np.matmul(w[:, :, 0, 0], x.transpose(1, 0, 2, 3).reshape(5, -1)).reshape(7, 2, 4, 6).transpose(1, 0, 2, 3)
    assert rel(y, ref) < 1e-14


@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (2, 0, 1), (2, 3, 7)])
def test_conv_grads_by_finite_differences(stride, pad, R):
    x = RNG.standard_normal((2, 3, 8, 7))
    w = RNG.standard_normal((4, 3, R, R))
    y = nm.conv2d_fwd(x, w, stride, pad)
    dy = RNG.standard_normal(y.shape)
    f = lambda: float((nm.conv2d_fwd(x, w, stride, pad) * dy).sum())
    assert rel(nm.conv2d_dgrad(dy, w, x.shape, stride, pad), fd_grad(f, x)) < 1e-7
    assert rel(nm.conv2d_wgrad(x, dy, R, R, stride, pad), fd_grad(f, w)) < 1e-7


def test_conv_dgrad_is_adjoint_of_fwd():
    x = RNG.standard_normal((2, 3, 8, 8))
    w = RNG.standard_normal((5, 3, 3, 3))
    dy = RNG.standard_normal((2, 5, 4, 4))
    lhs = (nm.conv2d_fwd(x, w, 2, 1) * dy).sum()
    rhs = (x * nm.conv2d_dgrad(dy, w, x.shape, 2, 1)).sum()
    assert abs(lhs - rhs) < 1e-10 * abs(lhs)


# ------------------------------------------------------------------ batch norm
def test_bn_is_column_standardisation():
    x = RNG.standard_normal((4, 3, 5, 6)) * 3 + 2
    y, mean, invstd = nm.bn_fwd(x, np.ones(3), np.zeros(3), 0.0)
    cols = x.transpose(1, 0, 2, 3).reshape(3, -1)
    assert np.allclose(mean, cols.mean(axis=1), rtol=1e-14)
    assert np.allclose(invstd, 1 / cols.std(axis=1), rtol=1e-13)       # numpy std is the biased one
    ycols = y.transpose(1, 0, 2, 3).reshape(3, -1)
    assert np.allclose(ycols.mean(axis=1), 0, atol=1e-14)
    assert np.allclose(ycols.var(axis=1), 1, rtol=1e-12)


def test_bn_bwd_by_finite_differences_and_identities():
    x = RNG.standard_normal((3, 4, 5, 5))
    gamma = RNG.uniform(0.5, 1.5, 4)
    beta = RNG.standard_normal(4) * 0.1
    eps = 1e-5
    dy = RNG.standard_normal(x.shape)
    f = lambda: float((nm.bn_fwd(x, gamma, beta, eps)[0] * dy).sum())
    y, mean, invstd = nm.bn_fwd(x, gamma, beta, eps)
    dx, dg, db = nm.bn_bwd_from_input(dy, x, gamma, mean, invstd)
    assert rel(dx, fd_grad(f, x)) < 1e-7
    assert rel(dg, fd_grad(f, gamma)) < 1e-8
    assert rel(db, fd_grad(f, beta)) < 1e-8
    # closed-form identities: the input gradient is orthogonal to 1 and to xhat in every channel
    xhat = (x - mean[None, :, None, None]) * invstd[None, :, None, None]
    assert np.abs(dx.sum(axis=(0, 2, 3))).max() < 1e-12
    # (to xhat only up to eps: sum xhat^2 = m*var/(var+eps), which leaves gamma*invstd^3*eps*dgamma)
    assert np.allclose((dx * xhat).sum(axis=(0, 2, 3)), gamma * invstd ** 3 * eps * dg, rtol=1e-9, atol=1e-14)
    # output-activated form agrees
    dx2, dg2, db2 = nm.bn_bwd_from_output(dy, y, gamma, beta, invstd)
    assert rel(dx2, dx) < 1e-12 and rel(dg2, dg) < 1e-12 and rel(db2, db) < 1e-14


def test_bn_apply_with_saved_stats_reproduces_forward():
    x = RNG.standard_normal((3, 4, 5, 5))
    gamma, beta = RNG.uniform(0.5, 1.5, 4), RNG.standard_normal(4)
    y, mean, invstd = nm.bn_fwd(x, gamma, beta, 1e-5)
    assert np.array_equal(nm.bn_apply(x, gamma, beta, mean, invstd), y)


# ------------------------------------------------------------------ ReLU and the sign mask
def test_mask_bit_order_hand_example():
    # N=1, C=2, H=1, W=40: 80 elements = 2 words.  Only (c=1, w=35) is positive:
    # N,H,W,C linear index e = 35*2 + 1 = 71 -> word 1, bit 7.
    x = -np.ones((1, 2, 1, 40))
    x[0, 1, 0, 35] = 0.5
    words = nm.pack_mask(nm.relu_pass(x))
    assert words.dtype == np.dtype("<u8") and words.tolist() == [0, 1 << 7]
    # element 0 -> word 0 bit 0; element 63 (w=31, c=1) -> word 0 bit 63
    x[:] = -1
    x[0, 0, 0, 0] = 1
    x[0, 1, 0, 31] = 1
    assert nm.pack_mask(nm.relu_pass(x)).tolist() == [(1 << 63) | 1, 0]


def test_mask_strict_predicate_and_roundtrip():
    x = RNG.standard_normal((2, 5, 7, 3))
    x[0, 0, 0, 0] = 0.0
    x[0, 0, 0, 1] = -0.0
    x[0, 0, 0, 2] = np.nan
    p = nm.relu_pass(x)
    assert not p[0, 0, 0, 0] and not p[0, 0, 0, 1] and not p[0, 0, 0, 2]
    words = nm.pack_mask(p)
    assert words.size == (x.size + 63) // 64
    assert sum(bin(int(w)).count("1") for w in words) == int((x > 0).sum())
    assert np.array_equal(nm.unpack_mask(words, x.shape), x > 0)
    dz = RNG.standard_normal(x.shape)
    xs = np.nan_to_num(x)
    assert np.array_equal(nm.relu_bwd_from_mask(dz, nm.pack_mask(nm.relu_pass(xs))), nm.relu_bwd_from_input(dz, xs))
    assert np.array_equal(nm.relu_bwd_from_output(dz, nm.relu_fwd(xs)), nm.relu_bwd_from_input(dz, xs))


def test_relu_forward_values_by_hand():
    """Forward values on hand-picked inputs: negative, both zeros and NaN give +0, positives pass unchanged;
    ReLU6 also passes 6 itself and holds everything above it at 6."""
    with np.errstate(invalid="ignore"):
        y = nm.relu_fwd(np.array([-1.0, 0.0, -0.0, 2.0, np.nan, 7.5, -np.inf, np.inf]))
        y6 = nm.relu6_fwd(np.array([-1.0, 0.0, -0.0, 3.0, 6.0, 7.0, np.nan, 5.999, np.inf]))
    assert y.tolist() == [0.0, 0.0, 0.0, 2.0, 0.0, 7.5, 0.0, np.inf]
    assert not np.signbit(y[:5]).any()
    assert y6.tolist() == [0.0, 0.0, 0.0, 3.0, 6.0, 6.0, 0.0, 5.999, 6.0]
    assert not np.signbit(y6).any()


def test_relu6_variants_agree():
    x = RNG.standard_normal((2, 3, 4, 5)) * 4
    dz = RNG.standard_normal(x.shape)
    a = nm.relu6_bwd_from_input(dz, x)
    assert np.array_equal(a, nm.relu6_bwd_from_output(dz, nm.relu6_fwd(x)))
    assert np.array_equal(a, nm.relu_bwd_from_mask(dz, nm.pack_mask(nm.relu6_pass(x))))
    assert np.array_equal(a, dz * ((x > 0) & (x < 6)))


# ------------------------------------------------------------------ pooling
def test_maxpool_hand_example_ties_and_padding():
    # 1x1x4x4, 3x3 window, stride 2, pad 1 -> 2x2 output.
    x = np.array([[1, 5, 5, 0],
                  [2, 5, 1, 0],
                  [0, 0, -1, -2],
                  [0, 0, -3, -4]], float)[None, None]
    y, idx = nm.maxpool_fwd(x, 3, 2, 1)
    # window (0,0) covers rows -1..1, cols -1..1: values {1,5;2,5}; first 5 is at (r=1,s=2) -> 1*3+2 = 5
    # window (0,1) covers rows -1..1, cols 1..3: {5,5,0;5,1,0}; first 5 at (r=1,s=0) -> 3
    # window (1,0) covers rows 1..3, cols -1..1: {2,5;0,0;0,0}; 5 at (r=0,s=2) -> 2
    # window (1,1) covers rows 1..3, cols 1..3: {5,1,0;0,-1,-2;0,-3,-4}; 5 at (r=0,s=0) -> 0
    assert y[0, 0].tolist() == [[5, 5], [5, 5]]
    assert idx[0, 0].tolist() == [[5, 3], [2, 0]]
    dy = np.array([[1.0, 10.0], [100.0, 1000.0]])[None, None]
    dx = nm.maxpool_bwd_from_index(dy, idx, x.shape, 3, 2, 1)
    want = np.zeros((4, 4))
    want[0, 1] = 1 + 10        # both top windows picked x[0,1]
    want[1, 1] = 100 + 1000
    assert dx[0, 0].tolist() == want.tolist()
    assert np.array_equal(nm.maxpool_bwd_from_input(dy, x, 3, 2, 1), dx)


def test_maxpool_bwd_by_finite_differences():
    x = RNG.standard_normal((2, 3, 7, 7))
    dy = RNG.standard_normal((2, 3, 4, 4))
    f = lambda: float((nm.maxpool_fwd(x, 3, 2, 1)[0] * dy).sum())
    _, idx = nm.maxpool_fwd(x, 3, 2, 1)
    assert rel(nm.maxpool_bwd_from_index(dy, idx, x.shape, 3, 2, 1), fd_grad(f, x)) < 1e-8


def test_avgpool_linear_losses():
    x = RNG.standard_normal((3, 4, 5, 6))
    assert np.allclose(nm.avgpool_fwd(x), x.reshape(3, 4, -1).mean(axis=2))
    dy = RNG.standard_normal((3, 4))
    f = lambda: float((nm.avgpool_fwd(x) * dy).sum())
    assert rel(nm.avgpool_bwd(dy, x.shape), fd_grad(f, x)) < 1e-8
    # linear
    a, w, b = RNG.standard_normal((3, 5)), RNG.standard_normal((4, 5)), RNG.standard_normal(4)
    dz = RNG.standard_normal((3, 4))
    f = lambda: float((nm.linear_fwd(a, w, b) * dz).sum())
    dw, db = nm.linear_wgrad(a, dz)
    assert rel(dw, fd_grad(f, w)) < 1e-8 and rel(db, fd_grad(f, b)) < 1e-8
    assert rel(nm.linear_dgrad(dz, w), fd_grad(f, a)) < 1e-8
    # cross-entropy: uniform logits give log(classes); gradient rows sum to zero; FD
    logits = np.zeros((4, 10))
    labels = np.array([0, 3, 9, 5])
    assert abs(nm.softmaxce_fwd(logits, labels) - np.log(10)) < 1e-14
    logits = RNG.standard_normal((4, 10)) * 3
    g = nm.softmaxce_bwd(logits, labels)
    assert np.abs(g.sum(axis=1)).max() < 1e-15
    f = lambda: nm.softmaxce_fwd(logits, labels)
    assert rel(g, fd_grad(f, logits)) < 1e-8


# ------------------------------------------------------------------ whole network
def _min_preact(ref, g):
    return min(np.abs(ref["acts"][n.ins[0]]).min() for n in g.nodes if n.op == "relu")


def test_tiny_chain_gradients_by_finite_differences():
    g = graphs.tiny_chain(batch=2, hw=6, channels=4, blocks=2)
    gt = g.text()
    exts, params = tensors.make_inputs(g, seed=4, gamma_beta="random")
    oe, op = tensors.oracle_inputs(exts, params)
    ref = onet.store_everything_step(gt, oe, op)
    assert _min_preact(ref, g) > 1e-4      # stay away from the ReLU kink
    f = lambda: onet.store_everything_step(gt, oe, op)["loss"]
    for pid in op:
        assert rel(ref["grads"][pid], fd_grad(f, op[pid])) < 2e-6, pid


def test_small_resnet_gradients_by_finite_differences():
    g = graphs.resnet50(batch=2, hw=64, classes=5, widths=(2, 2, 4, 4), depths=(1, 1, 1, 1), stem=2)
    gt = g.text()
    exts, params = tensors.make_inputs(g, seed=5, gamma_beta="random")
    oe, op = tensors.oracle_inputs(exts, params)
    ref = onet.store_everything_step(gt, oe, op)
    f = lambda: onet.store_everything_step(gt, oe, op)["loss"]
    rng = np.random.default_rng(0)
    # directional derivative over all parameters at once (cheap), plus a few single tensors
    direction = {p: rng.standard_normal(v.shape) for p, v in op.items()}
    h = 1e-7        # the direction is long (every parameter moves), so the step is short
    base = {p: v.copy() for p, v in op.items()}
    for p in op:
        op[p] = base[p] + h * direction[p]
    fp = f()
    for p in op:
        op[p] = base[p] - h * direction[p]
    fm = f()
    for p in op:
        op[p] = base[p]
    want = (fp - fm) / (2 * h)
    got = sum(float((ref["grads"][p] * direction[p]).sum()) for p in op)
    assert abs(got - want) < 1e-6 * max(1.0, abs(want))
    for pid in (1, 2, len(op) - 2, len(op) - 1):
        assert rel(ref["grads"][pid], fd_grad(f, op[pid])) < 1e-5, pid
