"""Pins for the oracle operators used by the VGG / UNet / MobileNetV2 configurations:
transposed convolution, depthwise convolution, channel concatenation, per-pixel cross-entropy,
linear layers over flattened images, masks of 2-D tensors.  Index definitions by loops on tiny
inputs, reductions to other routines (dense convolution with a block-diagonal filter, adjoint
identities), finite differences."""
import numpy as np
import pytest

from oracle import numerics as nm

RNG = np.random.default_rng(4321)


def fd_grad(f, x, h=1e-6):
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


# ------------------------------------------------------------------ transposed convolution
def tconv_loops(x, w, stride):
    N, C, H, W = x.shape
    _, K, R, S = w.shape
    y = np.zeros((N, K, (H - 1) * stride + R, (W - 1) * stride + S))
    for n in range(N):
        for c in range(C):
            for h in range(H):
                for v in range(W):
                    for k in range(K):
                        for r in range(R):
                            for s in range(S):
                                y[n, k, h * stride + r, v * stride + s] += x[n, c, h, v] * w[c, k, r, s]
    return y


@pytest.mark.parametrize("R,stride", [(2, 2), (3, 2), (2, 1)])
def test_tconv_fwd_matches_index_definition(R, stride):
    x = RNG.standard_normal((2, 3, 4, 5))
    w = RNG.standard_normal((3, 4, R, R))
    assert rel(nm.tconv2d_fwd(x, w, stride), tconv_loops(x, w, stride)) < 1e-14


def test_tconv_2x2_stride2_is_four_interleaved_matmuls():
    # non-overlapping case: output pixel (2h+r, 2v+s) is x[:, :, h, v] times the C x K slice w[:, :, r, s]
    x = RNG.standard_normal((2, 5, 3, 4))
    w = RNG.standard_normal((5, 6, 2, 2))
    y = nm.tconv2d_fwd(x, w, 2)
    assert y.shape == (2, 6, 6, 8)
    for r in range(2):
        for s in range(2):
            want = np.einsum("nchv,ck->nkhv", x, w[:, :, r, s])
            assert rel(y[:, :, r::2, s::2], want) < 1e-14


def test_tconv_is_the_adjoint_of_convolution():
    # <tconv(x, w), z> == <x, conv(z, w)> when w is read as a K=C_in, C=C_out convolution filter
    x = RNG.standard_normal((2, 3, 4, 5))
    w = RNG.standard_normal((3, 4, 2, 2))
    z = RNG.standard_normal((2, 4, 8, 10))
    lhs = np.sum(nm.tconv2d_fwd(x, w, 2) * z)
    rhs = np.sum(x * nm.conv2d_fwd(z, w, 2, 0))
    assert abs(lhs - rhs) < 1e-10 * abs(lhs)
    # the same statement for the gradient routines
    assert rel(nm.tconv2d_dgrad(z, w, 2), nm.conv2d_fwd(z, w, 2, 0)) < 1e-14
    assert rel(nm.tconv2d_fwd(x, w, 2), nm.conv2d_dgrad(x, w, z.shape, 2, 0)) < 1e-14


@pytest.mark.parametrize("R,stride", [(2, 2), (3, 2)])
def test_tconv_grads_by_finite_differences(R, stride):
    x = RNG.standard_normal((2, 3, 3, 4))
    w = RNG.standard_normal((3, 2, R, R))
    y0 = nm.tconv2d_fwd(x, w, stride)
    g = RNG.standard_normal(y0.shape)
    loss = lambda: float(np.sum(nm.tconv2d_fwd(x, w, stride) * g))
    assert rel(nm.tconv2d_dgrad(g, w, stride), fd_grad(loss, x)) < 1e-8
    assert rel(nm.tconv2d_wgrad(x, g, R, R, stride), fd_grad(loss, w)) < 1e-8


# ------------------------------------------------------------------ depthwise convolution
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_dwconv_is_dense_convolution_with_a_diagonal_filter(stride, pad):
    C = 5
    x = RNG.standard_normal((2, C, 7, 6))
    w = RNG.standard_normal((C, 1, 3, 3))
    dense = np.zeros((C, C, 3, 3))
    for c in range(C):
        dense[c, c] = w[c, 0]
    y = nm.dwconv2d_fwd(x, w, stride, pad)
    assert rel(y, nm.conv2d_fwd(x, dense, stride, pad)) < 1e-14
    g = RNG.standard_normal(y.shape)
    assert rel(nm.dwconv2d_dgrad(g, w, x.shape, stride, pad), nm.conv2d_dgrad(g, dense, x.shape, stride, pad)) < 1e-14
    full = nm.conv2d_wgrad(x, g, 3, 3, stride, pad)
    diag = np.stack([full[c, c] for c in range(C)])[:, None]
    assert rel(nm.dwconv2d_wgrad(x, g, 3, 3, stride, pad), diag) < 1e-14


def test_dwconv_hand_example():
    # one channel, 3x3 image, 3x3 filter of ones, pad 1: each output is the sum of the in-bounds neighbours
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    w = np.ones((1, 1, 3, 3))
    y = nm.dwconv2d_fwd(x, w, 1, 1)
    want = np.array([[12.0, 21.0, 16.0], [27.0, 45.0, 33.0], [24.0, 39.0, 28.0]])
    assert np.array_equal(y[0, 0], want)
    # stride 2 keeps the corners
    assert np.array_equal(nm.dwconv2d_fwd(x, w, 2, 1)[0, 0], want[::2, ::2])


@pytest.mark.parametrize("stride", [1, 2])
def test_dwconv_grads_by_finite_differences(stride):
    x = RNG.standard_normal((2, 3, 5, 6))
    w = RNG.standard_normal((3, 1, 3, 3))
    y0 = nm.dwconv2d_fwd(x, w, stride, 1)
    g = RNG.standard_normal(y0.shape)
    loss = lambda: float(np.sum(nm.dwconv2d_fwd(x, w, stride, 1) * g))
    assert rel(nm.dwconv2d_dgrad(g, w, x.shape, stride, 1), fd_grad(loss, x)) < 1e-8
    assert rel(nm.dwconv2d_wgrad(x, g, 3, 3, stride, 1), fd_grad(loss, w)) < 1e-8


# ------------------------------------------------------------------ concat, score maps, flattening linear
def test_concat_and_its_gradient():
    a = RNG.standard_normal((2, 3, 4, 5))
    b = RNG.standard_normal((2, 2, 4, 5))
    y = nm.concat_fwd(a, b)
    assert y.shape == (2, 5, 4, 5)
    assert np.array_equal(y[:, :3], a) and np.array_equal(y[:, 3:], b)
    g = RNG.standard_normal(y.shape)
    da, db = nm.concat_bwd(g, 3)
    # <concat(a,b), g> is linear: its gradient is the matching slice of g
    assert np.array_equal(da, g[:, :3]) and np.array_equal(db, g[:, 3:])
    assert abs(np.sum(y * g) - np.sum(a * da) - np.sum(b * db)) < 1e-12


def test_per_pixel_cross_entropy_equals_row_form():
    logits = RNG.standard_normal((2, 3, 4, 5))
    labels = RNG.integers(0, 3, size=(2, 4, 5))
    rows = np.transpose(logits, (0, 2, 3, 1)).reshape(-1, 3)
    assert abs(nm.softmaxce_fwd(logits, labels) - nm.softmaxce_fwd(rows, labels.reshape(-1))) < 1e-15
    # two classes: loss per pixel is log(1 + exp(-(margin))) -- the logistic loss
    two = RNG.standard_normal((1, 2, 2, 2))
    lab = RNG.integers(0, 2, size=(1, 2, 2))
    margin = np.where(lab == 1, two[:, 1] - two[:, 0], two[:, 0] - two[:, 1])
    assert abs(nm.softmaxce_fwd(two, lab) - np.mean(np.log1p(np.exp(-margin)))) < 1e-14
    loss = lambda: nm.softmaxce_fwd(logits, labels)
    assert rel(nm.softmaxce_bwd(logits, labels), fd_grad(loss, logits)) < 1e-8


def test_linear_over_flattened_image():
    x = RNG.standard_normal((3, 2, 2, 2))
    w = RNG.standard_normal((4, 2, 2, 2))
    b = RNG.standard_normal(4)
    y = nm.linear_fwd(x, w, b)
    want = np.array([[np.sum(x[n] * w[o]) + b[o] for o in range(4)] for n in range(3)])
    assert rel(y, want) < 1e-14
    g = RNG.standard_normal(y.shape)
    loss = lambda: float(np.sum(nm.linear_fwd(x, w, b) * g))
    dw, db = nm.linear_wgrad(x, g)
    assert dw.shape == w.shape
    assert rel(dw, fd_grad(loss, w)) < 1e-8 and rel(db, fd_grad(loss, b)) < 1e-8
    assert rel(nm.linear_dgrad(g, w, x.shape), fd_grad(loss, x)) < 1e-8
    # 2-D input keeps working
    x2 = RNG.standard_normal((3, 5))
    w2 = RNG.standard_normal((4, 5))
    assert rel(nm.linear_fwd(x2, w2, b), x2 @ w2.T + b) < 1e-15


SMALL_INCEPTIONS = (("a", 8, (8, 12), (4, 8), 4), "pool", ("b", 12, (8, 16), (4, 8), 8))


@pytest.mark.parametrize("net", ["vgg", "unet", "mbv2", "googlenet"])
def test_recomputing_schedules_reach_the_plain_gradients(net):
    """Section 3: a tensor that is not stored is recomputed, so the result does not change.  The fp64
    interpreter, which really deletes freed arrays, must give the store-everything gradients."""
    from oracle import network as onet, schedule as osch
    from workloads import graphs, schedules, tensors
    if net == "vgg":
        g = graphs.vgg16_bn(batch=2, hw=32, classes=10, widths=(8, 16, 16, 32, 32), fc=64)
    elif net == "unet":
        g = graphs.unet(batch=2, h=32, w=48, classes=2, base=8, depth=4)
    elif net == "googlenet":
        g = graphs.googlenet(batch=2, hw=32, classes=10, stem=(8, 8, 16), inceptions=SMALL_INCEPTIONS)
    else:
        g = graphs.mobilenet_v2(batch=2, hw=32, classes=10, stem=8, last=64,
                                stages=((1, 8, 1, 1), (6, 12, 2, 2), (6, 16, 2, 2), (6, 24, 1, 1)))
    exts, params = tensors.make_inputs(g, seed=1, gamma_beta="random")
    oe, op = tensors.oracle_inputs(exts, params)
    plain = onet.store_everything_step(g.text(), oe, op)
    top = max(np.linalg.norm(v) for v in plain["grads"].values())
    for sch in (schedules.store_everything_schedule(g), schedules.block_output_schedule(g)):
        got = osch.interpret(g.text(), sch.text(), oe, op)
        assert abs(got["loss"] - plain["loss"]) < 1e-12 * abs(plain["loss"])
        for p, want in plain["grads"].items():
            # measured against the largest gradient: some BatchNorm shift gradients vanish identically
            assert np.linalg.norm(got["grads"][p] - want) < 1e-12 * top, p
    assert got["recomputes"] > 0


def test_mask_of_a_matrix_is_packed_row_major():
    p = np.zeros((2, 70), bool)
    p[0, 0] = p[0, 65] = p[1, 3] = True       # element numbers 0, 65, 73
    words = nm.pack_mask(p)
    assert words.tolist() == [1, (1 << 1) | (1 << 9), 0]
    assert np.array_equal(nm.unpack_mask(words, p.shape), p)
