"""Per-kernel parity on a real MI355X: each gfx950 kernel, called through the C ABI, against the
fp64 oracle on identical seeded fp32 inputs.  Integer outputs (sign masks, pool indices) are
bit-exact; floating point is compared normwise per tensor (activations 1e-4, gradients 1e-3)."""
import numpy as np
import pytest

from oracle import numerics as nm
from workloads import tensors as wt
import paper_2010_14501_amd as M
from paper_2010_14501_amd import monet

pytestmark = pytest.mark.gpu

from parity_util import ACT_TOL, GRAD_TOL, rel, check_close


def torch_mod():
    import torch
    return torch


def dev(a):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


CONV_CASES = [
    # N, H, W, C, K, R, stride, pad
    (2, 16, 16, 16, 16, 3, 1, 1),       # the tiny chain's layer
    (3, 14, 14, 64, 128, 3, 1, 1),      # several tiles, ragged M (588 rows)
    (2, 15, 13, 32, 80, 3, 2, 1),       # stride 2, odd sizes, ragged K
    (2, 28, 28, 64, 256, 1, 1, 0),      # 1x1
    (2, 28, 28, 128, 64, 1, 2, 0),      # 1x1 stride 2 (downsample path)
    (2, 32, 32, 3, 64, 7, 2, 3),        # stem: C=3 takes the scalar-load path
    (1, 9, 9, 20, 24, 3, 1, 1),         # C % 16 != 0 and K % 16 != 0
    (5, 7, 7, 512, 512, 3, 1, 1),       # deep reduction (4608)
    (2, 14, 14, 160, 320, 3, 1, 1),     # an inception 3x3: channel counts that are multiples of 16 but not of 128
    (2, 28, 28, 24, 144, 1, 1, 0),      # 1x1 with 24 input channels: aligned forward loader, last reduction step half empty
    (2, 28, 28, 144, 24, 1, 1, 0),      # ... and 24 output channels: the same in the input gradient
    (3, 15, 13, 40, 36, 1, 2, 0),       # both at once, stride 2, ragged rows and columns
    (2, 9, 9, 4, 8, 1, 1, 0),           # a single, mostly empty step
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_trio_matches_oracle(case):
    torch = torch_mod()
    N, H, W, C, K, R, stride, pad = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    dy = rng.standard_normal((N, P, Q, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)
    dx, dwt, ddy = dev(x), dev(w), dev(dy)
    # forward
    y = torch.empty((N, P, Q, K), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, None, 0)
    want = wt.act_from_oracle(nm.conv2d_fwd(xo, wo, stride, pad))
    check_close(y.cpu().numpy(), want, ACT_TOL)
    need = max(monet.call("monet_conv_workspace_bytes", which, N, H, W, C, K, R, R, stride, pad, 5) for which in (0, 1))
    big = torch.empty(need // 4, dtype=torch.float32, device="cuda")     # split workspace
    for splits in (2, 5):
        y.fill_(float("nan"))
        monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad,
                   splits, big.data_ptr(), big.numel() * 4)
        check_close(y.cpu().numpy(), want, ACT_TOL, what=splits)
    # input gradient, plain and accumulating
    gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_dgrad", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, pad, 0, 1, None, 0)
    want = wt.act_from_oracle(nm.conv2d_dgrad(dyo, wo, xo.shape, stride, pad))
    check_close(gx.cpu().numpy(), want, GRAD_TOL)
    monet.call("monet_conv_dgrad", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, 1, None, 0)
    check_close(gx.cpu().numpy(), 2 * want, GRAD_TOL)
    for splits in (2, 5):
        gx.fill_(float("nan"))
        monet.call("monet_conv_dgrad", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, pad, 0,
                   splits, big.data_ptr(), big.numel() * 4)
        check_close(gx.cpu().numpy(), want, GRAD_TOL, what=splits)
        monet.call("monet_conv_dgrad", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1,
                   splits, big.data_ptr(), big.numel() * 4)
        check_close(gx.cpu().numpy(), 2 * want, GRAD_TOL, what=splits)
    # weight gradient: no workspace, and split with workspace
    want = wt.weight_from_oracle(nm.conv2d_wgrad(xo, dyo, R, R, stride, pad))
    for splits in (1, 3, 8):
        gw = torch.full((K, R, R, C), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(splits * K * R * R * C, dtype=torch.float32, device="cuda")
        monet.call("monet_conv_wgrad", None, dx.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, C, K, R, R, stride, pad,
                   splits, ws.data_ptr(), ws.numel() * 4)
        check_close(gw.cpu().numpy(), want, GRAD_TOL, what=splits)


def test_conv_ragged_last_round_is_split_and_counts_reset():
    """More than 256 tiles and not a multiple of it: with a workspace the tiles of the last round are cut and meet
    inside the kernel.  Several calls in a row (the arrival table has to be back at zero each time), forward and
    input gradient with accumulation, against the oracle and against the uncut kernel."""
    torch = torch_mod()
    N, H, W, C, K, R, stride, pad = 48, 28, 28, 128, 128, 1, 1, 0          # 37632 rows = 294 tiles of 128
    rng = np.random.default_rng(7)
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / C)))
    dy = rng.standard_normal((N, H, W, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)
    dx, dwt, ddy = dev(x), dev(w), dev(dy)
    need = [monet.call("monet_conv_workspace_bytes", which, N, H, W, C, K, R, R, stride, pad, 1) for which in (0, 1)]
    assert need[0] == need[1] == 2 * 38 * 128 * 128 * 4                      # 38 tiles beyond 256, two ranges of four steps
    ws = torch.full((need[0] // 4,), float("nan"), dtype=torch.float32, device="cuda")
    want_y = wt.act_from_oracle(nm.conv2d_fwd(xo, wo, stride, pad))
    want_dx = wt.act_from_oracle(nm.conv2d_dgrad(dyo, wo, xo.shape, stride, pad))
    y0 = torch.empty((N, H, W, K), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y0.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, None, 0)
    # a refused call (workspace announced smaller than two partial results) enqueues nothing and leaves the table alone;
    # an explicit reset of the table between good calls changes nothing either
    with pytest.raises(monet.MonetError):
        monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y0.data_ptr(), N, H, W, C, K, R, R, stride, pad, 2, ws.data_ptr(), 1024)
    for rep in range(3):
        if rep == 1:
            monet.call("monet_conv_reset_arrivals", None)
        y = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, ws.data_ptr(), need[0])
        check_close(y.cpu().numpy(), want_y, ACT_TOL, what=rep)
        assert torch.equal(y[:32], y0[:32])                                   # whole tiles: same kernel path, same bits
        assert rel(y.cpu().numpy(), y0.cpu().numpy()) < 1e-6
        gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_dgrad", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, pad, 0, 1, ws.data_ptr(), need[1])
        check_close(gx.cpu().numpy(), want_dx, GRAD_TOL, what=rep)
        monet.call("monet_conv_dgrad", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, 1, ws.data_ptr(), need[1])
        check_close(gx.cpu().numpy(), 2 * want_dx, GRAD_TOL, what=rep)


@pytest.mark.parametrize("case", [
    (3, 14, 14, 64, 128, 3, 1, 1),      # ragged last row group (588 rows)
    (2, 28, 28, 64, 256, 1, 1, 0),      # two column tiles
    (2, 15, 13, 32, 80, 3, 2, 1),       # stride 2, a column tile that is only partly used (80 of 128)
    (2, 28, 28, 128, 64, 1, 2, 0),      # the 256x64 tile: four row groups per workgroup
    (48, 28, 28, 128, 128, 1, 1, 0),    # ragged last round cut and met inside the kernel
    (2, 28, 28, 24, 144, 1, 1, 0),      # 1x1 with 24 input channels (last reduction step half empty)
    (3, 15, 13, 40, 36, 1, 2, 0),
])
def test_statistics_from_the_conv_epilogue_are_the_stand_alone_bits(case):
    """BatchNorm's forward statistics come out of the convolution's epilogue with the same bits as from a pass
    over the convolution's output, and match the oracle."""
    torch = torch_mod()
    N, H, W, C, K, R, stride, pad = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    w += np.float32(0.05)                                                # non-zero channel means
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    dx, dwt = dev(x), dev(w)
    rows = N * P * Q
    groups = (rows + 63) // 64
    sb = 8 * (groups + (groups + 63) // 64) * K                      # first and second level of the statistics
    scratch = torch.full((sb // 4,), float("nan"), dtype=torch.float32, device="cuda")
    need = monet.call("monet_conv_workspace_bytes", 0, N, H, W, C, K, R, R, stride, pad, 1)
    ws = torch.empty(max(need // 4, 1), dtype=torch.float32, device="cuda")
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    fused = torch.full((2 * K,), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_fwd_bn_stats", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad,
               ws.data_ptr() if need else None, need, fused.data_ptr(), 1e-5, scratch.data_ptr(), sb)
    y2 = torch.empty_like(y)
    monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y2.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1,
               ws.data_ptr() if need else None, need)
    assert torch.equal(y, y2)
    alone = torch.full((2 * K,), float("nan"), dtype=torch.float32, device="cuda")
    scratch.fill_(float("nan"))
    monet.call("monet_bn_stats", None, y2.data_ptr(), alone.data_ptr(), rows, K, 1e-5, scratch.data_ptr(), sb)
    assert torch.equal(fused, alone)
    mean, invstd = nm.bn_stats(wt.act_to_oracle(y2.cpu().numpy()), 1e-5)
    got = fused.cpu().numpy()
    check_close(got[:K], mean, ACT_TOL)
    check_close(got[K:], invstd, ACT_TOL)


@pytest.mark.parametrize("case", [
    (3, 14, 14, 64, 128, 3, 1, 1, 0),      # implicit GEMM, ragged rows
    (2, 28, 28, 64, 256, 1, 1, 0, 0),      # two column tiles
    (2, 15, 13, 32, 80, 3, 2, 1, 0),       # stride 2, a column tile that is only partly used
    (2, 28, 28, 128, 64, 1, 2, 0, 0),      # the 256x64 tile
    (48, 28, 28, 128, 128, 1, 1, 0, 0),    # ragged last round cut and met inside the kernel
    (2, 28, 28, 24, 128, 1, 1, 0, 0),      # 1x1 with 24 input channels (last reduction step half empty)
    (3, 14, 14, 64, 128, 3, 1, 1, 2),      # Winograd, 2x2 output tiles
    (3, 14, 14, 64, 128, 3, 1, 1, 4),      # Winograd, 4x4 output tiles (last tile row / column partly outside)
    (2, 9, 7, 32, 48, 3, 1, 1, 4),
])
def test_batchnorm_apply_in_the_conv_epilogue_is_the_stand_alone_bits(case):
    """A recomputed convolution that applies the BatchNorm behind it in its epilogue writes exactly what the
    convolution followed by the in-place apply kernel writes (implicit GEMM and both Winograd forms)."""
    torch = torch_mod()
    N, H, W, C, K, R, stride, pad, m = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    gamma = rng.uniform(0.5, 1.5, K).astype(np.float32)
    beta = rng.standard_normal(K, dtype=np.float32)
    stats = np.concatenate([rng.standard_normal(K, dtype=np.float32) * np.float32(0.3), rng.uniform(0.5, 2.0, K).astype(np.float32)])
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    dx, dwt, dg_, db_, dst = dev(x), dev(w), dev(gamma), dev(beta), dev(stats)
    if m:
        need = monet.call("monet_conv_winograd_workspace_bytes", N, H, W, C, K, m)
    else:
        need = monet.call("monet_conv_workspace_bytes", 0, N, H, W, C, K, R, R, stride, pad, 1)
    ws = torch.empty(max(need // 4, 1), dtype=torch.float32, device="cuda")
    wsp = ws.data_ptr() if need else None
    fused = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_fwd_bn_apply", None, dx.data_ptr(), dwt.data_ptr(), fused.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
               wsp, need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr())
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    if m:
        monet.call("monet_conv_winograd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, m, 0, 0, wsp, need)
    else:
        monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, wsp, need)
    monet.call("monet_bn_apply", None, y.data_ptr(), y.data_ptr(), dg_.data_ptr(), db_.data_ptr(), dst.data_ptr(), N * P * Q, K)
    assert torch.equal(fused, y)
    yo = nm.conv2d_fwd(wt.act_to_oracle(x), wt.weight_to_oracle(w), stride, pad)
    want = nm.bn_apply(yo, gamma.astype(np.float64), beta.astype(np.float64), stats[:K].astype(np.float64), stats[K:].astype(np.float64))
    check_close(fused.cpu().numpy(), wt.act_from_oracle(want), ACT_TOL)
    # ... and with the ReLU / ReLU6 behind the BatchNorm in the same epilogue: the bits of the stand-alone ReLU kernel run in
    # place on the tensor above (values scaled so that the upper clamp of ReLU6 is reached)
    for six in (0, 1):
        g6 = dev(gamma * np.float32(4.0 if six else 1.0))
        plain = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_fwd_bn_apply", None, dx.data_ptr(), dwt.data_ptr(), plain.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
                   wsp, need, g6.data_ptr(), db_.data_ptr(), dst.data_ptr())
        monet.call("monet_relu_fwd", None, plain.data_ptr(), plain.data_ptr(), None, N * P * Q * K, six)
        both = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), both.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
                   wsp, need, g6.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, None, None)
        assert torch.equal(both, plain), six
        assert float(both.min()) == 0.0 and (not six or float(both.max()) == 6.0)
        # the ReLU's result beside the BatchNorm's (the BatchNorm output is kept for its own backward operator)
        bn_out = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
        relu_out = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), bn_out.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
                   wsp, need, g6.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, relu_out.data_ptr(), None)
        want_bn = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_fwd_bn_apply", None, dx.data_ptr(), dwt.data_ptr(), want_bn.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
                   wsp, need, g6.data_ptr(), db_.data_ptr(), dst.data_ptr())
        assert torch.equal(bn_out, want_bn) and torch.equal(relu_out, plain), six
        # ... and the ReLU's sign code from the same epilogue: the words of the stand-alone kernel (64 | K; the Winograd
        # forms with transformed tensors in memory refuse it)
        words = (N * P * Q * K + 63) // 64
        mask = torch.full((words,), -1, dtype=torch.int64, device="cuda")
        if K % 64 == 0 and m == 0:
            for out2 in (None, relu_out):
                mask.fill_(-1)
                if out2 is not None:
                    out2.fill_(float("nan"))
                bn_out.fill_(float("nan"))
                monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), bn_out.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
                           wsp, need, g6.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, out2.data_ptr() if out2 is not None else None,
                           mask.data_ptr())
                want_mask = torch.full((words,), -1, dtype=torch.int64, device="cuda")
                scratch = torch.empty_like(want_bn)
                monet.call("monet_relu_fwd", None, want_bn.data_ptr(), scratch.data_ptr(), want_mask.data_ptr(), N * P * Q * K, six)
                assert torch.equal(mask, want_mask), (six, out2 is None)
                assert torch.equal(bn_out if out2 is None else out2, plain), six
                if out2 is not None:
                    assert torch.equal(bn_out, want_bn)
        else:
            with pytest.raises(monet.MonetError):
                monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), bn_out.data_ptr(), N, H, W, C, K, R, R, stride, pad, m,
                           wsp, need, g6.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, relu_out.data_ptr(), mask.data_ptr())
    with pytest.raises(monet.MonetError):       # no Winograd form with 3x3 output tiles
        monet.call("monet_conv_fwd_bn_apply", None, dx.data_ptr(), dwt.data_ptr(), fused.data_ptr(), N, H, W, C, K, R, R, stride, pad, 3,
                   wsp, need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr())


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("case", [
    (2, 14, 14, 64, 128),       # even map (for 4x4 tiles: the last tile row / column is half outside)
    (3, 7, 9, 32, 48),          # odd sizes: the last tile row / column is partly outside the map
    (1, 5, 5, 16, 16),          # smallest aligned channel counts
    (5, 7, 7, 512, 512),        # deep reduction
    (2, 56, 56, 64, 64),        # many tiles (1568 resp. 392 per GEMM)
    (1, 3, 2, 16, 16),          # a map smaller than one 4x4 tile
])
def test_winograd_convolution_matches_oracle(case, m):
    """F(2x2, 3x3) and F(4x4, 3x3): forward, input gradient (written and accumulated) and filter gradient against the
    oracle's direct definitions."""
    torch = torch_mod()
    N, H, W, C, K = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, 3, 3, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (9 * C))))
    dy = rng.standard_normal((N, H, W, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)
    dx, dwt, ddy = dev(x), dev(w), dev(dy)
    need = monet.call("monet_conv_winograd_workspace_bytes", N, H, W, C, K, m)
    tiles = N * ((H + m - 1) // m) * ((W + m - 1) // m)
    assert need == (m + 2) ** 2 * 4 * (K * C + tiles * (C + K))
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
    y = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_winograd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, m, 0, 0, ws.data_ptr(), need)
    check_close(y.cpu().numpy(), wt.act_from_oracle(nm.conv2d_fwd(xo, wo, 1, 1)), ACT_TOL)
    gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
    want = wt.act_from_oracle(nm.conv2d_dgrad(dyo, wo, xo.shape, 1, 1))
    monet.call("monet_conv_winograd", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, m, 1, 0, ws.data_ptr(), need)
    check_close(gx.cpu().numpy(), want, GRAD_TOL)
    monet.call("monet_conv_winograd", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, m, 1, 1, ws.data_ptr(), need)
    check_close(gx.cpu().numpy(), 2 * want, GRAD_TOL)
    with pytest.raises(monet.MonetError):
        monet.call("monet_conv_winograd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, 3, 0, 0, ws.data_ptr(), need)
    # a workspace that holds one image at a time: the layer goes through in N chunks, with the same bits
    per_img = (m + 2) ** 2 * 4 * ((H + m - 1) // m) * ((W + m - 1) // m) * (C + K)
    small = (m + 2) ** 2 * 4 * K * C + per_img + 64
    if N > 1:
        y2 = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_conv_winograd", None, dx.data_ptr(), dwt.data_ptr(), y2.data_ptr(), N, H, W, C, K, m, 0, 0, ws.data_ptr(), small)
        assert torch.equal(y, y2)
        if N > 2:      # two images at a time: the last chunk is shorter
            y2.fill_(float("nan"))
            monet.call("monet_conv_winograd", None, dx.data_ptr(), dwt.data_ptr(), y2.data_ptr(), N, H, W, C, K, m, 0, 0, ws.data_ptr(), small + per_img)
            assert torch.equal(y, y2)
    with pytest.raises(monet.MonetError):
        monet.call("monet_conv_winograd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, m, 0, 0, ws.data_ptr(), small - per_img)
    # filter gradient in the transformed domain
    need = monet.call("monet_conv_winograd_wgrad_workspace_bytes", N, H, W, C, K, m)
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
    gw = torch.full((K, 3, 3, C), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_winograd_wgrad", None, dx.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, C, K, m, ws.data_ptr(), need)
    want_w = wt.weight_from_oracle(nm.conv2d_wgrad(xo, dyo, 3, 3, 1, 1))
    check_close(gw.cpu().numpy(), want_w, GRAD_TOL)
    if N > 1:       # in chunks of one image: the chunks' shares are added in image order
        planes, tiles_img = (m + 2) ** 2, ((H + m - 1) // m) * ((W + m - 1) // m)
        ranges = max(1, min(1024 // (planes * ((K + 127) // 128) * ((C + 127) // 128)), tiles_img // 128))
        small = per_img + planes * 4 * K * C * (2 + (ranges if ranges > 1 else 0))
        ws.fill_(float("nan"))
        gw.fill_(float("nan"))
        monet.call("monet_conv_winograd_wgrad", None, dx.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, C, K, m, ws.data_ptr(), min(small, need))
        check_close(gw.cpu().numpy(), want_w, GRAD_TOL)


@pytest.mark.parametrize("case", [
    (2, 14, 14, 64, 128),       # two blocks of 64 output channels; the last tile row / column is half outside the map
    (3, 7, 9, 32, 48),          # odd sizes, output channels no multiple of 32, fewer tiles than a workgroup takes
    (1, 5, 5, 8, 4),            # smallest channel counts
    (2, 7, 7, 512, 512),        # deep reduction (64 chunks), eight channel blocks
    (3, 56, 56, 64, 64),        # many tiles: 588 per channel block, ragged last workgroup (588 = 18 * 32 + 12)
    (1, 3, 2, 16, 16),          # a map smaller than one 4x4 tile
    (2, 12, 20, 24, 40),        # reduction channels a multiple of 8 only, 40 output channels (second half mostly padding)
    # more work items than CUs with a short remainder, which is worked as half items of 32 output channels:
    (3, 224, 224, 8, 72),       # forward 588 items (512 + 76 halved, every second one with 8 channels in its first half and none
                                # in its second), input gradient 294 (256 + 38 halved, 8 output channels)
    (3, 120, 124, 8, 160),      # 264 items (256 + 8 halved) of three channel blocks, the third half empty; ragged last tile block
])
def test_fused_winograd_convolution_matches_oracle(case):
    """F(4x4, 3x3) in one kernel (no transformed tensors in memory): forward, input gradient written and accumulated,
    and the forward form with a BatchNorm apply step, against the oracle's direct definitions."""
    torch = torch_mod()
    N, H, W, C, K = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, 3, 3, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (9 * C))))
    dy = rng.standard_normal((N, H, W, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)
    dx, dwt, ddy = dev(x), dev(w), dev(dy)
    need = monet.call("monet_conv_winograd_fused_workspace_bytes", N, H, W, C, K, 0)
    assert need == 36 * 4 * ((K + 63) // 64 * 64) * C
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
    y = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_winograd_fused", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, 0, 0, ws.data_ptr(), need)
    want_y = nm.conv2d_fwd(xo, wo, 1, 1)
    check_close(y.cpu().numpy(), wt.act_from_oracle(want_y), ACT_TOL)
    with pytest.raises(monet.MonetError):
        monet.call("monet_conv_winograd_fused", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, 0, 0, ws.data_ptr(), need - 4)
    # BatchNorm apply step in the epilogue: the bits of the stand-alone apply kernel on the stored output
    gamma = rng.uniform(0.5, 1.5, K).astype(np.float32)
    beta = (0.1 * rng.standard_normal(K)).astype(np.float32)
    stats = np.concatenate([0.1 * rng.standard_normal(K), rng.uniform(0.5, 2.0, K)]).astype(np.float32)
    dg_, db_, dst = dev(gamma), dev(beta), dev(stats)
    fused = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_fwd_bn_apply", None, dx.data_ptr(), dwt.data_ptr(), fused.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 5,
               ws.data_ptr(), need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr())
    if K % 4 == 0:
        monet.call("monet_bn_apply", None, y.data_ptr(), y.data_ptr(), dg_.data_ptr(), db_.data_ptr(), dst.data_ptr(), N * H * W, K)
        assert torch.equal(fused, y)
        for six in (0, 1):      # the ReLU behind the BatchNorm in the same epilogue
            both = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
            monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), both.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 5,
                       ws.data_ptr(), need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, None, None)
            plain = y.clone()
            monet.call("monet_relu_fwd", None, plain.data_ptr(), plain.data_ptr(), None, N * H * W * K, six)
            assert torch.equal(both, plain), six
            bn_out = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
            relu_out = torch.full((N, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
            monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), bn_out.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 5,
                       ws.data_ptr(), need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, relu_out.data_ptr(), None)
            assert torch.equal(bn_out, y) and torch.equal(relu_out, plain), six
            words = (N * H * W * K + 63) // 64
            mask = torch.full((words,), -1, dtype=torch.int64, device="cuda")
            if K % 64 == 0:      # the ReLU's sign code from the same epilogue: the words of the stand-alone kernel
                bn_out.fill_(float("nan"))
                relu_out.fill_(float("nan"))
                monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), bn_out.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 5,
                           ws.data_ptr(), need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, relu_out.data_ptr(), mask.data_ptr())
                want_mask = torch.full((words,), -1, dtype=torch.int64, device="cuda")
                scratch = torch.empty_like(y)
                monet.call("monet_relu_fwd", None, y.data_ptr(), scratch.data_ptr(), want_mask.data_ptr(), N * H * W * K, six)
                assert torch.equal(mask, want_mask), six
                assert torch.equal(bn_out, y) and torch.equal(relu_out, plain), six
            else:
                with pytest.raises(monet.MonetError):
                    monet.call("monet_conv_fwd_bn_relu", None, dx.data_ptr(), dwt.data_ptr(), bn_out.data_ptr(), N, H, W, C, K, 3, 3, 1, 1, 5,
                               ws.data_ptr(), need, dg_.data_ptr(), db_.data_ptr(), dst.data_ptr(), six, relu_out.data_ptr(), mask.data_ptr())
    want = nm.bn_apply(want_y, gamma.astype(np.float64), beta.astype(np.float64), stats[:K].astype(np.float64), stats[K:].astype(np.float64))
    check_close(fused.cpu().numpy(), wt.act_from_oracle(want), ACT_TOL)
    # input gradient: reduction over K, which must be a multiple of 8
    if K % 8 == 0:
        need = monet.call("monet_conv_winograd_fused_workspace_bytes", N, H, W, C, K, 1)
        assert need == 36 * 4 * ((C + 63) // 64 * 64) * K
        ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
        gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
        want = wt.act_from_oracle(nm.conv2d_dgrad(dyo, wo, xo.shape, 1, 1))
        monet.call("monet_conv_winograd_fused", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, 1, 0, ws.data_ptr(), need)
        check_close(gx.cpu().numpy(), want, GRAD_TOL)
        monet.call("monet_conv_winograd_fused", None, ddy.data_ptr(), dwt.data_ptr(), gx.data_ptr(), N, H, W, C, K, 1, 1, ws.data_ptr(), need)
        check_close(gx.cpu().numpy(), 2 * want, GRAD_TOL)
    else:
        with pytest.raises(monet.MonetError):
            monet.call("monet_conv_winograd_fused", None, ddy.data_ptr(), dwt.data_ptr(), dx.data_ptr(), N, H, W, C, K, 1, 0, ws.data_ptr(), need)


IM2COL_CASES = [
    # N, H, W, C, K, R, stride, pad, chunk images (0: the recommended workspace)
    (2, 16, 16, 16, 16, 3, 1, 1, 0),
    (5, 14, 14, 64, 128, 3, 1, 1, 2),      # three chunks, the last one ragged
    (3, 15, 13, 32, 80, 3, 2, 1, 1),       # stride 2, odd sizes, one image per chunk
    (2, 32, 32, 3, 64, 7, 2, 3, 0),        # stem: 147 floats per patch, padded to 160 (filters padded too)
    (2, 9, 9, 20, 24, 3, 1, 1, 0),         # R*S*C = 180, padded to 192
    (4, 7, 7, 512, 512, 3, 1, 1, 3),
]


@pytest.mark.parametrize("case", IM2COL_CASES)
def test_convolution_through_patch_matrix_matches_oracle(case):
    """Forward (plain and accumulating) and filter gradient of the explicit patch-matrix form against the oracle, with
    the recommended workspace and with workspaces that force several chunks; a workspace below one image is refused."""
    torch = torch_mod()
    N, H, W, C, K, R, stride, pad, chunk = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    dy = rng.standard_normal((N, P, Q, K), dtype=np.float32)
    y0 = rng.standard_normal((N, P, Q, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)
    want_y = wt.act_from_oracle(nm.conv2d_fwd(xo, wo, stride, pad))
    want_w = wt.weight_from_oracle(nm.conv2d_wgrad(xo, dyo, R, R, stride, pad))
    dx, dwt, ddy = dev(x), dev(w), dev(dy)
    ld = -(-(C * R * R) // 16) * 16
    sizes = {}
    for wgrad in (0, 1):
        rec = monet.call("monet_conv_im2col_workspace_bytes", N, H, W, C, K, R, R, stride, pad, wgrad)
        if chunk:       # exactly `chunk` images of patches (+ padded filters / the gradient's tail, taken from the recommendation)
            rec_imgs_bytes = rec - 4 * min(N, max(1, (256 << 20) // 4 // (P * Q * ld))) * P * Q * ld
            rec = 4 * chunk * P * Q * ld + max(rec_imgs_bytes, 0) + (4 * K * ld * 260 if wgrad else 0)
        sizes[wgrad] = rec
    ws = torch.full((max(sizes.values()) // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
    y = torch.empty((N, P, Q, K), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_im2col_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad, 0, ws.data_ptr(), sizes[0])
    check_close(y.cpu().numpy(), want_y, ACT_TOL, what="forward")
    yacc = dev(y0)
    monet.call("monet_conv_im2col_fwd", None, dx.data_ptr(), dwt.data_ptr(), yacc.data_ptr(), N, H, W, C, K, R, R, stride, pad, 1, ws.data_ptr(), sizes[0])
    check_close(yacc.cpu().numpy(), want_y + y0, ACT_TOL, what="forward, accumulating")
    ws.fill_(float("nan"))
    dw = torch.full((K, R, R, C), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_im2col_wgrad", None, dx.data_ptr(), ddy.data_ptr(), dw.data_ptr(), N, H, W, C, K, R, R, stride, pad, ws.data_ptr(), sizes[1])
    check_close(dw.cpu().numpy(), want_w, GRAD_TOL, what="filter gradient")
    with pytest.raises(M.MonetError):
        monet.call("monet_conv_im2col_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride, pad, 0, ws.data_ptr(),
                   4 * (P * Q * ld - 16))


MANY_RANGE_CASES = [
    # N, H, W, C, K, R, stride, pad, splits: reduction ranges of a few steps each, several workgroups per compute unit
    (16, 112, 112, 16, 96, 1, 1, 0, 1792),      # MobileNetV2's first expansion (reduced batch): 7 steps per range
    (16, 112, 112, 16, 96, 1, 1, 0, 3136),      # 4 steps per range: one turn of the pipelined loop
    (16, 56, 56, 64, 64, 3, 1, 1, 640),         # padded 3x3: rows of a step straddle image borders
    (64, 14, 14, 256, 256, 3, 1, 1, 96),
    (16, 57, 57, 32, 48, 3, 2, 1, 640),         # stride 2, odd size
]


@pytest.mark.parametrize("case", MANY_RANGE_CASES)
def test_filter_gradient_with_many_short_ranges_on_every_tile_shape(case):
    """The aligned filter-gradient loader shares a per-step table of output positions through LDS; this runs it
    with thousands of short reduction ranges (several workgroups resident per compute unit, the loop entered and
    left after one or two turns) on each of the six tile shapes, against the oracle, twice: the two runs must agree
    bit for bit."""
    torch = torch_mod()
    N, H, W, C, K, R, stride, pad, splits = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    dy = rng.standard_normal((N, P, Q, K), dtype=np.float32)
    want = wt.weight_from_oracle(nm.conv2d_wgrad(wt.act_to_oracle(x), wt.act_to_oracle(dy), R, R, stride, pad))
    dx, ddy = dev(x), dev(dy)
    ws = torch.empty(splits * K * R * R * C, dtype=torch.float32, device="cuda")
    try:
        for cfg in range(6):
            monet.call("monet_conv_force_tile", cfg)
            got = []
            for rep in range(2):
                dw = torch.full((K, R, R, C), float("nan"), dtype=torch.float32, device="cuda")
                ws.fill_(float("nan"))
                monet.call("monet_conv_wgrad", None, dx.data_ptr(), ddy.data_ptr(), dw.data_ptr(), N, H, W, C, K, R, R, stride, pad, splits,
                           ws.data_ptr(), ws.numel() * 4)
                torch.cuda.synchronize()
                got.append(dw.cpu().numpy())
            assert np.array_equal(got[0], got[1]), (cfg, "two runs differ")
            check_close(got[0], want, 1e-5, what=f"tile shape {cfg}")
    finally:
        monet.call("monet_conv_force_tile", -1)


STEM_CASES = [
    # N, H, W, K, R, stride, pad, splits: the first layers of the five networks at reduced batch, sizes that leave ragged
    # tiles (odd maps, a last row tile with fewer rows, rows no multiple of four floats), rows wider than one tile
    (2, 224, 224, 64, 7, 2, 3, 64),       # ResNet-50 / inception: two output rows per tile
    (2, 224, 224, 32, 3, 2, 1, 64),       # MobileNetV2: one wave per position group
    (2, 224, 224, 64, 3, 1, 1, 64),       # VGG-16: one output row per tile
    (3, 37, 29, 64, 7, 2, 3, 16),
    (3, 37, 29, 32, 3, 2, 1, 7),
    (2, 33, 31, 96, 3, 1, 1, 5),
    (1, 40, 608, 64, 3, 1, 1, 9),         # UNet: rows of 608 positions in segments of 224
    (1, 19, 300, 128, 3, 1, 1, 4),
    (5, 9, 9, 32, 3, 1, 1, 2),
    (1, 7, 5, 64, 7, 2, 3, 2),            # a map smaller than the filter's reach
]


@pytest.mark.parametrize("case", STEM_CASES)
def test_first_layer_forward_and_filter_gradient_from_rows_staged_in_lds(case):
    """Convolutions of a three-channel image through the kernels that stage input rows in LDS: forward pass and filter
    gradient against the oracle, the filter gradient twice (bit-identical), and monet_conv_fwd / monet_conv_wgrad with
    the same arguments give the same bits, i.e. take these forms by themselves."""
    torch = torch_mod()
    N, H, W, K, R, stride, pad, splits = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, 3), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, 3), dtype=np.float32) * np.float32(np.sqrt(2.0 / (3 * R * R))))
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - R) // stride + 1
    dy = rng.standard_normal((N, P, Q, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)
    dx, dwt, ddy = dev(x), dev(w), dev(dy)
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_stem_fwd", None, dx.data_ptr(), dwt.data_ptr(), y.data_ptr(), N, H, W, K, R, R, stride, pad)
    check_close(y.cpu().numpy(), wt.act_from_oracle(nm.conv2d_fwd(xo, wo, stride, pad)), ACT_TOL, what="forward")
    y2 = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_conv_fwd", None, dx.data_ptr(), dwt.data_ptr(), y2.data_ptr(), N, H, W, 3, K, R, R, stride, pad, 1, None, 0)
    assert torch.equal(y, y2), "monet_conv_fwd did not take the first-layer form"
    ws = torch.empty(splits * K * R * R * 3, dtype=torch.float32, device="cuda")
    got = []
    for entry in ("monet_conv_stem_wgrad", "monet_conv_stem_wgrad", "monet_conv_wgrad"):
        gw = torch.full((K, R, R, 3), float("nan"), dtype=torch.float32, device="cuda")
        ws.fill_(float("nan"))
        if entry == "monet_conv_wgrad":
            monet.call(entry, None, dx.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, 3, K, R, R, stride, pad, splits, ws.data_ptr(), ws.numel() * 4)
        else:
            monet.call(entry, None, dx.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, K, R, R, stride, pad, splits, ws.data_ptr(), ws.numel() * 4)
        torch.cuda.synchronize()
        got.append(gw.cpu().numpy())
    assert np.array_equal(got[0], got[1]), "two runs differ"
    assert np.array_equal(got[0], got[2]), "monet_conv_wgrad did not take the first-layer form"
    check_close(got[0], wt.weight_from_oracle(nm.conv2d_wgrad(xo, dyo, R, R, stride, pad)), GRAD_TOL, what="filter gradient")


def test_first_layer_kernels_refuse_what_they_are_not_for():
    torch = torch_mod()
    t = torch.zeros(1 << 20, device="cuda")
    for (N, H, W, K, R, stride, pad) in [
        (1, 32, 32, 48, 3, 1, 1),      # output channels no multiple of 32
        (1, 32, 32, 64, 5, 1, 2),      # 5x5 filter
        (1, 32, 32, 64, 7, 1, 3),      # 7x7 at stride 1
        (1, 32, 32, 160, 3, 1, 1),     # more than four blocks of 32 output channels
    ]:
        with pytest.raises(M.MonetError):
            monet.call("monet_conv_stem_fwd", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), N, H, W, K, R, R, stride, pad)
    with pytest.raises(M.MonetError):      # no partial results asked for
        monet.call("monet_conv_stem_wgrad", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 1, 32, 32, 64, 3, 3, 1, 1, 1, t.data_ptr(), 1 << 22)
    with pytest.raises(M.MonetError):      # workspace one float short (five tiles of seven output rows: five workgroups)
        monet.call("monet_conv_stem_wgrad", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 1, 32, 32, 64, 3, 3, 1, 1, 8, t.data_ptr(),
                   5 * 64 * 27 * 4 - 4)


POINTWISE_WGRAD_CASES = [
    # N, H, W, C, K, splits: the channel pairs of MobileNetV2's expansion / projection layers (each selects another
    # combination of 16-byte and 4-byte loads of the wide side), position counts that leave a ragged tail, workgroups
    # whose share is shorter than one group of 16 positions per wave
    (2, 56, 56, 16, 96, 64),
    (3, 37, 29, 16, 96, 48),
    (2, 56, 56, 96, 24, 64),
    (2, 56, 56, 24, 144, 64),
    (2, 56, 56, 144, 32, 64),
    (2, 56, 56, 32, 192, 64),
    (2, 56, 56, 192, 32, 64),
    (2, 56, 56, 32, 16, 64),
    (1, 33, 31, 24, 144, 8),
    (1, 33, 31, 144, 24, 8),
    (5, 9, 9, 8, 40, 2),
    (4, 75, 75, 16, 96, 300),     # more splits than workgroups: 256 partial results are used
    (1, 17, 16, 12, 4, 4),        # 68 positions per workgroup: one group each for waves 0..3 and a tail of four rows
]


@pytest.mark.parametrize("case", POINTWISE_WGRAD_CASES)
def test_pointwise_filter_gradient_streamed_into_the_matrix_instruction(case):
    """The 1x1 filter gradient with few channels on one side, read straight from memory into the lane layout of the
    matrix instruction: against the oracle, twice (bit-identical), and monet_conv_wgrad with the same arguments must
    give the same bits, i.e. take this form by itself."""
    torch = torch_mod()
    N, H, W, C, K, splits = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    dy = rng.standard_normal((N, H, W, K), dtype=np.float32)
    want = wt.weight_from_oracle(nm.conv2d_wgrad(wt.act_to_oracle(x), wt.act_to_oracle(dy), 1, 1, 1, 0))
    dx, ddy = dev(x), dev(dy)
    ws = torch.empty(min(splits, 256) * K * C, dtype=torch.float32, device="cuda")
    got = []
    for entry in ("monet_conv_pointwise_wgrad", "monet_conv_pointwise_wgrad", "monet_conv_wgrad"):
        dw = torch.full((K, 1, 1, C), float("nan"), dtype=torch.float32, device="cuda")
        ws.fill_(float("nan"))
        if entry == "monet_conv_wgrad":
            monet.call(entry, None, dx.data_ptr(), ddy.data_ptr(), dw.data_ptr(), N, H, W, C, K, 1, 1, 1, 0, splits, ws.data_ptr(), ws.numel() * 4)
        else:
            monet.call(entry, None, dx.data_ptr(), ddy.data_ptr(), dw.data_ptr(), N, H, W, C, K, splits, ws.data_ptr(), ws.numel() * 4)
        torch.cuda.synchronize()
        got.append(dw.cpu().numpy())
    assert np.array_equal(got[0], got[1]), "two runs differ"
    assert np.array_equal(got[0], got[2]), "monet_conv_wgrad did not take the pointwise form"
    check_close(got[0], want, 1e-5, what="pointwise filter gradient")


def test_pointwise_filter_gradient_refuses_what_it_is_not_for():
    torch = torch_mod()
    t = torch.zeros(1 << 20, device="cuda")
    for (N, H, W, C, K, splits, ws_bytes) in [
        (2, 56, 56, 64, 64, 16, 1 << 22),      # both sides wider than 32 channels
        (2, 56, 56, 16, 256, 16, 1 << 22),     # wide side beyond 192
        (2, 56, 56, 16, 96, 1, 1 << 22),       # no partial results asked for
        (2, 56, 56, 16, 96, 16, 16 * 96 * 16 * 4 - 4),     # workspace one float short
        (1, 8, 8, 16, 96, 16, 1 << 22),        # fewer than 64 positions per workgroup
        (2, 56, 56, 18, 96, 16, 1 << 22),      # channels not a multiple of four
    ]:
        with pytest.raises(M.MonetError):
            monet.call("monet_conv_pointwise_wgrad", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), N, H, W, C, K, splits, t.data_ptr(), ws_bytes)


def test_conv_wgrad_rejects_small_workspace():
    torch = torch_mod()
    t = torch.zeros(16 * 16 * 16 * 2, device="cuda")
    with pytest.raises(M.MonetError):
        monet.call("monet_conv_wgrad", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 2, 16, 16, 16, 16, 3, 3, 1, 1, 4, t.data_ptr(), 64)
    with pytest.raises(M.MonetError):
        monet.call("monet_conv_fwd", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 2, 16, 16, 16, 16, 3, 3, 0, 1, 1, None, 0)
    with pytest.raises(M.MonetError):
        monet.call("monet_conv_fwd", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 2, 16, 16, 16, 16, 3, 3, 1, 1, 4, t.data_ptr(), 64)


BN_CASES = [(2 * 16 * 16, 16), (3 * 14 * 14, 64), (1000, 256), (77, 2048), (5 * 33 * 31, 128), (4096, 24), (2 * 14 * 14, 320)]


@pytest.mark.parametrize("rows,C", BN_CASES)
def test_batchnorm_matches_oracle(rows, C):
    torch = torch_mod()
    rng = np.random.default_rng(rows * 131 + C)
    x = (rng.standard_normal((rows, C)) * rng.uniform(0.5, 3, C) + rng.standard_normal(C) * 2).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    beta = (0.1 * rng.standard_normal(C)).astype(np.float32)
    dy = rng.standard_normal((rows, C), dtype=np.float32)
    eps = 1e-5
    # oracle works on N,C,H,W: use N=rows, H=W=1
    xo = x.astype(np.float64).reshape(rows, C, 1, 1)
    dyo = dy.astype(np.float64).reshape(rows, C, 1, 1)
    yo, mean, invstd = nm.bn_fwd(xo, gamma.astype(np.float64), beta.astype(np.float64), eps)
    dxo, dgo, dbo = nm.bn_bwd_from_input(dyo, xo, gamma.astype(np.float64), mean, invstd)
    dx_, dg_, dbeta_, dd = dev(x), dev(gamma), dev(beta), dev(dy)
    scratch = torch.empty(2 << 20, dtype=torch.float32, device="cuda")
    stats = torch.empty(2 * C, dtype=torch.float32, device="cuda")
    monet.call("monet_bn_stats", None, dx_.data_ptr(), stats.data_ptr(), rows, C, eps, scratch.data_ptr(), scratch.numel() * 4)
    st = stats.cpu().numpy()
    assert rel(st[:C], mean) < 1e-5 and rel(st[C:], invstd) < 1e-5
    y = torch.empty_like(dx_)
    monet.call("monet_bn_apply", None, dx_.data_ptr(), y.data_ptr(), dg_.data_ptr(), dbeta_.data_ptr(), stats.data_ptr(), rows, C)
    check_close(y.cpu().numpy(), yo.reshape(rows, C), ACT_TOL)
    # in place
    xin = dx_.clone()
    monet.call("monet_bn_apply", None, xin.data_ptr(), xin.data_ptr(), dg_.data_ptr(), dbeta_.data_ptr(), stats.data_ptr(), rows, C)
    assert torch.equal(xin, y)
    for from_output, t in ((0, dx_), (1, y)):
        gx = torch.full((rows, C), float("nan"), dtype=torch.float32, device="cuda")
        gg = torch.empty(C, dtype=torch.float32, device="cuda")
        gb = torch.empty(C, dtype=torch.float32, device="cuda")
        monet.call("monet_bn_bwd", None, dd.data_ptr(), t.data_ptr(), from_output, dg_.data_ptr(), dbeta_.data_ptr(), stats.data_ptr(),
                   gx.data_ptr(), gg.data_ptr(), gb.data_ptr(), rows, C, 0, scratch.data_ptr(), scratch.numel() * 4)
        check_close(gx.cpu().numpy(), dxo.reshape(rows, C), GRAD_TOL)
        check_close(gg.cpu().numpy(), dgo, GRAD_TOL)
        check_close(gb.cpu().numpy(), dbo, GRAD_TOL)
        monet.call("monet_bn_bwd", None, dd.data_ptr(), t.data_ptr(), from_output, dg_.data_ptr(), dbeta_.data_ptr(), stats.data_ptr(),
                   gx.data_ptr(), gg.data_ptr(), gb.data_ptr(), rows, C, 1, scratch.data_ptr(), scratch.numel() * 4)
        check_close(gx.cpu().numpy(), 2 * dxo.reshape(rows, C), GRAD_TOL)


def test_batchnorm_statistics_with_large_offset():
    """Mean far from zero: a sum-of-squares formulation would lose the variance here."""
    torch = torch_mod()
    rows, C = 200000, 16
    rng = np.random.default_rng(7)
    x = (1000.0 + rng.standard_normal((rows, C))).astype(np.float32)
    mean, invstd = nm.bn_stats(x.astype(np.float64).reshape(rows, C, 1, 1), 1e-5)
    scratch = torch.empty(2 << 20, dtype=torch.float32, device="cuda")
    stats = torch.empty(2 * C, dtype=torch.float32, device="cuda")
    d = dev(x)
    monet.call("monet_bn_stats", None, d.data_ptr(), stats.data_ptr(), rows, C, 1e-5, scratch.data_ptr(), scratch.numel() * 4)
    st = stats.cpu().numpy()
    assert rel(st[:C], mean) < 1e-6 and rel(st[C:], invstd) < 1e-3


@pytest.mark.parametrize("shape", [(2, 16, 16, 16), (1, 5, 7, 3), (3, 9, 11, 40), (1, 1, 1, 64), (1, 1, 1, 1), (2, 33, 17, 130)])
@pytest.mark.parametrize("six", [0, 1])
def test_relu_and_mask_bit_exact(shape, six):
    torch = torch_mod()
    rng = np.random.default_rng(sum(shape) + six)
    x = (rng.standard_normal(shape) * (4 if six else 1)).astype(np.float32)
    flat = x.reshape(-1)
    flat[::7] = 0.0
    if flat.size > 3:
        flat[1] = -0.0
        flat[2] = np.nan
        flat[3] = 6.0
    n = x.size
    words = (n + 63) // 64
    d = dev(x)
    y = torch.empty_like(d)
    mask = torch.full((words + 1,), -1, dtype=torch.int64, device="cuda")     # one guard word
    monet.call("monet_relu_fwd", None, d.data_ptr(), y.data_ptr(), mask.data_ptr(), n, six)
    xo = wt.act_to_oracle(x)
    passes = nm.relu6_pass(xo) if six else nm.relu_pass(xo)
    want_mask = nm.pack_mask(passes)
    got_mask = mask.cpu().numpy().view(np.uint64)
    assert np.array_equal(got_mask[:words], want_mask)          # bit-exact, tail bits zero
    assert got_mask[words] == np.uint64(0xFFFFFFFFFFFFFFFF)     # nothing written past the end
    want_y = wt.act_from_oracle((nm.relu6_fwd if six else nm.relu_fwd)(xo))
    assert np.array_equal(y.cpu().numpy(), want_y.astype(np.float32))
    # in place, without a mask
    z = d.clone()
    monet.call("monet_relu_fwd", None, z.data_ptr(), z.data_ptr(), None, n, six)
    assert torch.equal(z, y)
    # backward: three variants give the same bits
    dz = rng.standard_normal(shape, dtype=np.float32)
    ddz = dev(dz)
    want = wt.act_from_oracle(wt.act_to_oracle(dz) * passes).astype(np.float32)
    for mode, t in ((0, d), (1, y), (2, mask)):
        gx = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_relu_bwd", None, ddz.data_ptr(), t.data_ptr(), mode, gx.data_ptr(), n, six, 0)
        assert np.array_equal(gx.cpu().numpy(), want), mode
        monet.call("monet_relu_bwd", None, ddz.data_ptr(), t.data_ptr(), mode, gx.data_ptr(), n, six, 1)
        assert np.array_equal(gx.cpu().numpy(), want + want), mode


@pytest.mark.parametrize("case", [(2, 16, 16, 8, 3, 2, 1), (1, 9, 7, 4, 2, 2, 0), (2, 12, 12, 64, 3, 2, 1), (1, 5, 5, 4, 3, 1, 1),
                                  (2, 14, 14, 64, 3, 1, 1), (1, 7, 9, 8, 3, 1, 1), (3, 28, 28, 192, 3, 1, 1),
                                  (1, 9, 7, 8, 3, 2, 1), (2, 13, 18, 12, 3, 2, 1), (1, 6, 5, 4, 3, 1, 1)])
def test_maxpool_index_bit_exact(case):
    torch = torch_mod()
    N, H, W, C, k, stride, pad = case
    rng = np.random.default_rng(sum(case))
    x = np.maximum(rng.standard_normal((N, H, W, C)), 0).astype(np.float32)      # post-ReLU: many exact ties at 0
    P = (H + 2 * pad - k) // stride + 1
    Q = (W + 2 * pad - k) // stride + 1
    dy = rng.standard_normal((N, P, Q, C), dtype=np.float32)
    yo, idxo = nm.maxpool_fwd(wt.act_to_oracle(x), k, stride, pad)
    d = dev(x)
    y = torch.empty((N, P, Q, C), dtype=torch.float32, device="cuda")
    idx = torch.empty((N, P, Q, C), dtype=torch.uint8, device="cuda")
    monet.call("monet_maxpool_fwd", None, d.data_ptr(), y.data_ptr(), idx.data_ptr(), N, H, W, C, k, stride, pad)
    assert np.array_equal(idx.cpu().numpy(), wt.act_from_oracle(idxo))
    assert np.array_equal(y.cpu().numpy(), wt.act_from_oracle(yo).astype(np.float32))
    want = wt.act_from_oracle(nm.maxpool_bwd_from_index(wt.act_to_oracle(dy), idxo, (N, C, H, W), k, stride, pad))
    ddy = dev(dy)
    got = {}
    for use_idx in (True, False):
        gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_maxpool_bwd", None, ddy.data_ptr(), d.data_ptr(), idx.data_ptr() if use_idx else None, gx.data_ptr(),
                   N, H, W, C, k, stride, pad, 0)
        assert rel(gx.cpu().numpy(), want) < 1e-6
        got[use_idx] = gx.clone()
        # added to what is there: the same sum once more (doubling is exact)
        monet.call("monet_maxpool_bwd", None, ddy.data_ptr(), d.data_ptr(), idx.data_ptr() if use_idx else None, gx.data_ptr(),
                   N, H, W, C, k, stride, pad, 1)
        assert torch.equal(gx, got[use_idx] + got[use_idx])
    # the kernels that read the stored index (row segments, compile-time windows) add the windows in the general kernel's order
    assert torch.equal(got[True], got[False])
