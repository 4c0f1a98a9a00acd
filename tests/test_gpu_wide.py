"""GPU parity for the operators and networks of the VGG-16 / UNet / MobileNetV2 configurations:
transposed convolution, depthwise convolution, channel concatenation, per-pixel cross-entropy
(kernel by kernel through the C ABI against the fp64 oracle), then whole training steps of reduced
versions of the three networks (reduced width or resolution: the fp64 oracle has to finish in
seconds) under a store-everything and a recomputing schedule."""
import numpy as np
import pytest

from oracle import numerics as nm
from oracle import schedule as osch
from workloads import graphs, schedules, tensors as wt
from paper_2010_14501_amd import monet
from paper_2010_14501_amd.runner import StepRunner
from parity_util import (ACT_TOL, GRAD_TOL, DEEP_ACT_TOL, DECISION_BAND, rel, check_close, compare_grads,
                         oracle_with_gpu_decisions)

pytestmark = pytest.mark.gpu


def torch_mod():
    import torch
    return torch


def dev(a):
    return torch_mod().from_numpy(np.ascontiguousarray(a)).cuda()


# ------------------------------------------------------------------ transposed convolution
TCONV_CASES = [
    # N, H, W, C, K, R, stride
    (2, 6, 9, 32, 16, 2, 2),        # the up-sampling layer's form
    (3, 13, 19, 128, 64, 2, 2),     # several tiles, ragged rows
    (1, 5, 7, 20, 12, 2, 2),        # channel counts that are not multiples of 16
    (2, 4, 5, 16, 16, 3, 2),        # overlapping taps
]


@pytest.mark.parametrize("case", TCONV_CASES)
def test_tconv_trio_matches_oracle(case):
    torch = torch_mod()
    N, H, W, C, K, R, stride = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    P, Q = (H - 1) * stride + R, (W - 1) * stride + R
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = rng.standard_normal((C, R, R, K), dtype=np.float32) * np.float32(np.sqrt(1.0 / C))
    dy = rng.standard_normal((N, P, Q, K), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)     # wo: C,K,R,S
    dx_, dw_, ddy = dev(x), dev(w), dev(dy)
    y = torch.full((N, P, Q, K), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_tconv_fwd", None, dx_.data_ptr(), dw_.data_ptr(), y.data_ptr(), N, H, W, C, K, R, R, stride)
    check_close(y.cpu().numpy(), wt.act_from_oracle(nm.tconv2d_fwd(xo, wo, stride)), ACT_TOL)
    gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
    want = wt.act_from_oracle(nm.tconv2d_dgrad(dyo, wo, stride))
    monet.call("monet_tconv_dgrad", None, ddy.data_ptr(), dw_.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, 0)
    check_close(gx.cpu().numpy(), want, GRAD_TOL)
    monet.call("monet_tconv_dgrad", None, ddy.data_ptr(), dw_.data_ptr(), gx.data_ptr(), N, H, W, C, K, R, R, stride, 1)
    check_close(gx.cpu().numpy(), 2 * want, GRAD_TOL)
    want = wt.weight_from_oracle(nm.tconv2d_wgrad(xo, dyo, R, R, stride))
    ws = torch.empty(4 * w.size, dtype=torch.float32, device="cuda")
    for splits in (1, 3):
        gw = torch.full((C, R, R, K), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_tconv_wgrad", None, dx_.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, C, K, R, R, stride,
                   splits, ws.data_ptr(), ws.numel() * 4)
        check_close(gw.cpu().numpy(), want, GRAD_TOL, what=splits)


# ------------------------------------------------------------------ depthwise convolution
DW_CASES = [
    # N, H, W, C, R, stride, pad
    (2, 14, 14, 32, 3, 1, 1),
    (3, 15, 13, 96, 3, 2, 1),       # stride 2, odd extents
    (2, 28, 28, 960, 3, 1, 1),      # the widest expansion
    (1, 9, 11, 10, 3, 1, 1),        # C % 4 != 0: scalar path
    (2, 8, 8, 24, 3, 2, 0),         # no padding
    (4, 56, 56, 144, 3, 2, 1),      # many slabs in the filter-gradient reduction
    (3, 7, 5, 16, 3, 1, 1),         # rows shorter than one segment of the row kernels
    (2, 112, 112, 32, 3, 1, 1),     # long rows: many segments, the last one ragged
]


@pytest.mark.parametrize("case", DW_CASES)
def test_dwconv_trio_matches_oracle(case):
    torch = torch_mod()
    N, H, W, C, R, stride, pad = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = rng.standard_normal((C, R, R, 1), dtype=np.float32) * np.float32(1.0 / R)
    dy = rng.standard_normal((N, P, Q, C), dtype=np.float32)
    xo, wo, dyo = wt.act_to_oracle(x), wt.weight_to_oracle(w), wt.act_to_oracle(dy)     # wo: C,1,R,S
    dx_, dw_, ddy = dev(x), dev(w), dev(dy)
    y = torch.full((N, P, Q, C), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_dwconv_fwd", None, dx_.data_ptr(), dw_.data_ptr(), y.data_ptr(), N, H, W, C, R, R, stride, pad)
    check_close(y.cpu().numpy(), wt.act_from_oracle(nm.dwconv2d_fwd(xo, wo, stride, pad)), ACT_TOL)
    gx = torch.full((N, H, W, C), float("nan"), dtype=torch.float32, device="cuda")
    want = wt.act_from_oracle(nm.dwconv2d_dgrad(dyo, wo, xo.shape, stride, pad))
    monet.call("monet_dwconv_dgrad", None, ddy.data_ptr(), dw_.data_ptr(), gx.data_ptr(), N, H, W, C, R, R, stride, pad, 0)
    check_close(gx.cpu().numpy(), want, GRAD_TOL)
    monet.call("monet_dwconv_dgrad", None, ddy.data_ptr(), dw_.data_ptr(), gx.data_ptr(), N, H, W, C, R, R, stride, pad, 1)
    check_close(gx.cpu().numpy(), 2 * want, GRAD_TOL)
    want = wt.weight_from_oracle(nm.dwconv2d_wgrad(xo, dyo, R, R, stride, pad))
    for scratch_floats in (R * R * C, 1 << 20):     # one slab only, and many slabs
        scratch = torch.empty(scratch_floats, dtype=torch.float32, device="cuda")
        gw = torch.full((C, R, R, 1), float("nan"), dtype=torch.float32, device="cuda")
        monet.call("monet_dwconv_wgrad", None, dx_.data_ptr(), ddy.data_ptr(), gw.data_ptr(), N, H, W, C, R, R, stride, pad,
                   scratch.data_ptr(), scratch.numel() * 4)
        check_close(gw.cpu().numpy(), want, GRAD_TOL, what=scratch_floats)
    # the reduction order is fixed: two runs give the same bits
    gw2 = torch.empty_like(gw)
    monet.call("monet_dwconv_wgrad", None, dx_.data_ptr(), ddy.data_ptr(), gw2.data_ptr(), N, H, W, C, R, R, stride, pad,
               scratch.data_ptr(), scratch.numel() * 4)
    assert torch.equal(gw, gw2)


def test_dwconv_rejects_more_than_nine_taps():
    torch = torch_mod()
    t = torch.zeros(4096, dtype=torch.float32, device="cuda")
    with pytest.raises(monet.MonetError):
        monet.call("monet_dwconv_fwd", None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 1, 8, 8, 4, 5, 5, 1, 2)


# ------------------------------------------------------------------ concatenation copies
@pytest.mark.parametrize("rows,ca,cb", [(1000, 64, 64), (77, 12, 20), (513, 5, 3), (0, 8, 8)])
def test_column_copy_is_exact(rows, ca, cb):
    torch = torch_mod()
    rng = np.random.default_rng(rows + ca)
    a = rng.standard_normal((rows, ca), dtype=np.float32)
    b = rng.standard_normal((rows, cb), dtype=np.float32)
    da, db = dev(a), dev(b)
    out = torch.full((rows, ca + cb), float("nan"), dtype=torch.float32, device="cuda")
    monet.call("monet_column_copy", None, da.data_ptr(), ca, out.data_ptr(), ca + cb, ca, rows, 0)
    monet.call("monet_column_copy", None, db.data_ptr(), cb, out.data_ptr() + 4 * ca, ca + cb, cb, rows, 0)
    want = np.concatenate([a, b], axis=1)
    assert np.array_equal(out.cpu().numpy(), want)
    # backward: slices of the gradient, written or accumulated
    ga = torch.full((rows, ca), 1.0, dtype=torch.float32, device="cuda")
    monet.call("monet_column_copy", None, out.data_ptr(), ca + cb, ga.data_ptr(), ca, ca, rows, 1)
    assert np.array_equal(ga.cpu().numpy(), a + np.float32(1.0))
    gb = torch.empty((rows, cb), dtype=torch.float32, device="cuda")
    monet.call("monet_column_copy", None, out.data_ptr() + 4 * ca, ca + cb, gb.data_ptr(), cb, cb, rows, 0)
    assert np.array_equal(gb.cpu().numpy(), b)


# ------------------------------------------------------------------ cross-entropy over many short rows
@pytest.mark.parametrize("rows,classes", [(2 * 32 * 48, 2), (100003, 5), (7, 21)])
def test_softmaxce_rows_matches_oracle(rows, classes):
    torch = torch_mod()
    rng = np.random.default_rng(rows)
    z = (3 * rng.standard_normal((rows, classes))).astype(np.float32)
    lab = rng.integers(0, classes, size=rows, dtype=np.int32)
    dz, dl = dev(z), dev(lab)
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    scratch = torch.empty(1024, dtype=torch.float32, device="cuda")
    monet.call("monet_softmaxce_rows_fwd", None, dz.data_ptr(), dl.data_ptr(), loss.data_ptr(), rows, classes, scratch.data_ptr(), 4096)
    want = nm.softmaxce_fwd(z.astype(np.float64), lab)
    assert abs(float(loss.item()) - want) < ACT_TOL * abs(want)
    g = torch.full((rows, classes), 1.0, dtype=torch.float32, device="cuda")
    wantg = nm.softmaxce_bwd(z.astype(np.float64), lab)
    monet.call("monet_softmaxce_rows_bwd", None, dz.data_ptr(), dl.data_ptr(), g.data_ptr(), rows, classes, 0)
    check_close(g.cpu().numpy(), wantg, GRAD_TOL)
    monet.call("monet_softmaxce_rows_bwd", None, dz.data_ptr(), dl.data_ptr(), g.data_ptr(), rows, classes, 1)
    check_close(g.cpu().numpy(), 2 * wantg, GRAD_TOL)


# ------------------------------------------------------------------ whole steps
def small_vgg():
    return graphs.vgg16_bn(batch=2, hw=32, classes=10, widths=(8, 16, 16, 32, 32), fc=64)


def small_unet():
    return graphs.unet(batch=2, h=32, w=48, classes=2, base=8, depth=4)


def small_mbv2():
    return graphs.mobilenet_v2(batch=2, hw=32, classes=10, stem=8, last=64,
                               stages=((1, 8, 1, 1), (6, 12, 2, 2), (6, 16, 2, 2), (6, 24, 1, 1)))


def alternate_blocks_schedule(g, variants=schedules.DEFAULT_VARIANTS):
    """Every second block is recomputed (its own tensors are not kept)."""
    keep = {b for b in range(len(g.blocks)) if b % 2 == 0} | {len(g.blocks) - 1}
    bimpl = schedules.choose_bimpls(g, variants)
    F = schedules.block_checkpoint_set(g, bimpl, keep)
    return schedules.expand(g, F, bimpl, allow_inplace=True, conv_algo=variants["conv_fwd"])


def small_googlenet():
    # 64x64 input: the second module still sees 4x4 positions, i.e. 32 samples per BatchNorm channel
    return graphs.googlenet(batch=2, hw=64, classes=10, stem=(8, 8, 16),
                            inceptions=(("a", 8, (8, 12), (4, 8), 4), "pool", ("b", 12, (8, 16), (4, 8), 8)))


NETS = {
    "vgg": small_vgg, "unet": small_unet, "mbv2": small_mbv2, "googlenet": small_googlenet,
    # full channel widths at a resolution the fp64 oracle manages
    "vgg_wide": lambda: graphs.vgg16_bn(batch=2, hw=32, classes=1000, fc=512),
    "unet_wide": lambda: graphs.unet(batch=1, h=32, w=48),
    "mbv2_wide": lambda: graphs.mobilenet_v2(batch=2, hw=64),
    # the inception network at its real geometry: on smaller maps the 3x3 / stride-1 pool branch turns nearly constant
    # over the positions and its BatchNorm ill-conditioned, which says nothing about the kernels
    "googlenet_wide": lambda: graphs.googlenet(batch=2, hw=224),
    # the networks of the paper's model list at their input sizes, at the batch the fp64 oracle does in a minute:
    # only these reach F(4x4) Winograd on 224x224x64 maps and its chunked workspace, 112-pixel depthwise rows,
    # non-square 416x608 maps and 2x2 pools on large maps
    "vgg_full": lambda: graphs.vgg16_bn(batch=2),
    "mbv2_full": lambda: graphs.mobilenet_v2(batch=2),
    "unet_full": lambda: graphs.unet(batch=1),
}
VARIANT_SETS = {"default": schedules.DEFAULT_VARIANTS, "igemm": schedules.IGEMM_VARIANTS, "im2col": schedules.IM2COL_VARIANTS}
# the explicit patch-matrix form of every 3x3 / 7x7 convolution (forward, recomputation, filter gradient): a small
# network of each family with 3x3 layers, the inception network at 224x224 (7x7 / stride 2 stem with 3 input channels,
# R*S*C no multiple of 16) and VGG-16 at full resolution (several chunks per layer)
CASES = ([(name, "default") for name in NETS] + [(name, "igemm") for name in NETS if name.endswith("_full")] +
         [(name, "im2col") for name in ("vgg", "unet", "googlenet_wide", "vgg_full")])


@pytest.mark.parametrize("name,vname", CASES)
def test_network_step_against_oracle(name, vname):
    g = NETS[name]()
    variants = VARIANT_SETS[vname]
    exts, params = wt.make_inputs(g, seed=3, gamma_beta="random")
    ref, st, _ = oracle_with_gpu_decisions(g, exts, params, variants)
    print(f"{name} {vname}: {st['differ']} of {st['total']} decisions differ, farthest from the kink {st['max_dist']:.2e} rms "
          f"(band {DECISION_BAND:.0e}); worst BatchNorm-output error {st['worst_act']:.2e} normwise, "
          f"{st['worst_act_maxabs']:.2e} rms element-wise")
    assert st["differ"] < 1e-4 * st["total"] + 8
    assert st["worst_act"] < DEEP_ACT_TOL and st["worst_act_maxabs"] < 50 * DEEP_ACT_TOL
    got = {}
    for sname, make in (("store", lambda g: schedules.store_everything_schedule(g, variants)),
                        ("block_outputs", lambda g: schedules.block_output_schedule(g, variants)),
                        ("alternate", lambda g: alternate_blocks_schedule(g, variants))):
        sch = make(g)
        want = osch.interpret(g.text(), sch.text())
        run = StepRunner(g.text(), sch.text(), exts, params, poison=True)
        peak = run.step()
        assert peak == want["peak"] == run.plan.exact_peak <= run.plan.predicted_peak, sname
        assert abs(run.loss_value() - ref["loss"]) < ACT_TOL * abs(ref["loss"]), sname
        got[sname] = run.grads_numpy()
        worst = compare_grads(got[sname], ref, g=g)
        print(f"{name} {vname}/{sname}: peak {peak}, recomputes {want['recomputes']}, worst gradient error {worst:.2e}")
        del run
    # recomputation alone must not change a bit
    for sname in ("block_outputs", "alternate"):
        same = [np.array_equal(got["store"][p], got[sname][p]) for p in got["store"]]
        assert all(same), (sname, [p for p, s in enumerate(same) if not s])
