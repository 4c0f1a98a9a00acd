"""CPU tests of the parity helpers themselves: the two error measures, and the wrapper that lets the
store-everything oracle step share decisions fp32 cannot take (ReLU signs next to 0, nearly equal window taps)."""
import numpy as np
import pytest

from oracle import network as onet
from oracle import numerics as nm
from workloads import graphs, tensors
from parity_util import SharedDecisions, check_close, kink_distance, maxabs, rel, step_with_decisions, tap_values

SMALL_INCEPTIONS = (("a", 8, (8, 12), (4, 8), 4), "pool", ("b", 12, (8, 16), (4, 8), 8))


def test_one_wrong_element_fails_the_elementwise_measure_only():
    rng = np.random.default_rng(0)
    want = rng.standard_normal(1 << 20)
    got = want.astype(np.float32)
    assert check_close(got, want, 1e-4)[0] < 1e-7
    got[12345] += 0.05                                   # 5 % of the rms, one element of a million
    assert rel(got, want) < 1e-4                         # invisible in the norm
    assert 0.04 < maxabs(got, want) < 0.06
    with pytest.raises(AssertionError):
        check_close(got, want, 1e-4)
    # a reference that vanishes is measured on the floor's scale
    assert maxabs(np.full(4, 1e-9), np.zeros(4), floor=2.0) == pytest.approx(1e-9)


def test_kink_distance_counts_both_kinks_of_relu6():
    x = np.array([0.0, 3.0, 5.9, 6.2, -4.0])
    rms = np.sqrt(np.mean(x * x))
    assert np.allclose(kink_distance(x) * rms, [0, 3, 5.9, 6.2, 4])
    assert np.allclose(kink_distance(x, six=True) * rms, [0, 3, 0.1, 0.2, 4])


def test_shared_strict_decisions_change_nothing():
    """Handing the step its own strict ReLU6 decisions must reproduce the plain step exactly (in particular an
    element above 6 stays at 6), and nothing is recorded as differing."""
    g = graphs.mobilenet_v2(batch=2, hw=16, classes=5, stem=8, last=32, stages=((1, 8, 1, 1), (6, 12, 2, 2)))
    exts, params = tensors.make_inputs(g, seed=5, gamma_beta="random")
    params = {p: (3.0 * v if g.params[p][1].endswith(".gamma") else v) for p, v in params.items()}   # push values past 6
    oe, op = tensors.oracle_inputs(exts, params)
    plain = onet.store_everything_step(g.text(), oe, op)
    strict, above = {}, 0
    for n in g.nodes:
        if n.op == "relu6":
            x = plain["acts"][n.ins[0]]
            strict[n.id] = (x > 0) & (x < 6)
            above += int((x > 6).sum())
    assert above > 0
    shared, sd = step_with_decisions(g.text(), oe, op, strict, band=1e-3)
    assert shared["loss"] == plain["loss"]
    assert all(np.array_equal(shared["grads"][p], plain["grads"][p]) for p in plain["grads"])
    assert sd.summary()["differ"] == 0 and sd.summary()["total"] == sum(v.size for v in strict.values())


def test_a_flipped_sign_is_adopted_inside_the_band_only():
    """Two planted flips in the first ReLU of a chain: the one whose pre-activation is 1e-5 rms from 0 is adopted
    (and the backward pass then routes gradient through it), the one at 0.3 rms is refused and reported."""
    g = graphs.tiny_chain()
    exts, params = tensors.make_inputs(g, seed=1, gamma_beta="random")
    oe, op = tensors.oracle_inputs(exts, params)
    plain = onet.store_everything_step(g.text(), oe, op)
    relu = next(n for n in g.nodes if n.op == "relu")
    x = plain["acts"][relu.ins[0]]
    rms = np.sqrt(np.mean(x * x))
    order = np.argsort(np.abs(x), axis=None)
    near = np.unravel_index(order[0], x.shape)
    far = np.unravel_index(order[x.size // 4], x.shape)
    given = {relu.id: (x > 0).copy()}
    given[relu.id][near] ^= True
    given[relu.id][far] ^= True
    band = 2.0 * abs(x[near]) / rms
    assert abs(x[far]) / rms > 10 * band
    shared, sd = step_with_decisions(g.text(), oe, op, given, band=band)
    r = sd.records[relu.id]
    assert (r["differ"], r["adopted"]) == (2, 1)
    assert r["max_dist"] == pytest.approx(abs(x[far]) / rms)
    assert sd.taken[relu.id][near] == given[relu.id][near] and sd.taken[relu.id][far] != given[relu.id][far]
    # the input gradient of the ReLU follows the adopted decision
    dx_plain, dx_shared = plain["agrads"][relu.ins[0]], shared["agrads"][relu.ins[0]]
    assert (dx_plain[near] == 0) != (dx_shared[near] == 0)
    assert abs(shared["loss"] - plain["loss"]) <= 2 * abs(x[near]) * 1e3     # the loss moves by the tiny value only


def test_window_maxima_within_the_band_follow_the_given_tap():
    """2x2 / stride-2 pooling of a hand-made 4x4 map: a tap 1e-6 below the maximum may be taken instead
    (the gradient then goes there), one far below it, padding, or an index outside the window may not."""
    x = np.array([[1.0, 1.0 - 1e-6, 5.0, 2.0],
                  [0.5, 0.2, 4.0, 3.0],
                  [7.0, 7.0, -1.0, -2.0],
                  [6.0, 1.0, -3.0, -1.0 - 1e-7]]).reshape(1, 1, 4, 4)
    given = np.array([1, 3, 1, 200], np.uint8).reshape(1, 1, 2, 2)       # near-tie, far below, exact tie, invalid
    assert tap_values(x, given, 2, 2, 0, (2, 2)).ravel().tolist() == [1.0 - 1e-6, 3.0, 7.0, -np.inf]

    class Node:
        id, op, ins, attrs = 1, "maxpool", (0,), dict(k=2, stride=2, pad=0)
    sd = SharedDecisions({1: given}, band=1e-3)
    y, aux = sd.forward(None, Node, lambda ref: x, {}, {})
    assert y.ravel().tolist() == [1.0, 5.0, 7.0, -1.0]                    # the forward value stays the maximum
    assert aux["poolidx"]().ravel().tolist() == [1, 0, 1, 0]
    r = sd.records[1]
    assert (r["differ"], r["adopted"]) == (4, 2) and r["max_dist"] == np.inf
    dy = np.array([10.0, 20.0, 30.0, 40.0]).reshape(1, 1, 2, 2)
    dx = nm.maxpool_bwd_from_index(dy, sd.taken[1], x.shape, 2, 2, 0)
    want = np.zeros((4, 4)); want[0, 1] = 10; want[0, 2] = 20; want[2, 1] = 30; want[2, 2] = 40
    assert np.array_equal(dx[0, 0], want)
    # with padding: a given tap that points into the padding ring is refused
    Node.attrs = dict(k=3, stride=2, pad=1)
    _, idx = nm.maxpool_fwd(x, 3, 2, 1)
    sd = SharedDecisions({1: np.zeros(idx.shape, np.uint8)}, band=1e-3)   # tap (0,0): padding for the first row / column of windows
    _, aux = sd.forward(None, Node, lambda ref: x, {}, {})
    assert np.array_equal(aux["poolidx"]()[0, 0, 0, :], idx[0, 0, 0, :])


def test_shared_strict_window_maxima_change_nothing():
    """Handing the step its own max-pool indices must reproduce the plain step exactly.  Handing it the next tap
    everywhere changes an index only where that tap ties with the maximum exactly (all-zero windows after a
    ReLU; a stride-1 pool over a stride-2 pool sees the same element twice): the gradient then takes another
    route to the same place, so the result agrees to rounding."""
    g = graphs.googlenet(batch=2, hw=32, classes=10, stem=(8, 8, 16), inceptions=SMALL_INCEPTIONS)
    exts, params = tensors.make_inputs(g, seed=5, gamma_beta="random")
    oe, op = tensors.oracle_inputs(exts, params)
    plain = onet.store_everything_step(g.text(), oe, op)
    own, shifted = {}, {}
    for n in g.nodes:
        if n.op == "maxpool":
            idx = nm.maxpool_fwd(plain["acts"][n.ins[0]], n.attrs["k"], n.attrs["stride"], n.attrs["pad"])[1]
            own[n.id] = idx
            shifted[n.id] = ((idx + 1) % (n.attrs["k"] ** 2)).astype(np.uint8)
    assert len(own) >= 5
    shared, sd = step_with_decisions(g.text(), oe, op, own, band=1e-9)
    assert shared["loss"] == plain["loss"]
    assert all(np.array_equal(shared["grads"][p], plain["grads"][p]) for p in plain["grads"])
    assert all(np.array_equal(sd.taken[i], own[i]) for i in own) and sd.summary()["differ"] == 0
    shared, sd = step_with_decisions(g.text(), oe, op, shifted, band=1e-9)
    assert shared["loss"] == plain["loss"]
    top = max(np.linalg.norm(v) for v in plain["grads"].values())
    assert all(np.linalg.norm(shared["grads"][p] - plain["grads"][p]) < 1e-13 * top for p in plain["grads"])
    for i in own:
        changed = sd.taken[i] != own[i]
        assert changed.sum() == sd.records[i]["adopted"] and changed.mean() < 0.5
