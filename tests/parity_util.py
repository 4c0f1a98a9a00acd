"""Shared pieces of the GPU parity tests (not a test module).

Floating-point comparisons are made twice per tensor: normwise (the stated tolerance) and element-wise
(`MAXABS_FACTOR` times the tolerance, on the scale of the reference's rms), so that one wrong element of a
large tensor cannot hide in the norm.

Decisions that fp32 cannot take (the sign of a ReLU input next to 0, the larger of two nearly equal window
taps) are handled here, outside the oracle: `SharedDecisions` wraps the oracle's operator functions, records
for every decision the GPU took differently how far the oracle's value is from the kink, and lets the
store-everything step go on with the GPU's decision only where that distance is below `DECISION_BAND`.
"""
import numpy as np

from oracle import network as onet
from oracle import numerics as nm
from workloads import schedules, tensors

ACT_TOL, GRAD_TOL = 1e-4, 1e-3
# BatchNorm outputs along the depth of a 50-layer network: fp32 rounding is amplified layer by layer
DEEP_ACT_TOL = 3e-4
MAXABS_FACTOR = 50.0      # element-wise bound: max|gpu - oracle| <= MAXABS_FACTOR * tol * rms(oracle)
# A decision may differ only where the oracle's value lies this close (in units of the tensor's rms) to the kink.
# The smallest decade that holds the measured distances of every differing decision: the farthest one over all
# parity runs is 5.6e-4 (ResNet-50 at batch 8, F(4x4) Winograd layers on; 3.2e-4 with the implicit GEMM alone),
# where the same tensors differ element-wise by up to 1.6e-3 rms; the shallower networks stay below 2e-4.
DECISION_BAND = 1e-3


def rel(got, want, floor=0.0):
    """Normwise relative error; a reference whose norm is below `floor` is measured against `floor`
    (a gradient that is zero in exact arithmetic has no scale of its own)."""
    want = np.asarray(want, np.float64)
    d = np.linalg.norm(np.asarray(got, np.float64) - want)
    n = max(np.linalg.norm(want), floor)
    return d if n == 0 else d / n


def maxabs(got, want, floor=0.0):
    """Largest element-wise difference on the scale of the reference's rms (of `floor` / sqrt(numel) when the
    reference's norm is below `floor`)."""
    want = np.asarray(want, np.float64)
    d = np.abs(np.asarray(got, np.float64) - want).max() if want.size else 0.0
    scale = max(np.linalg.norm(want), floor) / np.sqrt(max(want.size, 1))
    return d if scale == 0 else d / scale


def check_close(got, want, tol, what="", floor=0.0):
    """Asserts both error measures; returns (normwise, element-wise)."""
    e, m = rel(got, want, floor), maxabs(got, want, floor)
    assert e < tol, (what, "normwise", e)
    assert m < MAXABS_FACTOR * tol, (what, "max-abs over rms", m)
    return e, m


def compare_grads(got, ref, tol=GRAD_TOL, g=None):
    """Worst normwise error over the parameter gradients (each also checked element-wise).  The gradient of a
    BatchNorm shift vanishes identically when the BatchNorm feeds a convolution that is followed by another
    BatchNorm (a per-channel constant is removed again); the oracle then holds rounding noise of its own, so
    with the graph given such a gradient is measured on the scale of the same layer's scale gradient."""
    worst = 0.0
    for pid, want in ref["grads"].items():
        floor = 0.0
        if g is not None and g.params[pid][1].endswith(".beta"):
            floor = 1e-2 * np.linalg.norm(ref["grads"][pid - 1])
        e, _ = check_close(got[pid], tensors.weight_from_oracle(want), tol, what=("grad", pid), floor=floor)
        worst = max(worst, e)
    return worst


def to_oracle_shape(shape):
    if len(shape) == 4:
        n, h, w, c = shape
        return (n, c, h, w)
    return tuple(shape)


# ---------------------------------------------------------------------------------------------------------
# decisions shared between the two sides
def kink_distance(x, six=False):
    """|x| (for ReLU6 also |x - 6|) in units of the tensor's rms."""
    rms = np.sqrt(np.mean(x * x))
    d = np.abs(x)
    if six:
        d = np.minimum(d, np.abs(x - 6.0))
    return d / rms if rms > 0 else d


def tap_values(x, taps, k, stride, pad, out_hw):
    """Value of tap `taps` (r*k+s per window) in every k x k window of x; -inf for padding or an index
    outside the window."""
    N, C, H, W = x.shape
    P, Q = out_hw
    xp = np.full((N, C, H + 2 * pad, W + 2 * pad), -np.inf)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    val = np.full((N, C, P, Q), -np.inf)
    for r in range(k):
        for s in range(k):
            win = xp[:, :, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride]
            val = np.where(taps == r * k + s, win, val)
    return val


class SharedDecisions:
    """Operator functions for `oracle.network.store_everything_step` that take ReLU pass bits and max-pool
    taps from `given` ({relu node: boolean N,C,H,W array, max-pool node: uint8 tap indices}) where the
    oracle's own value is within `band` (times the input's rms) of the kink, and the oracle's strict decision
    everywhere else.  `records[node]` = dict(op, total, differ, adopted, max_dist): how many of the given
    decisions differ from the strict ones, how many of those were adopted (inside the band), and the
    largest distance from the kink among ALL differing ones (inside the band or not)."""

    def __init__(self, given, band=DECISION_BAND):
        self.given, self.band = given, band
        self.taken, self.records = {}, {}

    def forward(self, g, n, get, params, stats, recompute=False):
        y, aux = onet.forward_op(g, n, get, params, stats, recompute)
        if n.id not in self.given:
            return y, aux
        x = get(n.ins[0])
        given = self.given[n.id]
        if n.op in ("relu", "relu6"):
            six = n.op == "relu6"
            strict = nm.relu6_pass(x) if six else nm.relu_pass(x)
            differ = strict != given
            dist = kink_distance(x, six)
            adopt = differ & (dist < self.band)
            passes = np.where(adopt, given, strict)
            # an element that does not pass sits on the nearer saturation value (0, or 6 for ReLU6)
            y = np.where(passes, x, np.where(x < 3.0, 0.0, 6.0) if six else 0.0)
            aux["mask"] = lambda: nm.pack_mask(passes)
            self.taken[n.id] = passes
        elif n.op == "maxpool":
            k, stride, pad = int(n.attrs["k"]), int(n.attrs["stride"]), int(n.attrs["pad"])
            strict = aux["poolidx"]()
            differ = strict != given
            rms = np.sqrt(np.mean(x * x))
            dist = (y - tap_values(x, given, k, stride, pad, y.shape[2:])) / (rms if rms > 0 else 1.0)
            adopt = differ & (dist < self.band)
            idx = np.where(adopt, given, strict).astype(np.uint8)
            aux["poolidx"] = lambda: idx
            self.taken[n.id] = idx           # the forward value stays the window maximum
        else:
            raise ValueError(n.op)
        self.records[n.id] = dict(op=n.op, total=int(differ.size), differ=int(differ.sum()), adopted=int(adopt.sum()),
                                  max_dist=float(dist[differ].max()) if differ.any() else 0.0)
        return y, aux

    def backward(self, g, bop, algo, gy, get, params, stats):
        n = g.nodes[bop.node]
        if n.id in self.taken and bop.kind in ("relu_bwd", "relu6_bwd"):
            return {0: gy * self.taken[n.id]}, {}
        if n.id in self.taken and bop.kind == "maxpool_bwd":
            a = n.attrs
            xs = onet.nchw_shape(g.shape_of(n.ins[0]))
            return {0: nm.maxpool_bwd_from_index(gy, self.taken[n.id], xs, int(a["k"]), int(a["stride"]), int(a["pad"]))}, {}
        return onet.backward_op(g, bop, algo, gy, get, params, stats)

    def summary(self):
        r = self.records.values()
        return dict(total=sum(v["total"] for v in r), differ=sum(v["differ"] for v in r),
                    adopted=sum(v["adopted"] for v in r), max_dist=max((v["max_dist"] for v in r), default=0.0))


def step_with_decisions(graph_text, oe, op, given, band=DECISION_BAND):
    sd = SharedDecisions(given, band)
    ref = onet.store_everything_step(graph_text, oe, op, forward=sd.forward, backward=sd.backward)
    return ref, sd


def gpu_forward_tensors(g, exts, params, variants=None):
    """What the GPU's forward pass produced: ReLU pass bits and max-pool taps ({node: array} in the oracle's
    N,C,H,W order), the inputs of those operators, and every BatchNorm output ({node: N,H,W,C array}).
    A store-everything run under `variants` (masks and indices kept, nothing in place, the decision
    operators' inputs kept as well), stopped after the last forward operator."""
    import torch
    import paper_2010_14501_amd as M
    from paper_2010_14501_amd.runner import StepRunner
    variants = dict(schedules.DEFAULT_VARIANTS if variants is None else variants, inplace=False)
    bimpl = schedules.choose_bimpls(g, variants)
    F = schedules.store_everything_set(g, bimpl)
    F |= {n.ins[0] for n in g.nodes if n.op in ("relu", "relu6", "maxpool") and n.ins[0] > 0}
    sch = schedules.expand(g, F, bimpl, allow_inplace=False, conv_algo=variants["conv_fwd"])
    run = StepRunner(g.text(), sch.text(), exts, params)
    trace = run.plan.trace()
    last = [i for i, e in enumerate(trace) if e["kind"] == M.RUN_FWD][-1]
    run.plan.set_stop_after(last)
    run.step()
    torch.cuda.synchronize()

    def read(node):
        off = run.plan.tensor_offset(last, node.id)
        return None if off < 0 else run.read(off, node.shape)

    bits, pre, bn = {}, {}, {}
    for n in g.nodes:
        off = run.plan.tensor_offset(last, n.id)
        if off < 0:
            continue
        if n.op == "mask":
            relu = g.nodes[n.ins[0] - 1]
            words = run.read(off, (n.shape[0],), torch.int64).view(np.uint64)
            bits[relu.id] = nm.unpack_mask(words, to_oracle_shape(relu.shape))
        elif n.op == "poolidx":
            pool = g.nodes[n.ins[0] - 1]
            bits[pool.id] = np.ascontiguousarray(np.transpose(run.read(off, n.shape, torch.uint8), (0, 3, 1, 2)))
        elif n.op == "bn":
            bn[n.id] = run.read(off, n.shape)
    for node in bits:
        src = g.nodes[node - 1].ins[0]
        if src > 0:
            pre[node] = read(g.nodes[src - 1])
    return bits, pre, bn


def oracle_with_gpu_decisions(g, exts, params, variants=None, band=DECISION_BAND):
    """Store-everything oracle step sharing the GPU's undecidable decisions.  Checks, bit for bit, that
    (1) every decision of the GPU is the strict predicate applied to the GPU's own fp32 input (so a decision
    differs from the oracle's only because that input differs), and (2) every decision that differs from the
    oracle's lies inside the band.  Returns (ref, stats, gpu BatchNorm outputs); stats carries the counts, the
    largest distance of a differing decision from the kink, and the worst BatchNorm-output errors."""
    oe, op = tensors.oracle_inputs(exts, params)
    bits, pre, gpu_bn = gpu_forward_tensors(g, exts, params, variants)
    for node, x in pre.items():
        n = g.nodes[node - 1]
        if x is None:
            continue
        xo = tensors.act_to_oracle(x)        # exact: fp32 -> fp64
        if n.op == "maxpool":
            own = nm.maxpool_fwd(xo, n.attrs["k"], n.attrs["stride"], n.attrs["pad"])[1]
        else:
            own = nm.relu6_pass(xo) if n.op == "relu6" else nm.relu_pass(xo)
        assert np.array_equal(bits[node], own), ("decision is not the strict predicate of the GPU's own input", node)
    ref, sd = step_with_decisions(g.text(), oe, op, bits, band)
    st = sd.summary()
    outside = {i: r for i, r in sd.records.items() if r["adopted"] != r["differ"]}
    assert not outside, ("decisions differ outside the band", band, outside)
    errs = [(rel(a, tensors.act_from_oracle(ref["acts"][i])), maxabs(a, tensors.act_from_oracle(ref["acts"][i])))
            for i, a in gpu_bn.items()]
    st["worst_act"] = max((e for e, _ in errs), default=0.0)
    st["worst_act_maxabs"] = max((m for _, m in errs), default=0.0)
    st["records"] = sd.records
    # every differing decision is explained by the error of its own input: the GPU decided strictly on its own value
    # (checked above), so the oracle's value cannot be farther from the kink than the two inputs are from each other
    # (a window maximum: than twice that)
    for node, r in sd.records.items():
        if r["differ"] and pre.get(node) is not None:
            n = g.nodes[node - 1]
            gap = maxabs(pre[node], tensors.act_from_oracle(ref["acts"][n.ins[0]]))
            assert r["max_dist"] <= (2.0 if n.op == "maxpool" else 1.0) * gap * (1 + 1e-9), (node, r, gap)
    return ref, st, gpu_bn
