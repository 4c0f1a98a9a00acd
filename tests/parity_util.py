"""Shared pieces of the GPU parity tests (not a test module)."""
import numpy as np

from oracle import network as onet
from oracle import numerics as nm
from workloads import schedules, tensors

ACT_TOL, GRAD_TOL = 1e-4, 1e-3
UNDECIDED_BAND = 1e-3     # a ReLU input within 1e-3 * rms of a kink cannot be decided at the 1e-4 activation tolerance


def rel(got, want, floor=0.0):
    """Normwise relative error; a reference whose norm is below `floor` is measured against `floor`
    (a gradient that is zero in exact arithmetic has no scale of its own)."""
    want = np.asarray(want, np.float64)
    d = np.linalg.norm(np.asarray(got, np.float64) - want)
    n = max(np.linalg.norm(want), floor)
    return d if n == 0 else d / n


def compare_grads(got, ref, tol=GRAD_TOL, g=None):
    """Worst normwise error over the parameter gradients.  The gradient of a BatchNorm shift vanishes
    identically when the BatchNorm feeds a convolution that is followed by another BatchNorm (a
    per-channel constant is removed again); the oracle then holds rounding noise of its own, so with
    the graph given such a gradient is measured on the scale of the same layer's scale gradient."""
    worst = 0.0
    for pid, want in ref["grads"].items():
        floor = 0.0
        if g is not None and g.params[pid][1].endswith(".beta"):
            floor = 1e-2 * np.linalg.norm(ref["grads"][pid - 1])
        e = rel(got[pid], tensors.weight_from_oracle(want), floor=floor)
        worst = max(worst, e)
        assert e < tol, (pid, e)
    return worst


def to_oracle_shape(shape):
    if len(shape) == 4:
        n, h, w, c = shape
        return (n, c, h, w)
    return tuple(shape)


def gpu_relu_decisions(g, exts, params):
    """ReLU pass bits and max-pool tap indices as the GPU took them, and its BatchNorm outputs: a store-everything run (the lean
    variants keep every mask, nothing in place), stopped after the last forward operator."""
    import torch
    import paper_2010_14501_amd as M
    from paper_2010_14501_amd.runner import StepRunner
    sch = schedules.store_everything_schedule(g, dict(schedules.DEFAULT_VARIANTS, inplace=False))
    run = StepRunner(g.text(), sch.text(), exts, params)
    trace = run.plan.trace()
    last = [i for i, e in enumerate(trace) if e["kind"] == M.RUN_FWD][-1]
    run.plan.set_stop_after(last)
    run.step()
    torch.cuda.synchronize()
    out, acts = {}, {}
    for n in g.nodes:
        off = run.plan.tensor_offset(last, n.id)
        if off < 0:
            continue
        if n.op == "mask":
            relu = g.nodes[n.ins[0] - 1]
            words = run.read(off, (n.shape[0],), torch.int64).view(np.uint64)
            out[relu.id] = nm.unpack_mask(words, to_oracle_shape(relu.shape))
        elif n.op == "poolidx":
            pool = g.nodes[n.ins[0] - 1]
            out[pool.id] = np.ascontiguousarray(np.transpose(run.read(off, n.shape, torch.uint8), (0, 3, 1, 2)))
        elif n.op == "bn":
            acts[n.id] = run.read(off, n.shape)
    return out, acts


def oracle_with_gpu_ties(g, exts, params):
    """Store-everything oracle step in which ReLU decisions and max-pool taps inside the undecidable band
    follow the GPU; checks that every decided bit / index is bit-exact.  Returns (ref, stats dict, gpu BatchNorm outputs)."""
    oe, op = tensors.oracle_inputs(exts, params)
    gpu_bits, gpu_bn = gpu_relu_decisions(g, exts, params)
    ref = onet.store_everything_step(g.text(), oe, op, ties=(UNDECIDED_BAND, gpu_bits))
    flips, undecided_total, total = 0, 0, 0
    for node, (passes, undecided) in ref["decisions"].items():
        n = g.nodes[node - 1]
        x = ref["acts"][n.ins[0]]
        if n.op == "maxpool":       # tap indices: outside the undecidable windows the GPU's choice is the oracle's
            strict = nm.maxpool_fwd(x, n.attrs["k"], n.attrs["stride"], n.attrs["pad"])[1]
            assert np.array_equal(gpu_bits[node][~undecided], strict[~undecided]), node
            flips += int(undecided.sum())
            undecided_total += int(undecided.sum())
            total += strict.size
            continue
        strict = (x > 0) & (x < 6) if n.op == "relu6" else (x > 0)
        assert np.array_equal(gpu_bits[node][~undecided], strict[~undecided]), node
        flips += int((gpu_bits[node][undecided] != strict[undecided]).sum())
        undecided_total += int(undecided.sum())
        total += x.size
    worst_act = max((rel(a, tensors.act_from_oracle(ref["acts"][i])) for i, a in gpu_bn.items()), default=0.0)
    return ref, dict(flips=flips, undecided=undecided_total, total=total, worst_act=worst_act), gpu_bn
