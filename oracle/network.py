"""Store-everything forward/backward of a graph in fp64 (test infrastructure).

This is plain back-propagation over the forward DAG of Section 3: every
activation is kept, every backward operator uses the input-activated textbook
form.  The schedule interpreter must reproduce these gradients for every
feasible schedule (Section 3: an activation that is not stored is recomputed
when needed, so the result does not change).

Arrays are N,C,H,W; convolution weights K,C,R,S; `params[pid]` and
`exts[ref]` are supplied by the caller in that convention.
"""
import numpy as np

from . import numerics as nm
from .graphtext import OGraph


def nchw_shape(shape):
    """Graph text declares N,H,W,C; the oracle holds N,C,H,W."""
    if len(shape) == 4:
        n, h, w, c = shape
        return (n, c, h, w)
    return tuple(shape)


def forward_op(g: OGraph, n, get, params, stats, recompute=False):
    """Output of node n (and its aux outputs as a dict op->array).

    `get(ref)` returns an input array.  BatchNorm statistics are taken from
    `stats[n.id]` on recomputation (Appendix D: statistics are reused) and
    written there otherwise.
    """
    a = n.attrs
    x = get(n.ins[0])
    aux = {}
    if n.op == "conv":
        y = nm.conv2d_fwd(x, params[n.pars[0]], int(a["stride"]), int(a["pad"]))
    elif n.op == "bn":
        gamma, beta = params[n.pars[0]], params[n.pars[1]]
        if recompute:
            mean, invstd = stats[n.id]
            y = nm.bn_apply(x, gamma, beta, mean, invstd)
        else:
            y, mean, invstd = nm.bn_fwd(x, gamma, beta, float(a["eps"]))
            stats[n.id] = (mean, invstd)
    elif n.op in ("relu", "relu6"):
        six = n.op == "relu6"
        y = nm.relu6_fwd(x) if six else nm.relu_fwd(x)
        aux["mask"] = lambda: nm.pack_mask(nm.relu6_pass(x) if six else nm.relu_pass(x))
    elif n.op == "maxpool":
        y, idx = nm.maxpool_fwd(x, int(a["k"]), int(a["stride"]), int(a["pad"]))
        aux["poolidx"] = lambda: idx
    elif n.op == "tconv":
        y = nm.tconv2d_fwd(x, params[n.pars[0]], int(a["stride"]))
    elif n.op == "dwconv":
        y = nm.dwconv2d_fwd(x, params[n.pars[0]], int(a["stride"]), int(a["pad"]))
    elif n.op == "concat":
        y = nm.concat_fwd(x, get(n.ins[1]))
    elif n.op == "add":
        y = x + get(n.ins[1])
    elif n.op == "avgpool":
        y = nm.avgpool_fwd(x)
    elif n.op == "linear":
        y = nm.linear_fwd(x, params[n.pars[0]], params[n.pars[1]])
    elif n.op == "softmaxce":
        y = np.array([nm.softmaxce_fwd(x, get(n.ins[1]))])
    elif n.op == "sumloss":
        y = np.array([nm.sumloss_fwd(x)])
    else:
        raise ValueError(n.op)
    return y, aux


def backward_op(g: OGraph, bop, algo, gy, get, params, stats):
    """(input gradients {input position: array}, parameter gradients {pid: array}).

    `get(ref)` returns a forward tensor the chosen implementation depends on.
    """
    n = g.nodes[bop.node]
    a = n.attrs
    kind = bop.kind
    if kind == "conv_wgrad":
        x = get(n.ins[0])
        return {}, {n.pars[0]: nm.conv2d_wgrad(x, gy, int(a["R"]), int(a["S"]), int(a["stride"]), int(a["pad"]))}
    if kind == "conv_dgrad":
        xs = nchw_shape(g.shape_of(n.ins[0]))
        return {0: nm.conv2d_dgrad(gy, params[n.pars[0]], xs, int(a["stride"]), int(a["pad"]))}, {}
    if kind == "tconv_wgrad":
        return {}, {n.pars[0]: nm.tconv2d_wgrad(get(n.ins[0]), gy, int(a["R"]), int(a["S"]), int(a["stride"]))}
    if kind == "tconv_dgrad":
        return {0: nm.tconv2d_dgrad(gy, params[n.pars[0]], int(a["stride"]))}, {}
    if kind == "dwconv_wgrad":
        return {}, {n.pars[0]: nm.dwconv2d_wgrad(get(n.ins[0]), gy, int(a["R"]), int(a["S"]), int(a["stride"]), int(a["pad"]))}
    if kind == "dwconv_dgrad":
        xs = nchw_shape(g.shape_of(n.ins[0]))
        return {0: nm.dwconv2d_dgrad(gy, params[n.pars[0]], xs, int(a["stride"]), int(a["pad"]))}, {}
    if kind == "concat_bwd":
        da, db = nm.concat_bwd(gy, nchw_shape(g.shape_of(n.ins[0]))[1])
        return {0: da, 1: db}, {}
    if kind == "bn_bwd":
        gamma, beta = params[n.pars[0]], params[n.pars[1]]
        mean, invstd = stats[n.id]
        if algo == "from_input":
            dx, dg, db = nm.bn_bwd_from_input(gy, get(n.ins[0]), gamma, mean, invstd)
        elif algo == "from_output":
            dx, dg, db = nm.bn_bwd_from_output(gy, get(n.id), gamma, beta, invstd)
        else:
            raise ValueError(algo)
        return {0: dx}, {n.pars[0]: dg, n.pars[1]: db}
    if kind in ("relu_bwd", "relu6_bwd"):
        six = kind == "relu6_bwd"
        if algo == "from_input":
            dx = (nm.relu6_bwd_from_input if six else nm.relu_bwd_from_input)(gy, get(n.ins[0]))
        elif algo == "from_output":
            dx = (nm.relu6_bwd_from_output if six else nm.relu_bwd_from_output)(gy, get(n.id))
        elif algo == "from_mask":
            dx = nm.relu_bwd_from_mask(gy, get(g.aux_children[n.id][0]))
        else:
            raise ValueError(algo)
        return {0: dx}, {}
    if kind == "maxpool_bwd":
        xs = nchw_shape(g.shape_of(n.ins[0]))
        k, st, pd = int(a["k"]), int(a["stride"]), int(a["pad"])
        if algo == "from_input":
            dx = nm.maxpool_bwd_from_input(gy, get(n.ins[0]), k, st, pd)
        elif algo == "from_index":
            dx = nm.maxpool_bwd_from_index(gy, get(g.aux_children[n.id][0]), xs, k, st, pd)
        else:
            raise ValueError(algo)
        return {0: dx}, {}
    if kind == "add_bwd":
        return {0: gy, 1: gy}, {}
    if kind == "avgpool_bwd":
        return {0: nm.avgpool_bwd(gy, nchw_shape(g.shape_of(n.ins[0])))}, {}
    if kind == "linear_wgrad":
        dw, db = nm.linear_wgrad(get(n.ins[0]), gy)
        return {}, {n.pars[0]: dw, n.pars[1]: db}
    if kind == "linear_dgrad":
        return {0: nm.linear_dgrad(gy, params[n.pars[0]], nchw_shape(g.shape_of(n.ins[0])))}, {}
    if kind == "softmaxce_bwd":
        return {0: nm.softmaxce_bwd(get(n.ins[0]), get(n.ins[1]))}, {}
    if kind == "sumloss_bwd":
        return {0: nm.sumloss_bwd(nchw_shape(g.shape_of(n.ins[0])))}, {}
    raise ValueError(kind)


def store_everything_step(graph_text, exts, params, forward=None, backward=None):
    """Plain training step.  Returns dict(loss, acts{i: array}, aux{i: array}, grads{pid: array},
    agrads{i: array}, stats{i: (mean, invstd)}).

    `forward` / `backward` stand in for `forward_op` / `backward_op` (same arguments, same results) when a
    caller wants to look at, or wrap, the operators one by one; left out, the definitions above are used."""
    g = OGraph(graph_text)
    forward = forward_op if forward is None else forward
    backward = backward_op if backward is None else backward
    acts, auxv, stats = {}, {}, {}

    def get(ref):
        return exts[ref] if ref <= 0 else acts[ref]

    for i in range(1, g.N + 1):
        n = g.nodes[i]
        if n.is_aux:
            continue
        y, aux = forward(g, n, get, params, stats)
        acts[i] = y
        for c in g.aux_children[i]:
            auxv[c] = aux[g.nodes[c].op]()
    loss = float(acts[g.N][0])

    def get_any(ref):
        if ref <= 0:
            return exts[ref]
        return auxv[ref] if g.nodes[ref].is_aux else acts[ref]

    grads, agrads = {}, {}
    for k in range(g.B, 0, -1):
        bop = g.bops[k]
        n = g.nodes[bop.node]
        gy = None if n.persist else agrads[n.id]
        din, dpar = backward(g, bop, bop.impls[0]["algo"], gy, get_any, params, stats)
        for pos, d in din.items():
            j = n.ins[pos]
            if j > 0:
                agrads[j] = agrads[j] + d if j in agrads else d.copy()
        for pid, d in dpar.items():
            grads[pid] = d
    return dict(loss=loss, acts=acts, aux=auxv, grads=grads, agrads=agrads, stats=stats)
