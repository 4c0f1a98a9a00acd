"""Seeded synthetic tensors for a graph, and layout shuffles between the two conventions.

Storage convention (what the graph text declares and the HIP library reads):
activations N,H,W,C, convolution weights K,R,S,C.  The CPU oracle works in
N,C,H,W / K,C,R,S; the helpers below only permute axes.
"""
import numpy as np

from .graphs import Graph


def make_inputs(g: Graph, seed=0, gamma_beta="unit"):
    """(exts {ref: array}, params {pid: array}) in storage convention, fp32 / int32.

    Images ~ N(0,1); labels uniform; conv weights He-normal (std sqrt(2/fan_in), fan_in = C*R*S);
    linear weights N(0, 1/fan_in), bias 0; BatchNorm gamma=1, beta=0 (`unit`) or
    gamma ~ U(0.5,1.5), beta ~ N(0, 0.1^2) (`random`).
    """
    rng = np.random.default_rng(seed)
    exts, params = {}, {}
    classes = None
    for n in g.nodes:
        if n.op == "softmaxce":
            classes = g.shape_of(n.ins[0])[-1]
    for ref, name, dt, shp in g.exts:
        if dt == "f32":
            exts[ref] = rng.standard_normal(shp, dtype=np.float32)
        else:
            exts[ref] = rng.integers(0, classes, size=shp, dtype=np.int32)
    for pid, name, shp in g.params:
        if name.endswith(".gamma"):
            params[pid] = (np.ones(shp, np.float32) if gamma_beta == "unit"
                           else rng.uniform(0.5, 1.5, shp).astype(np.float32))
        elif name.endswith(".beta"):
            params[pid] = (np.zeros(shp, np.float32) if gamma_beta == "unit"
                           else (0.1 * rng.standard_normal(shp)).astype(np.float32))
        elif name.endswith(".b"):
            params[pid] = np.zeros(shp, np.float32)
        elif len(shp) == 4:
            K, R, S, C = shp
            params[pid] = (rng.standard_normal(shp, dtype=np.float32) * np.float32(np.sqrt(2.0 / (C * R * S))))
        else:
            out, inp = shp
            params[pid] = (rng.standard_normal(shp, dtype=np.float32) * np.float32(np.sqrt(1.0 / inp)))
    return exts, params


def act_to_oracle(a):
    """N,H,W,C -> N,C,H,W (float64 for float data); other ranks pass through."""
    a = np.asarray(a)
    if a.ndim == 4:
        a = np.transpose(a, (0, 3, 1, 2))
    return a.astype(np.float64) if a.dtype.kind == "f" else a.copy()


def act_from_oracle(a):
    a = np.asarray(a)
    if a.ndim == 4:
        a = np.transpose(a, (0, 2, 3, 1))
    return np.ascontiguousarray(a)


def weight_to_oracle(w):
    """K,R,S,C -> K,C,R,S; other ranks pass through."""
    w = np.asarray(w)
    if w.ndim == 4:
        w = np.transpose(w, (0, 3, 1, 2))
    return w.astype(np.float64)


def weight_from_oracle(w):
    w = np.asarray(w)
    if w.ndim == 4:
        w = np.transpose(w, (0, 2, 3, 1))
    return np.ascontiguousarray(w)


def oracle_inputs(exts, params):
    return ({r: act_to_oracle(a) for r, a in exts.items()},
            {p: weight_to_oracle(w) for p, w in params.items()})
