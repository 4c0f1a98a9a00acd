"""Forward graphs of the synthetic networks, written as `monet-graph` text.

The text is the forward DAG of the paper's Section 3 (nodes 1..N in
topological order, edges given by each node's `in=` list), extended as its
Appendix D describes: intermediate storage nodes (ReLU sign mask, max-pool
window index) follow their creator, convolution and linear layers own two
backward operators (input-gradient, parameter-gradient), and every forward
and backward operator lists its implementations with workspace bytes, cost
and, for backward ones, the forward tensors they depend on.

Format (one record per line, fields separated by blanks):

    monet-graph 1
    ext   <ref<=0> <name> <f32|i32> <d0xd1x...>        caller-owned tensors
    param <pid> <name> <d0xd1x...>                      fp32 parameters
    node  <i> <op> in=<ref,...> par=<pid,...|-> shape=<dims> [key=value ...]
    fimpl <i> <l> algo=<name> ws=<bytes> cost=<float> [inplace=1] [key=value]
    bop   <k> <kind> node=<i>
    bimpl <k> <l> algo=<name> deps=<ref,...|-> ws=<bytes> cost=<float> [key=value]

Activations are NHWC, convolution weights K,R,S,C, linear weights out,in.
`ref` > 0 names a node's output, `ref` <= 0 an `ext` tensor.  Backward
operators are numbered in forward order of their node (input-gradient before
parameter-gradient), so that running them from the highest number down gives
the parameter gradient first (Appendix D).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

RIDGE_FLOP_PER_BYTE = 20.0  # cost unit: one byte moved counts as 20 flop


def _dims(shape):
    return "x".join(str(int(d)) for d in shape)


def numel(shape):
    n = 1
    for d in shape:
        n *= int(d)
    return n


@dataclass
class Node:
    id: int
    op: str
    ins: list
    pars: list
    shape: tuple
    attrs: dict = field(default_factory=dict)


class Graph:
    AUX_OPS = ("mask", "poolidx")

    def __init__(self):
        self.exts = []      # (ref, name, dtype, shape)
        self.params = []    # (pid, name, shape)
        self.nodes = []     # Node, id = index+1
        self.fimpls = {}    # node id -> [dict]
        self.bops = []      # dict(k, kind, node)
        self.bimpls = {}    # k -> [dict]
        self.blocks = []    # [(name, [node ids])]  (builder-side grouping for schedule helpers)
        self._cur_block = None

    # ---- construction -------------------------------------------------
    def ext(self, name, dtype, shape):
        ref = -len(self.exts)
        self.exts.append((ref, name, dtype, tuple(shape)))
        return ref

    def param(self, name, shape):
        pid = len(self.params)
        self.params.append((pid, name, tuple(shape)))
        return pid

    def shape_of(self, ref):
        if ref <= 0:
            return self.exts[-ref][3]
        return self.nodes[ref - 1].shape

    def begin_block(self, name):
        self._cur_block = (name, [])
        self.blocks.append(self._cur_block)

    def end_block(self):
        self._cur_block = None

    def _add(self, op, ins, pars, shape, **attrs):
        n = Node(len(self.nodes) + 1, op, list(ins), list(pars), tuple(shape), dict(attrs))
        self.nodes.append(n)
        if self._cur_block is not None:
            self._cur_block[1].append(n.id)
        return n.id

    def _bytes(self, ref):
        return 4 * numel(self.shape_of(ref))

    # ---- operators ----------------------------------------------------
    def conv(self, x, K, R, S=None, stride=1, pad=0, name="conv", wgrad_splits=None):
        S = R if S is None else S
        N, H, W, C = self.shape_of(x)
        P = (H + 2 * pad - R) // stride + 1
        Q = (W + 2 * pad - S) // stride + 1
        if wgrad_splits is None:
            wgrad_splits = (wgrad_split_count(N * P * Q, K, C * R * S),)
        w = self.param(name + ".w", (K, R, S, C))
        i = self._add("conv", [x], [w], (N, P, Q, K), R=R, S=S, stride=stride, pad=pad)
        flop = 2.0 * N * P * Q * K * C * R * S
        self.fimpls[i] = [dict(algo="igemm", ws=0, cost=flop)]
        # Layers with few output tiles leave most of the 256 CUs idle: offer a variant that cuts the
        # reduction into `splits` ranges (more workgroups) and pays for it with workspace.
        sp, ws = conv_split_plan(N * P * Q, K, C * R * S)
        if ws:
            self.fimpls[i].append(dict(algo="igemm_splitk", ws=ws, cost=flop * 0.8, splits=sp))
        # Winograd F(2x2, 3x3): 2.25x fewer multiplications for 16 transformed filters, 4x the input and 4x the
        # output as workspace.  Offered where it was measured faster than the implicit GEMM: 3x3 / stride 1 / pad 1
        # with at least 256 channels on both sides (1.4-1.8x), or at least 128 on maps up to 28x28 (1.2-1.5x); at 128
        # channels on large maps it gains 4 % for a workspace of 8x the layer's activations, at 64 it is slower.
        eligible = R == 3 and S == 3 and stride == 1 and pad == 1 and C % 16 == 0 and K % 16 == 0
        wino = eligible and (min(C, K) >= 256 or (min(C, K) >= 128 and H * W <= 28 * 28))
        # F(4x4, 3x3): 4x fewer multiplications, 36 transformed filters, 2.25x the input and 2.25x the output of a
        # chunk of images as workspace.  Measured 1.2-1.4x faster than the implicit GEMM at 64 channels and 2-3x
        # from 128 up (forward and input gradient); the filter gradient gains 1.4-2.5x from 96 channels up and
        # loses at 64.
        wino4 = eligible and min(C, K) >= 64
        wino4_wgrad = wino4 and min(C, K) >= 96
        # F(4x4, 3x3) in one kernel: the transformed input and the products stay on chip, the workspace holds the 36
        # transformed filters only (output channels padded to 64).  It reads the input once per 64 output channels and
        # streams the filters from L2 per 32 tiles, so it wins where maps are large or channels few (measured against the
        # workspace form, forward: x1.9 at 64 channels on 224x224 and 416x608, x1.3-1.5 at 128, x1.1 at 256 on 56x56,
        # level at 28x28x128 and, since the ragged last round of a launch is worked as half items, at 14x14x256, where it also takes the
        # recomputed ReLU and its mask into its epilogue) and loses on small maps with more channels (14x14x512, 7x7x512).  The library
        # addresses the input with 32-bit byte offsets: tensors of 4 GiB and more keep the workspace form.
        wino4f = wino4 and 4 * N * H * W * max(C, K) < (1 << 32) and not (H * W <= 14 * 14 and min(C, K) >= 320)

        # Workspace of the Winograd forms (mirrors the library): the transformed filters, plus the transformed input and
        # the products of one chunk of whole images -- the library works through a layer in chunks of about half a GiB
        # of transformed tensors, which costs 0-2 % of time and caps the workspace of the largest layers at a tenth.
        def wino_chunk(m):
            planes = (m + 2) ** 2
            per_img = planes * math.ceil(H / m) * math.ceil(W / m) * (C + K)
            cap = min(N, max(1, -(-((512 << 20) // 4) // per_img)))
            chunks = -(-N // cap)
            return planes, per_img, -(-N // chunks)          # equal chunks

        def wino_ws(m):
            planes, per_img, imgs = wino_chunk(m)
            return _align(4 * (planes * K * C + imgs * per_img))

        def wino_wgrad_ws(m):      # + the transformed filter gradient, a chunk's share of it, partial sums of its reduction ranges
            planes, per_img, imgs = wino_chunk(m)
            tiles = imgs * math.ceil(H / m) * math.ceil(W / m)
            ranges = max(1, min(1024 // (planes * math.ceil(K / 128) * math.ceil(C / 128)), tiles // 128))
            return _align(4 * (imgs * per_img + planes * K * C * (2 + (ranges if ranges > 1 else 0))))

        if wino:
            self.fimpls[i].append(dict(algo="winograd", ws=wino_ws(2), cost=flop * 0.6))
        if wino4:
            self.fimpls[i].append(dict(algo="winograd4", ws=wino_ws(4), cost=flop * 0.4))
        if wino4f:
            self.fimpls[i].append(dict(algo="winograd4f", ws=_align(4 * 36 * (-(-K // 64) * 64) * C), cost=flop * 0.3))
        # Explicit patch matrix + GEMM (the matrix-multiplication form): patches of a chunk of whole images in the
        # workspace (mirrors the library's recommendation: about 256 MiB of patches per chunk, rows padded to 16
        # floats, a padded filter copy where R*S*C is no multiple of 16).  Offered for every filter larger than 1x1;
        # it moves R*S times the input through memory, so it loses to the implicit GEMM almost everywhere (measured
        # costs decide).  Appended last: implementation indices of schedules written before it existed stay valid.
        im2col = (R * S > 1) and K % 4 == 0
        ld = -(-(C * R * S) // 16) * 16

        def col_imgs():
            cap = max(1, min(N, (256 << 20) // 4 // (P * Q * ld)))
            span = (((1 << 30) - (1 << 18)) // max(ld, K)) // (P * Q)
            cap = min(cap, max(span, 1))
            chunks = -(-N // cap)
            return -(-N // chunks)

        if im2col:
            wpad = K * ld if ld != C * R * S else 0
            self.fimpls[i].append(dict(algo="im2col", ws=_align(4 * (wpad + col_imgs() * P * Q * ld)), cost=flop * 1.5))
        dg = [dict(algo="igemm", deps=[], ws=0, cost=flop)]
        if wino:
            dg.append(dict(algo="winograd", deps=[], ws=wino_ws(2), cost=flop * 0.6))
        if wino4:
            dg.append(dict(algo="winograd4", deps=[], ws=wino_ws(4), cost=flop * 0.4))
        sp, ws = conv_split_plan(N * math.ceil(H / stride) * math.ceil(W / stride), C,
                                 max(1, R // stride) * max(1, S // stride) * K, stride * stride, N * H * W * C)
        if ws:
            dg.append(dict(algo="igemm_splitk", deps=[], ws=ws, cost=flop * 0.8, splits=sp))
        if wino4f:      # appended last: implementation indices of schedules written before this form existed stay valid
            dg.append(dict(algo="winograd4f", deps=[], ws=_align(4 * 36 * (-(-C // 64) * 64) * K), cost=flop * 0.3))
        wbytes = 4 * K * R * S * C
        wg = [dict(algo="direct", ws=0, cost=flop * 4.0)]
        for sp in wgrad_splits:
            wg.append(dict(algo="splitk", ws=_align(sp * wbytes), cost=flop * (1.0 + 0.02 * sp), splits=sp))
        if wino:      # the filter gradient in the same transformed domain (measured 1.2-1.85x where it is offered)
            wg.append(dict(algo="winograd", cost=flop * 0.65, ws=wino_wgrad_ws(2)))
        if wino4_wgrad:
            wg.append(dict(algo="winograd4", cost=flop * 0.45, ws=wino_wgrad_ws(4)))
        if im2col:      # patches of a chunk, the chunk's K x ld result and the parts of its split reduction
            imgs = col_imgs()
            steps = -(-(imgs * P * Q) // 16)
            tiles = -(-K // 128) * -(-ld // 128)
            sp = max(1, min(-(-512 // tiles), steps // 4, 256))
            wg.append(dict(algo="im2col", cost=flop * 1.5, ws=_align(4 * (imgs * P * Q * ld + K * ld * (1 + (sp if sp > 1 else 0))))))
        self._pending_bops(i, [("conv_dgrad", dg)] if x > 0 else [],
                           [("conv_wgrad", [dict(d, deps=[x] if x > 0 else []) for d in wg])])
        return i

    def bn(self, x, name="bn", eps=1e-5):
        shp = self.shape_of(x)
        C = shp[-1]
        g = self.param(name + ".gamma", (C,))
        b = self.param(name + ".beta", (C,))
        i = self._add("bn", [x], [g, b], shp, eps=eps)
        by = self._bytes(i)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="oop", ws=0, cost=3 * by * c),
                          dict(algo="inplace", ws=0, cost=3 * by * c, inplace=1)]
        self._pending_bops(i, [("bn_bwd", [dict(algo="from_input", deps=[x] if x > 0 else [], ws=0, cost=5 * by * c),
                                            dict(algo="from_output", deps=[i], ws=0, cost=5 * by * c)])])
        return i

    def relu(self, x, six=False):
        shp = self.shape_of(x)
        op = "relu6" if six else "relu"
        i = self._add(op, [x], [], shp)
        words = (numel(shp) + 63) // 64
        m = self._add("mask", [i], [], (words,))
        by = self._bytes(i)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="oop", ws=0, cost=2 * by * c),
                          dict(algo="inplace", ws=0, cost=2 * by * c, inplace=1)]
        self._pending_bops(i, [(op + "_bwd", [dict(algo="from_input", deps=[x] if x > 0 else [], ws=0, cost=3 * by * c),
                                               dict(algo="from_output", deps=[i], ws=0, cost=3 * by * c),
                                               dict(algo="from_mask", deps=[m], ws=0, cost=(2 + 1 / 32) * by * c)])])
        return i

    def maxpool(self, x, k, stride, pad=0):
        N, H, W, C = self.shape_of(x)
        P = (H + 2 * pad - k) // stride + 1
        Q = (W + 2 * pad - k) // stride + 1
        i = self._add("maxpool", [x], [], (N, P, Q, C), k=k, stride=stride, pad=pad)
        ix = self._add("poolidx", [i], [], (N, P, Q, C))
        bi, bo = self._bytes(x), self._bytes(i)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="direct", ws=0, cost=(bi + bo) * c)]
        self._pending_bops(i, [("maxpool_bwd", [dict(algo="from_input", deps=[x] if x > 0 else [], ws=0, cost=(2 * bi + bo) * c),
                                                 dict(algo="from_index", deps=[ix], ws=0, cost=(bi + 1.25 * bo) * c)])])
        return i

    def add(self, a, b):
        shp = self.shape_of(a)
        assert shp == self.shape_of(b)
        i = self._add("add", [a, b], [], shp)
        by = self._bytes(i)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="oop", ws=0, cost=3 * by * c)]
        self._pending_bops(i, [("add_bwd", [dict(algo="copy", deps=[], ws=0, cost=4 * by * c)])])
        return i

    def avgpool(self, x):
        N, H, W, C = self.shape_of(x)
        i = self._add("avgpool", [x], [], (N, C))
        by = self._bytes(x)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="direct", ws=0, cost=by * c)]
        self._pending_bops(i, [("avgpool_bwd", [dict(algo="direct", deps=[], ws=0, cost=by * c)])])
        return i

    def concat(self, a, b):
        """Channel concatenation (last storage axis)."""
        sa, sb = self.shape_of(a), self.shape_of(b)
        assert sa[:-1] == sb[:-1]
        i = self._add("concat", [a, b], [], sa[:-1] + (sa[-1] + sb[-1],))
        by = self._bytes(i)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="copy", ws=0, cost=2 * by * c)]
        self._pending_bops(i, [("concat_bwd", [dict(algo="copy", deps=[], ws=0, cost=2 * by * c)])])
        return i

    def tconv(self, x, K, R=2, stride=2, name="tconv"):
        """Transposed convolution without padding; weights C_in,R,S,C_out (the K,R,S,C filter of the
        convolution it is the adjoint of)."""
        N, H, W, C = self.shape_of(x)
        P, Q = (H - 1) * stride + R, (W - 1) * stride + R
        w = self.param(name + ".w", (C, R, R, K))
        i = self._add("tconv", [x], [w], (N, P, Q, K), R=R, S=R, stride=stride)
        flop = 2.0 * N * H * W * K * C * R * R
        self.fimpls[i] = [dict(algo="igemm", ws=0, cost=flop)]
        wbytes = 4 * K * R * R * C
        sp = wgrad_split_count(N * H * W, C, K * R * R)
        wg = [dict(algo="direct", ws=0, cost=flop * 4.0),
              dict(algo="splitk", ws=_align(sp * wbytes), cost=flop * (1.0 + 0.02 * sp), splits=sp)]
        self._pending_bops(i, [("tconv_dgrad", [dict(algo="igemm", deps=[], ws=0, cost=flop)])] if x > 0 else [],
                           [("tconv_wgrad", [dict(d, deps=[x] if x > 0 else []) for d in wg])])
        return i

    def dwconv(self, x, R=3, stride=1, pad=1, name="dw"):
        """Depthwise convolution: one R x R filter per channel; weights C,R,S,1."""
        N, H, W, C = self.shape_of(x)
        P = (H + 2 * pad - R) // stride + 1
        Q = (W + 2 * pad - R) // stride + 1
        w = self.param(name + ".w", (C, R, R, 1))
        i = self._add("dwconv", [x], [w], (N, P, Q, C), R=R, S=R, stride=stride, pad=pad)
        bi, bo = self._bytes(x), self._bytes(i)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="direct", ws=0, cost=(bi + bo) * c)]
        self._pending_bops(i, [("dwconv_dgrad", [dict(algo="direct", deps=[], ws=0, cost=(bi + bo) * c)])] if x > 0 else [],
                           [("dwconv_wgrad", [dict(algo="direct", deps=[x] if x > 0 else [], ws=0, cost=(bi + bo) * c)])])
        return i

    def linear(self, x, out, name="fc"):
        """Fully connected layer over the flattened input; a 4-D input N,H,W,C gets weights out,H,W,C."""
        shp = self.shape_of(x)
        N, I = shp[0], numel(shp[1:])
        w = self.param(name + ".w", (out,) + tuple(shp[1:]))
        b = self.param(name + ".b", (out,))
        i = self._add("linear", [x], [w, b], (N, out))
        flop = 2.0 * N * I * out
        self.fimpls[i] = [dict(algo="gemm", ws=0, cost=flop)]
        self._pending_bops(i, [("linear_dgrad", [dict(algo="gemm", deps=[], ws=0, cost=flop)])] if x > 0 else [],
                           [("linear_wgrad", [dict(algo="gemm", deps=[x] if x > 0 else [], ws=0, cost=flop)])])
        return i

    def softmaxce(self, x, labels):
        i = self._add("softmaxce", [x, labels], [], (1,), persist=1)
        by = self._bytes(x)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="direct", ws=0, cost=by * c)]
        self._pending_bops(i, [("softmaxce_bwd", [dict(algo="direct", deps=[x], ws=0, cost=2 * by * c)])])
        return i

    def sumloss(self, x):
        i = self._add("sumloss", [x], [], (1,), persist=1)
        by = self._bytes(x)
        c = RIDGE_FLOP_PER_BYTE
        self.fimpls[i] = [dict(algo="direct", ws=0, cost=by * c)]
        self._pending_bops(i, [("sumloss_bwd", [dict(algo="fill", deps=[], ws=0, cost=by * c)])])
        return i

    def _pending_bops(self, node, *groups):
        for grp in groups:
            for kind, impls in grp:
                k = len(self.bops) + 1
                self.bops.append(dict(k=k, kind=kind, node=node))
                self.bimpls[k] = impls

    # ---- lookups used by schedule helpers -----------------------------
    def is_aux(self, i):
        return self.nodes[i - 1].op in self.AUX_OPS

    def aux_of(self, i):
        """Aux node created by node i, or 0."""
        if i < len(self.nodes) and self.nodes[i].op in self.AUX_OPS and self.nodes[i].ins == [i]:
            return i + 1
        return 0

    def bops_of(self, node):
        return [b for b in self.bops if b["node"] == node]

    def fimpl_index(self, i, algo):
        for l, d in enumerate(self.fimpls.get(i, [])):
            if d["algo"] == algo:
                return l
        raise KeyError((i, algo))

    def bimpl_index(self, k, algo, **match):
        for l, d in enumerate(self.bimpls[k]):
            if d["algo"] == algo and all(d.get(a) == v for a, v in match.items()):
                return l
        raise KeyError((k, algo, match))

    # ---- text ---------------------------------------------------------
    def text(self):
        out = ["monet-graph 1"]
        for ref, name, dt, shp in self.exts:
            out.append(f"ext {ref} {name} {dt} {_dims(shp)}")
        for pid, name, shp in self.params:
            out.append(f"param {pid} {name} {_dims(shp)}")
        for n in self.nodes:
            ins = ",".join(str(r) for r in n.ins)
            par = ",".join(str(p) for p in n.pars) if n.pars else "-"
            rec = f"node {n.id} {n.op} in={ins} par={par} shape={_dims(n.shape)}"
            for k, v in n.attrs.items():
                rec += f" {k}={v!r}" if isinstance(v, float) else f" {k}={v}"
            out.append(rec)
        for i in sorted(self.fimpls):
            for l, d in enumerate(self.fimpls[i]):
                rec = f"fimpl {i} {l} algo={d['algo']} ws={int(d['ws'])} cost={float(d['cost'])!r}"
                for k, v in d.items():
                    if k not in ("algo", "ws", "cost"):
                        rec += f" {k}={v}"
                out.append(rec)
        for b in self.bops:
            out.append(f"bop {b['k']} {b['kind']} node={b['node']}")
        for k in sorted(self.bimpls):
            for l, d in enumerate(self.bimpls[k]):
                deps = ",".join(str(r) for r in d["deps"]) if d["deps"] else "-"
                rec = f"bimpl {k} {l} algo={d['algo']} deps={deps} ws={int(d['ws'])} cost={float(d['cost'])!r}"
                for kk, v in d.items():
                    if kk not in ("algo", "ws", "cost", "deps"):
                        rec += f" {kk}={v}"
                out.append(rec)
        return "\n".join(out) + "\n"


def conv_split_plan(rows, cols, reduction, classes=1, out_elems=None):
    """(splits, workspace bytes) of the reduction-split variant of a forward / input-gradient GEMM with a
    rows x cols result per residue class (`classes` = stride^2 and `out_elems` = |dx| for the input gradient),
    or (1, 0) where the plain variant is as fast.

    The kernel library works on 128x128 tiles (256x64 for results up to 64 columns wide), one workgroup per
    tile and reduction range, and a CU's time grows with the number of workgroups it is handed: a launch costs
    ceil(workgroups / 256) rounds.  Rules read off a sweep over the ResNet-50 b184 layers:
      * fewer than two tiles per CU (or fewer than eight with stride > 1): cut every tile into the number of
        ranges s (at most 16, at least 128 reduction elements each) that minimises rounds / s, with 1 % per range
        for the slabs of partial results a second kernel adds;
      * otherwise, stride 1, at least 48 reduction steps of 16: `splits` stays 1 and a workspace lets the library
        cut only the tiles beyond a multiple of 256, into as many ranges as keep them within one round (their
        parts are added inside the kernel; with a short reduction the device-wide release this needs costs
        more than the idle CUs);
      * otherwise: plain."""
    bm, bn = (256, 64) if cols <= 64 else (128, 128)
    tiles = math.ceil(rows / bm) * math.ceil(cols / bn)
    steps = math.ceil(reduction / 16)
    items = tiles * classes
    out_elems = rows * cols * classes if out_elems is None else out_elems
    if items < (512 if classes == 1 else 2048):
        best, best_cost = 1, None
        for s in range(1, max(1, min(16, reduction // 128)) + 1):
            cost = math.ceil(items * s / 256) / s * (1 + 0.01 * s)
            if best_cost is None or cost < best_cost - 1e-9:
                best, best_cost = s, cost
        return (best, _align(best * 4 * out_elems)) if best > 1 else (1, 0)
    tail = tiles % 256
    if classes == 1 and tail and steps >= 48:
        s = min(256 // tail, steps // 4, 16)
        if s >= 2:
            return 1, _align(s * tail * 4 * bm * bn)
    return 1, 0


def wgrad_split_count(M, K, cols):
    """Reduction splits of a K x cols weight-gradient GEMM that sums over M output positions:
    enough waves to keep loads in flight on 256 CUs (about 16 per CU), at least 8 reduction steps
    of 16 rows per split, and at most 128 MiB of partial sums.  The tile shape follows the kernel
    library's choice for that GEMM."""
    if K <= 64:
        tile_rows, tile_cols, waves = (64, 256, 4) if cols % 256 == 0 else (64, 64, 1)
    elif cols <= 64:
        tile_rows, tile_cols, waves = (256, 64, 4) if K >= 256 else (128, 64, 2)
    else:
        tile_rows, tile_cols, waves = (128, 128, 4)
    tiles = math.ceil(K / tile_rows) * math.ceil(cols / tile_cols)
    # a CU's time grows with the number of workgroups it is handed, so the total stays at or just under a
    # whole number of workgroups per CU (1024 four-wave workgroups = 4 per CU): one workgroup over costs a full round
    sp = max(1, 4096 // (tiles * waves))
    return max(1, min(sp, M // 128, (128 << 20) // (4 * K * cols)))


def _align(b, a=256):
    return (int(b) + a - 1) // a * a


# ----------------------------------------------------------------------
# networks
# ----------------------------------------------------------------------
def tiny_chain(batch=2, hw=16, channels=16, blocks=4, wgrad_splits=(4,)):
    """Chain of conv3x3(s1,p1)-BN-ReLU blocks with a sum-of-outputs loss."""
    g = Graph()
    x = g.ext("x", "f32", (batch, hw, hw, channels))
    a = x
    for b in range(blocks):
        g.begin_block(f"b{b}")
        c = g.conv(a, channels, 3, stride=1, pad=1, name=f"conv{b}", wgrad_splits=wgrad_splits)
        n = g.bn(c, name=f"bn{b}")
        a = g.relu(n)
        g.end_block()
    g.sumloss(a)
    return g


def resnet50(batch=184, hw=224, classes=1000, widths=(64, 128, 256, 512), depths=(3, 4, 6, 3), stem=64,
             wgrad_splits=None):
    """Bottleneck ResNet (v1.5: stride on the 3x3), softmax cross-entropy loss."""
    g = Graph()
    x = g.ext("x", "f32", (batch, hw, hw, 3))
    labels = g.ext("labels", "i32", (batch,))

    def cbr(a, K, R, stride, pad, name, relu=True):
        c = g.conv(a, K, R, stride=stride, pad=pad, name=name, wgrad_splits=wgrad_splits)
        n = g.bn(c, name=name.replace("conv", "bn"))
        return g.relu(n) if relu else n

    g.begin_block("stem")
    a = cbr(x, stem, 7, 2, 3, "stem.conv")
    a = g.maxpool(a, 3, 2, 1)
    g.end_block()
    for si, (wd, dp) in enumerate(zip(widths, depths)):
        for bi in range(dp):
            stride = 2 if (bi == 0 and si > 0) else 1
            g.begin_block(f"l{si + 1}b{bi}")
            nm = f"l{si + 1}b{bi}"
            h = cbr(a, wd, 1, 1, 0, nm + ".conv1")
            h = cbr(h, wd, 3, stride, 1, nm + ".conv2")
            h = cbr(h, wd * 4, 1, 1, 0, nm + ".conv3", relu=False)
            if bi == 0:
                sk = cbr(a, wd * 4, 1, stride, 0, nm + ".convd", relu=False)
            else:
                sk = a
            s = g.add(h, sk)
            a = g.relu(s)
            g.end_block()
    g.begin_block("head")
    p = g.avgpool(a)
    f = g.linear(p, classes, name="fc")
    g.softmaxce(f, labels)
    g.end_block()
    return g


def _cbr(g, a, K, R, stride, pad, name, six=False):
    c = g.conv(a, K, R, stride=stride, pad=pad, name=name + ".conv")
    n = g.bn(c, name=name + ".bn")
    return g.relu(n, six=six)


def vgg16_bn(batch=176, hw=224, classes=1000, widths=(64, 128, 256, 512, 512), convs=(2, 2, 3, 3, 3), fc=4096):
    """VGG-16 with BatchNorm: 13 conv3x3-BN-ReLU triples in five stages, each closed by a 2x2
    max-pool, then three fully connected layers (no dropout).  One block per triple; the pool
    joins the last triple of its stage."""
    g = Graph()
    x = g.ext("x", "f32", (batch, hw, hw, 3))
    labels = g.ext("labels", "i32", (batch,))
    a = x
    for si, (wd, cnt) in enumerate(zip(widths, convs)):
        for ci in range(cnt):
            g.begin_block(f"s{si + 1}c{ci}")
            a = _cbr(g, a, wd, 3, 1, 1, f"s{si + 1}c{ci}")
            if ci == cnt - 1:
                a = g.maxpool(a, 2, 2, 0)
            g.end_block()
    g.begin_block("fc1")
    a = g.relu(g.linear(a, fc, name="fc1"))
    g.end_block()
    g.begin_block("fc2")
    a = g.relu(g.linear(a, fc, name="fc2"))
    g.end_block()
    g.begin_block("head")
    f = g.linear(a, classes, name="fc3")
    g.softmaxce(f, labels)
    g.end_block()
    return g


def unet(batch=11, h=416, w=608, classes=2, base=64, depth=4):
    """Encoder-decoder with skip connections: `depth` levels of two conv3x3-BN-ReLU triples and a
    2x2 max-pool, a bottleneck, then per level a 2x2 stride-2 transposed convolution, channel
    concatenation with the skip tensor and two more triples; a 1x1 convolution gives per-pixel
    class scores for a cross-entropy averaged over batch and pixels.  One block per level."""
    assert h % (1 << depth) == 0 and w % (1 << depth) == 0
    g = Graph()
    x = g.ext("x", "f32", (batch, h, w, 3))
    labels = g.ext("labels", "i32", (batch, h, w))
    a = x
    skips = []
    for d in range(depth):
        wd = base << d
        g.begin_block(f"down{d}")
        a = _cbr(g, a, wd, 3, 1, 1, f"down{d}a")
        a = _cbr(g, a, wd, 3, 1, 1, f"down{d}b")
        g.end_block()
        skips.append(a)
        g.begin_block(f"pool{d}")
        a = g.maxpool(a, 2, 2, 0)
        g.end_block()
    g.begin_block("mid")
    a = _cbr(g, a, base << depth, 3, 1, 1, "mida")
    a = _cbr(g, a, base << depth, 3, 1, 1, "midb")
    g.end_block()
    for d in reversed(range(depth)):
        wd = base << d
        g.begin_block(f"up{d}")
        u = g.tconv(a, wd, 2, 2, name=f"up{d}.tconv")
        a = g.concat(skips[d], u)
        a = _cbr(g, a, wd, 3, 1, 1, f"up{d}a")
        a = _cbr(g, a, wd, 3, 1, 1, f"up{d}b")
        g.end_block()
    g.begin_block("head")
    f = g.conv(a, classes, 1, stride=1, pad=0, name="out.conv")
    g.softmaxce(f, labels)
    g.end_block()
    return g


MOBILENET_V2_STAGES = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1))


def mobilenet_v2(batch=272, hw=224, classes=1000, stages=MOBILENET_V2_STAGES, stem=32, last=1280):
    """Inverted-residual network: per block a 1x1 expansion (factor t), a depthwise 3x3 and a linear
    1x1 projection, each followed by BatchNorm, ReLU6 after the first two; identity skip when the
    block keeps shape.  `stages` rows are (t, channels, repeats, stride of the first repeat).
    Blocks are the triples, so that a schedule can recompute the depthwise ones."""
    g = Graph()
    x = g.ext("x", "f32", (batch, hw, hw, 3))
    labels = g.ext("labels", "i32", (batch,))
    g.begin_block("stem")
    a = _cbr(g, x, stem, 3, 2, 1, "stem", six=True)
    g.end_block()
    cin = stem
    bi = 0
    for t, cout, reps, stride0 in stages:
        for r in range(reps):
            stride = stride0 if r == 0 else 1
            nm = f"b{bi}"
            h = a
            if t != 1:
                g.begin_block(nm + ".expand")
                h = _cbr(g, h, cin * t, 1, 1, 0, nm + ".expand", six=True)
                g.end_block()
            g.begin_block(nm + ".dw")
            d = g.dwconv(h, 3, stride, 1, name=nm + ".dw")
            h = g.relu(g.bn(d, name=nm + ".dw.bn"), six=True)
            g.end_block()
            g.begin_block(nm + ".project")
            p = g.conv(h, cout, 1, stride=1, pad=0, name=nm + ".project.conv")
            h = g.bn(p, name=nm + ".project.bn")
            if stride == 1 and cin == cout:
                h = g.add(h, a)
            g.end_block()
            a = h
            cin = cout
            bi += 1
    g.begin_block("last")
    a = _cbr(g, a, last, 1, 1, 0, "last", six=True)
    g.end_block()
    g.begin_block("head")
    p = g.avgpool(a)
    f = g.linear(p, classes, name="fc")
    g.softmaxce(f, labels)
    g.end_block()
    return g


# (1x1, (3x3 reduce, 3x3), (5x5 reduce, 5x5), pool projection) per inception module, and where the 3x3 / stride-2
# max-pools sit (after 3b and 4e): the published table of the architecture
GOOGLENET_INCEPTIONS = (
    ("3a", 64, (96, 128), (16, 32), 32), ("3b", 128, (128, 192), (32, 96), 64), "pool",
    ("4a", 192, (96, 208), (16, 48), 64), ("4b", 160, (112, 224), (24, 64), 64), ("4c", 128, (128, 256), (24, 64), 64),
    ("4d", 112, (144, 288), (32, 64), 64), ("4e", 256, (160, 320), (32, 128), 128), "pool",
    ("5a", 256, (160, 320), (32, 128), 128), ("5b", 384, (192, 384), (48, 128), 128),
)


def googlenet(batch=320, hw=224, classes=1000, stem=(64, 64, 192), inceptions=GOOGLENET_INCEPTIONS):
    """Inception network with BatchNorm after every convolution (no auxiliary classifiers, no dropout):
    conv7x7/2 - pool - conv1x1 - conv3x3 - pool, then inception modules of four parallel branches
    (1x1 | 1x1-3x3 | 1x1-5x5 | pool3x3/1-1x1) joined along the channels, stride-2 pools between the groups,
    global average pool and one linear layer.  One block per stem stage and per module; the four branch outputs
    are joined pairwise, so every element is copied twice on the way into the module output."""
    g = Graph()
    x = g.ext("x", "f32", (batch, hw, hw, 3))
    labels = g.ext("labels", "i32", (batch,))
    g.begin_block("stem1")
    a = g.maxpool(_cbr(g, x, stem[0], 7, 2, 3, "conv1"), 3, 2, 1)
    g.end_block()
    g.begin_block("stem2")
    a = _cbr(g, a, stem[1], 1, 1, 0, "conv2")
    g.end_block()
    g.begin_block("stem3")
    a = g.maxpool(_cbr(g, a, stem[2], 3, 1, 1, "conv3"), 3, 2, 1)
    g.end_block()
    pending_pool = False
    for spec in inceptions:
        if spec == "pool":
            pending_pool = True
            continue
        nm, c1, (r3, c3), (r5, c5), cp = spec
        g.begin_block("inc" + nm)
        if pending_pool:                      # the pool between two groups opens the next module's block
            a = g.maxpool(a, 3, 2, 1)
            pending_pool = False
        b1 = _cbr(g, a, c1, 1, 1, 0, nm + ".b1")
        b2 = _cbr(g, _cbr(g, a, r3, 1, 1, 0, nm + ".b2r"), c3, 3, 1, 1, nm + ".b2")
        b3 = _cbr(g, _cbr(g, a, r5, 1, 1, 0, nm + ".b3r"), c5, 5, 1, 2, nm + ".b3")
        b4 = _cbr(g, g.maxpool(a, 3, 1, 1), cp, 1, 1, 0, nm + ".b4")
        a = g.concat(g.concat(b1, b2), g.concat(b3, b4))
        g.end_block()
    g.begin_block("head")
    p = g.avgpool(a)
    f = g.linear(p, classes, name="fc")
    g.softmaxce(f, labels)
    g.end_block()
    return g
