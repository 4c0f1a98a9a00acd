"""Schedules as `monet-schedule` text, and helpers that write them.

A schedule is the paper's solver output (Appendix A, "Solver variables"):
s^N_i, s^{k-1}_i, r^k_i, the implementation selectors delta_{i,l},
delta^k_{i,l}, delta-hat_{k,l}; an in-place forward implementation stands for
the paper's q variable (Appendix C.3).  Stage k is backward operator k of the
graph text, run from the highest k down; the forward pass is written `fwd`.

Format:

    monet-schedule 1
    fwd <i> impl=<l> save=<0|1>        every node; aux nodes carry impl=-1
    stage <k> impl=<l>                  every backward operator
    r <k> <i> impl=<l>                  r^k_i = 1 (aux nodes: impl=-1)
    s <k> <i>                           s^{k-1}_i = 1

The integer program that chooses these bits lives in `ilp.py` (small graphs);
`expand` is a fixed policy for everything else: given the set F of tensors kept by the
forward pass and one backward implementation per operator, it recomputes a
missing dependency from the nearest tensors still held, and keeps every
tensor exactly until its last use (each tensor is recomputed at most once).
The result is an ordinary schedule; the executor and the oracle validate it
like any other.
"""
from __future__ import annotations

from .graphs import Graph

# A tuple names implementations in order of preference: the first one the operator offers is taken (the graph
# offers the workspace-hungry convolution variants only where they were measured to pay).
DEFAULT_VARIANTS = dict(
    bn_bwd="from_output", relu_bwd="from_mask", relu6_bwd="from_mask", maxpool_bwd="from_index",
    conv_wgrad=("winograd4", "winograd", "splitk"), tconv_wgrad="splitk", conv_dgrad=("winograd4f", "winograd4", "winograd", "igemm_splitk"),
    conv_fwd=("winograd4f", "winograd4", "winograd", "igemm_splitk"), inplace=True,
)
# the same without the Winograd form: every convolution on the implicit GEMM
IGEMM_VARIANTS = dict(DEFAULT_VARIANTS, conv_wgrad="splitk", conv_dgrad="igemm_splitk", conv_fwd="igemm_splitk")
# Winograd through the workspace only (transformed tensors in memory), as before the one-kernel form existed
WINOGRAD_WS_VARIANTS = dict(DEFAULT_VARIANTS, conv_dgrad=("winograd4", "winograd", "igemm_splitk"), conv_fwd=("winograd4", "winograd", "igemm_splitk"))
# Winograd with 2x2 output tiles where it is offered (the 4x4 form is faster and smaller wherever both are)
WINOGRAD2_VARIANTS = dict(DEFAULT_VARIANTS, conv_wgrad=("winograd", "splitk"), conv_dgrad=("winograd", "igemm_splitk"),
                          conv_fwd=("winograd", "igemm_splitk"))
# every convolution with a filter larger than 1x1 through the explicit patch matrix (forward and filter gradient)
IM2COL_VARIANTS = dict(DEFAULT_VARIANTS, conv_wgrad=("im2col", "splitk"), conv_fwd=("im2col", "igemm_splitk"))
STANDARD_VARIANTS = dict(
    bn_bwd="from_input", relu_bwd="from_output", relu6_bwd="from_output", maxpool_bwd="from_input",
    conv_wgrad=("winograd4", "winograd", "splitk"), tconv_wgrad="splitk", conv_dgrad=("winograd4f", "winograd4", "winograd", "igemm_splitk"),
    conv_fwd=("winograd4f", "winograd4", "winograd", "igemm_splitk"), inplace=False,
)


class Schedule:
    def __init__(self, n_nodes, n_bops):
        self.N, self.B = n_nodes, n_bops
        self.fwd_impl = {}                                   # node -> l (aux: -1)
        self.fwd_save = set()                                # s^N
        self.stage_impl = {}                                 # k -> l
        self.r = {k: {} for k in range(1, n_bops + 1)}       # k -> {node: l}
        self.s = {k: set() for k in range(1, n_bops + 1)}    # k -> {node}: s^{k-1}

    def text(self):
        out = ["monet-schedule 1"]
        for i in range(1, self.N + 1):
            out.append(f"fwd {i} impl={self.fwd_impl[i]} save={1 if i in self.fwd_save else 0}")
        for k in range(self.B, 0, -1):
            out.append(f"stage {k} impl={self.stage_impl[k]}")
            for i in sorted(self.r[k]):
                out.append(f"r {k} {i} impl={self.r[k][i]}")
            for i in sorted(self.s[k]):
                out.append(f"s {k} {i}")
        return "\n".join(out) + "\n"


class StoredSchedule:
    """A schedule kept as the text the executor reads (e.g. one a solver run wrote to a file)."""

    def __init__(self, text):
        self._text = text

    def text(self):
        return self._text


def choose_bimpls(g: Graph, variants, saved=None):
    """One implementation index per backward operator, from per-kind names.

    `variants[kind]` is an algo name, or a dict {node: algo, None: default}.
    When `saved` is given, a ReLU whose output is kept anyway but whose mask is
    not uses its output (no extra tensor needed).
    """
    out = {}
    for b in g.bops:
        k, kind, node = b["k"], b["kind"], b["node"]
        want = variants.get(kind)
        if isinstance(want, dict):
            want = want.get(node, want.get(None))
        impls = g.bimpls[k]
        l = 0
        for name in ((want,) if isinstance(want, str) else (want or ())):
            found = [j for j, d in enumerate(impls) if d["algo"] == name]
            if found:
                l = found[0]
                break
        if saved is not None and kind in ("relu_bwd", "relu6_bwd"):
            aux = g.aux_of(node)
            if impls[l]["algo"] == "from_mask" and node in saved and aux not in saved:
                l = g.bimpl_index(k, "from_output")
        out[k] = l
    return out


def deps_of(g: Graph, k, l):
    return [d for d in g.bimpls[k][l]["deps"] if d > 0]


def residual_tail_stages(g: Graph):
    """{k of a ReLU backward: k of the BatchNorm backward two stages later} for block tails
    BatchNorm -> add -> ReLU, whose backward operators run back to back (k, k-1, k-2)."""
    out = {}
    for b in g.bops:
        k = b["k"]
        if b["kind"] not in ("relu_bwd", "relu6_bwd") or k < 3:
            continue
        relu = g.nodes[b["node"] - 1]
        b1, b2 = g.bops[k - 2], g.bops[k - 3]          # stages k-1 and k-2
        if b1["kind"] != "add_bwd" or b1["node"] != relu.ins[0] or b2["kind"] != "bn_bwd":
            continue
        if b2["node"] in g.nodes[b1["node"] - 1].ins:
            out[k] = k - 2
    return out


def expand(g: Graph, F, bimpl, allow_inplace=True, conv_algo="igemm_splitk", hoist_residual_tail=False):
    """Schedule for forward-saved set F (node ids) and backward impl choice {k: l}.

    With `hoist_residual_tail`, what the BatchNorm backward at the tail of a residual block needs is already
    recomputed in the stage of the block's final ReLU backward, two stages earlier: the three backward
    operators then run back to back (and can share a kernel) instead of having the recomputation between them."""
    N, B = len(g.nodes), len(g.bops)
    sch = Schedule(N, B)
    F = set(F)
    sch.stage_impl = dict(bimpl)
    persist = {n.id for n in g.nodes if n.attrs.get("persist")}
    consumers = {i: [] for i in range(1, N + 1)}
    for n in g.nodes:
        if g.is_aux(n.id):
            continue
        for j in n.ins:
            if j > 0:
                consumers[j].append(n.id)

    def pick_fimpl(i, inplace):
        n = g.nodes[i - 1]
        if n.op == "conv":
            for name in ((conv_algo,) if isinstance(conv_algo, str) else conv_algo):
                try:
                    return g.fimpl_index(i, name)
                except KeyError:        # a preferred variant is only offered where it pays
                    continue
            return 0
        if inplace:
            return g.fimpl_index(i, "inplace")
        return 0

    def can_inplace(i):
        return any(d.get("inplace") for d in g.fimpls.get(i, []))

    # ---- forward pass ------------------------------------------------
    for n in g.nodes:
        i = n.id
        if g.is_aux(i):
            sch.fwd_impl[i] = -1
            continue
        j = n.ins[0]
        ip = (allow_inplace and can_inplace(i) and j > 0 and j not in F and not g.is_aux(j)
              and consumers[j] == [i])
        sch.fwd_impl[i] = pick_fimpl(i, ip)
    sch.fwd_save = set(F)

    # ---- phase A: what is recomputed where, and when each tensor is used
    present = set(F)
    born = {j: B + 1 for j in F}        # stage at which the tensor came to exist
    last_use = {}                        # tensor -> lowest stage that reads it
    recomputed = {}                      # k -> sorted list of nodes
    dep_stages = {}                      # tensor -> stages whose backward operator reads it
    for k in range(1, B + 1):
        for d in deps_of(g, k, bimpl[k]):
            dep_stages.setdefault(d, []).append(k)
    hoisted = residual_tail_stages(g) if hoist_residual_tail else {}
    for k in range(B, 0, -1):
        need = deps_of(g, k, bimpl[k])
        early = deps_of(g, hoisted[k], bimpl[hoisted[k]]) if k in hoisted else []
        todo = set()

        def want(t):
            if t in present or t in todo:
                return
            if t in persist:
                raise ValueError(f"persistent node {t} cannot be a dependency")
            todo.add(t)
            n = g.nodes[t - 1]
            if g.is_aux(t):
                c = n.ins[0]
                if c in present:
                    raise ValueError(
                        f"aux node {t} is missing at stage {k} but its creator {c} is held: "
                        f"save the aux node too or pick an implementation that reads the output")
                want(c)
                return
            for j in n.ins:
                if j > 0:
                    if j in present:
                        last_use[j] = k
                    else:
                        want(j)
            # an aux tensor can only be written while its creator runs: emit it now
            # if this or a later stage reads it
            a = g.aux_of(t)
            if a and a not in present and any(kk <= k for kk in dep_stages.get(a, [])):
                todo.add(a)

        for t in need:
            want(t)
        for t in need:
            last_use[t] = k
        for t in early:
            want(t)
        for t in early:
            last_use[t] = hoisted[k]
        for t in todo:
            born[t] = k
        present |= todo
        recomputed[k] = sorted(todo)

    # ---- phase B: s bits = held until last use; in-place where nothing reads the input again
    for k in range(B, 0, -1):
        for j in born:
            if born[j] >= k and j in last_use:
                lu = last_use[j]
                if lu < k or (lu == k and born[j] != k):
                    sch.s[k].add(j)
    for k in range(B, 0, -1):
        R = set(recomputed[k])
        D = set(deps_of(g, k, bimpl[k]))
        for i in recomputed[k]:
            if g.is_aux(i):
                sch.r[k][i] = -1
                continue
            n = g.nodes[i - 1]
            j = n.ins[0]
            ip = (allow_inplace and can_inplace(i) and j > 0 and j in R and not g.is_aux(j)
                  and j not in sch.s[k] and j not in D
                  and not any(t in R and t != i for t in consumers[j]))
            sch.r[k][i] = pick_fimpl(i, ip)
    return sch


# ----------------------------------------------------------------------
# forward-saved sets
# ----------------------------------------------------------------------
def store_everything_set(g: Graph, bimpl):
    """Every forward tensor some backward operator reads: no recomputation."""
    F = set()
    for b in g.bops:
        F.update(deps_of(g, b["k"], bimpl[b["k"]]))
    return F


def block_checkpoint_set(g: Graph, bimpl, checkpoint_blocks):
    """Segment rule on `g.blocks`: a checkpointed block keeps its output and those
    of its own tensors that its backward operators read; other blocks keep nothing."""
    F = set()
    for bi, (_, nodes) in enumerate(g.blocks):
        if bi not in checkpoint_blocks:
            continue
        own = set(nodes)
        for i in nodes:
            for b in g.bops_of(i):
                for d in deps_of(g, b["k"], bimpl[b["k"]]):
                    if d in own:
                        F.add(d)
        main = [i for i in nodes if not g.is_aux(i) and not g.nodes[i - 1].attrs.get("persist")]
        if main:
            F.add(main[-1])
    # an intermediate tensor is written while its creator runs: keep it with a kept creator
    for b in g.bops:
        for d in deps_of(g, b["k"], bimpl[b["k"]]):
            if g.is_aux(d) and g.nodes[d - 1].ins[0] in F:
                F.add(d)
    return F


def block_output_set(g: Graph, blocks=None):
    """Outputs of the named blocks (all blocks when None)."""
    F = set()
    for bi, (_, nodes) in enumerate(g.blocks):
        if blocks is not None and bi not in blocks:
            continue
        main = [i for i in nodes if not g.is_aux(i) and not g.nodes[i - 1].attrs.get("persist")]
        if main:
            F.add(main[-1])
    return F


def tiny_chain_schedule(g: Graph, checkpoint_blocks, variants=None):
    variants = DEFAULT_VARIANTS if variants is None else variants
    bimpl = choose_bimpls(g, variants)
    F = block_checkpoint_set(g, bimpl, set(checkpoint_blocks))
    return expand(g, F, bimpl, allow_inplace=variants.get("inplace", True), conv_algo=variants.get("conv_fwd", "igemm"))


def store_everything_schedule(g: Graph, variants=None):
    variants = STANDARD_VARIANTS if variants is None else variants
    bimpl = choose_bimpls(g, variants)
    return expand(g, store_everything_set(g, bimpl), bimpl, allow_inplace=variants.get("inplace", False),
                  conv_algo=variants.get("conv_fwd", "igemm"))


def block_output_schedule(g: Graph, variants=None, blocks=None):
    """Keep block outputs only; block internals are recomputed in backward."""
    return schedule_for_saved_set(g, block_output_set(g, blocks), variants)


def schedule_for_saved_set(g: Graph, F, variants=None):
    """Schedule that keeps exactly the forward tensors F (plus the intermediate tensors of kept creators
    that a backward operator reads) and recomputes everything else it needs."""
    variants = DEFAULT_VARIANTS if variants is None else variants
    F = set(F)
    bimpl = choose_bimpls(g, variants, saved=F)
    # an aux tensor can only be written while its creator runs: where the creator's output is
    # kept, keep the aux tensor its backward reads as well (max-pool window index)
    for b in g.bops:
        for d in deps_of(g, b["k"], bimpl[b["k"]]):
            if g.is_aux(d) and g.nodes[d - 1].ins[0] in F:
                F.add(d)
    return expand(g, F, bimpl, allow_inplace=variants.get("inplace", True), conv_algo=variants.get("conv_fwd", "igemm"),
                  hoist_residual_tail=True)


def block_checkpoint_schedule(g: Graph, keep, variants=None):
    """Segment rule: blocks whose index is in `keep` hold what their backward reads, the others are recomputed."""
    variants = DEFAULT_VARIANTS if variants is None else variants
    bimpl = choose_bimpls(g, variants)
    F = block_checkpoint_set(g, bimpl, set(keep))
    return expand(g, F, bimpl, allow_inplace=variants.get("inplace", True), conv_algo=variants.get("conv_fwd", "igemm"))


def vgg_alternate_schedule(g: Graph, variants=None):
    """VGG: every second convolution triple of a stage is recomputed (blocks named s<stage>c<index>)."""
    keep = {i for i, (name, _) in enumerate(g.blocks) if not (name.startswith("s") and int(name.split("c")[1]) % 2 == 1)}
    return block_checkpoint_schedule(g, keep, variants)


def unet_skip_schedule(g: Graph, variants=None):
    """UNet: the forward pass keeps the skip tensors (outputs of the down blocks) only."""
    return block_output_schedule(g, variants, blocks={i for i, (name, _) in enumerate(g.blocks) if name.startswith("down")})


def mobilenet_depthwise_schedule(g: Graph, variants=None):
    """MobileNetV2: the depthwise triples (blocks named *.dw) are recomputed, everything else is kept."""
    keep = {i for i, (name, _) in enumerate(g.blocks) if not name.endswith(".dw")}
    return block_checkpoint_schedule(g, keep, variants)


def googlenet_alternate_schedule(g: Graph, variants=None):
    """Inception network: every second block (stem stage or inception module) keeps what its backward reads,
    the others are recomputed from the kept block outputs around them."""
    keep = {b for b in range(len(g.blocks)) if b % 2 == 0} | {len(g.blocks) - 1}
    return block_checkpoint_schedule(g, keep, variants)
