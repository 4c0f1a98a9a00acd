"""Schedule oracle: the paper's forward and backward algorithms run literally (test infrastructure).

`interpret` walks Algorithm 1 (forward pass) and Algorithm 2 (backward pass
with recomputation) over Python sets L, S^k, L-hat, frees a tensor the moment
the algorithms drop it, and writes one event per allocation, free, operator
run and save.  `closed_form` evaluates the memory formulas of Section 3/4
(Eq. 1 forward, Eq. 5 backward, Eq. 3 recomputation with the exact L_i^k, and
the bound with L-bar of Appendix B) from the schedule bits alone, without
simulating; the two must agree.  `validate` checks the feasibility
constraints (Eq. 7, Eq. 8, Appendix C.3 in-place rules, Appendix D strict
dependency of intermediate nodes).

With `numerics=True` the interpreter also carries fp64 arrays through the
schedule (a freed tensor is really deleted), using the operator variants the
schedule selects.

Readings where the paper leaves room:
  * one stage per backward operator; a convolution owns a parameter-gradient
    stage followed by an input-gradient stage (Appendix D);
  * an intermediate (aux) node is written by its creator's kernel, in the
    stage in which the aux node itself is marked computed (r, or s^N in the
    forward pass); it is never a consumer that keeps its creator alive;
  * an in-place operator renames its input's buffer (no new bytes);
  * tensors saved for a stage but with index above the inner-loop position
    stay until the loop reaches them (last term of Eq. 3);
  * parameters, parameter gradients, caller inputs, BatchNorm statistics and
    the scalar loss are outside the accounting (constants of the model).
"""
import numpy as np

from .graphtext import OGraph, OSchedule, align
from . import network as net

ALLOC, FREE, RUN_FWD, RUN_RECOMPUTE, RUN_BWD, SAVE, ALIAS = range(7)
T_FWD, T_GRAD, T_FWS, T_BWS = range(4)


class ScheduleError(ValueError):
    pass


def _deps(g, sch, k):
    return [d for d in g.bops[k].impls[sch.stage_impl[k]]["deps"] if d > 0]


def _grad_inputs(g, bop):
    """Input positions of the forward node that backward operator `bop` writes gradients for."""
    if bop.kind.endswith("_wgrad"):
        return []
    n = g.nodes[bop.node]
    if bop.kind == "softmaxce_bwd":
        return [0]
    return [p for p, j in enumerate(n.ins) if j > 0]


def _computed_in_stage(g, sch, k):
    return sch.r[k]


# ----------------------------------------------------------------------
def validate(g: OGraph, sch: OSchedule):
    N, B = g.N, g.B
    for i, n in g.nodes.items():
        l = sch.fwd_impl[i]
        if n.is_aux:
            if l != -1:
                raise ScheduleError(f"aux node {i} carries a forward implementation")
        elif not (0 <= l < len(n.fimpls)):
            raise ScheduleError(f"delta: node {i} has no forward implementation {l}")
        if n.persist and i in sch.fwd_save:
            raise ScheduleError(f"node {i} is persistent and cannot be saved")
    for k, b in g.bops.items():
        if not (0 <= sch.stage_impl[k] < len(b.impls)):
            raise ScheduleError(f"delta-hat: backward operator {k} has no implementation {sch.stage_impl[k]}")
    # forward pass: aux only with its creator (always computed), in-place rules
    for i, n in g.nodes.items():
        if n.is_aux or not n.fimpls[sch.fwd_impl[i]]["inplace"]:
            continue
        j = n.ins[0]
        if j <= 0 or g.nodes[j].is_aux or g.nbytes(j) != g.nbytes(i):
            raise ScheduleError(f"C.3: node {i} cannot run in place over {j}")
        if j in sch.fwd_save:
            raise ScheduleError(f"C.3: node {i} runs in place over {j}, which the forward pass saves")
        if any(t != i for t in g.consumers[j]):
            raise ScheduleError(f"C.3: node {i} runs in place over {j}, which another operator reads")
    for k in range(B, 0, -1):
        rk, sk = sch.r[k], sch.s[k]
        enter = sch.saved_entering(k, B)
        fk = g.bops[k].node
        D = _deps(g, sch, k)
        overwritten = {}
        for i in sorted(rk):
            n = g.nodes[i]
            if i in enter:
                raise ScheduleError(f"stage {k}: node {i} is recomputed although it is already held")
            if i > fk and not (n.is_aux and n.ins[0] == fk):
                raise ScheduleError(f"Appendix B: stage {k} recomputes node {i} beyond its own node {fk}")
            if n.persist:
                raise ScheduleError(f"stage {k}: persistent node {i} cannot be recomputed")
            if n.is_aux:
                if rk[i] != -1 or n.ins[0] not in rk:
                    raise ScheduleError(f"Appendix D: aux node {i} recomputed at stage {k} without its creator")
                continue
            if not (0 <= rk[i] < len(n.fimpls)):
                raise ScheduleError(f"delta^k: node {i} has no forward implementation {rk[i]}")
            for j in n.ins:
                if j <= 0:
                    continue
                if j in overwritten:
                    raise ScheduleError(f"C.3: stage {k} node {i} reads {j}, overwritten in place by {overwritten[j]}")
                if not (j in sk or j in rk):
                    raise ScheduleError(f"Eq.7: stage {k} recomputes node {i} but input {j} is neither saved nor recomputed")
            if n.fimpls[rk[i]]["inplace"]:
                j = n.ins[0]
                if j <= 0 or g.nodes[j].is_aux or g.nbytes(j) != g.nbytes(i) or j not in rk:
                    raise ScheduleError(f"C.3: stage {k} node {i} cannot run in place over {j}")
                if j in sk:
                    raise ScheduleError(f"C.3: stage {k} node {i} runs in place over saved tensor {j}")
                if j in D:
                    raise ScheduleError(f"C.3: stage {k} node {i} overwrites dependency {j} of the backward operator")
                if any(t > i and t in rk for t in g.consumers[j]):
                    raise ScheduleError(f"C.3: stage {k} node {i} overwrites {j}, still read by a later recomputation")
                overwritten[j] = i
        for i in sk:
            if g.nodes[i].persist:
                raise ScheduleError(f"stage {k}: persistent node {i} cannot be saved")
            if not (i in enter or i in rk):
                raise ScheduleError(f"Eq.7: stage {k} saves node {i}, which is neither held nor recomputed")
            if i in overwritten:
                raise ScheduleError(f"C.3: stage {k} saves node {i}, overwritten in place")
        for d in D:
            if not (d in sk or d in rk):
                raise ScheduleError(f"Eq.8: backward operator {k} depends on node {d}, neither saved nor recomputed")
            if d in overwritten:
                raise ScheduleError(f"C.3: backward operator {k} depends on node {d}, overwritten in place")


# ----------------------------------------------------------------------
class _Numerics:
    """fp64 arrays carried through the schedule."""

    def __init__(self, g, exts, params):
        self.g, self.exts, self.params = g, exts, params
        self.x, self.gr, self.stats, self.pgrads = {}, {}, {}, {}
        self.loss = None

    def get(self, ref):
        return self.exts[ref] if ref <= 0 else self.x[ref]


def interpret(graph_text, schedule_text, exts=None, params=None, check=True):
    """Run Algorithms 1 and 2.  Returns dict(events, peak, fwd_peak, recomputes, [loss, grads])."""
    g = OGraph(graph_text)
    sch = OSchedule(schedule_text, g)
    if check:
        validate(g, sch)
    N, B = g.N, g.B
    num = _Numerics(g, exts, params) if exts is not None else None
    events = []
    live = 0
    peak = 0
    held = {}       # forward tensor id -> bytes (what is physically in memory)
    grads = {}      # node id -> bytes

    def ev(kind, stage, node, impl, aux, nbytes):
        nonlocal live, peak
        if kind == ALLOC:
            live += nbytes
        elif kind == FREE:
            live -= nbytes
        peak = max(peak, live)
        events.append((kind, stage, node, impl, aux, nbytes, live))

    def run_forward(i, l, stage, emit, kind):
        n = g.nodes[i]
        impl = n.fimpls[l]
        inplace = impl["inplace"]
        for j in n.ins:
            if j > 0 and j not in held:
                raise ScheduleError(f"stage {stage}: node {i} reads {j}, which is not in memory")
        if not inplace and not n.persist:
            held[i] = g.nbytes(i)
            ev(ALLOC, stage, i, -1, T_FWD, held[i])
        for c in emit:
            held[c] = g.nbytes(c)
            ev(ALLOC, stage, c, -1, T_FWD, held[c])
        if impl["ws"]:
            ev(ALLOC, stage, i, -1, T_FWS, align(impl["ws"]))
        ev(kind, stage, i, l, (1 if inplace else 0) | (2 if emit else 0), 0)
        if num is not None:
            y, aux = net.forward_op(g, n, num.get, num.params, num.stats, recompute=(kind == RUN_RECOMPUTE))
            if n.persist:
                num.loss = float(y[0])
            else:
                num.x[i] = y
            for c in emit:
                num.x[c] = aux[g.nodes[c].op]()
        if impl["ws"]:
            ev(FREE, stage, i, -1, T_FWS, align(impl["ws"]))
        if inplace:
            j = n.ins[0]
            held[i] = held.pop(j)
            ev(ALIAS, stage, i, -1, j, held[i])
            if num is not None:
                del num.x[j]

    def drop(stage, j):
        ev(FREE, stage, j, -1, T_FWD, held.pop(j))
        if num is not None:
            del num.x[j]

    # ---------------- Algorithm 1
    stage = B + 1
    for i in range(1, N + 1):
        n = g.nodes[i]
        if not n.is_aux:
            emit = [c for c in g.aux_children[i] if c in sch.fwd_save]
            run_forward(i, sch.fwd_impl[i], stage, emit, RUN_FWD)
        for j in sorted(held):
            if j > i:
                continue
            if j in sch.fwd_save or any(t > i for t in g.consumers[j]):
                continue
            drop(stage, j)
        if i in sch.fwd_save:
            if i not in held:
                raise ScheduleError(f"forward pass saves node {i}, which is not in memory")
            ev(SAVE, stage, i, -1, 0, held[i])
    fwd_peak = peak
    recomputes = 0

    # ---------------- Algorithm 2
    last_bop = {}
    for k, b in g.bops.items():
        last_bop[b.node] = min(k, last_bop.get(b.node, k))
    for k in range(B, 0, -1):
        bop = g.bops[k]
        rk, sk = sch.r[k], sch.s[k]
        D = set(_deps(g, sch, k))
        for i in range(1, N + 1):
            n = g.nodes[i]
            if i in rk and not n.is_aux:
                emit = [c for c in g.aux_children[i] if c in rk]
                run_forward(i, rk[i], k, emit, RUN_RECOMPUTE)
                recomputes += 1
            for j in sorted(held):
                if j > i:
                    continue
                if j in sk or j in D or any(t > i and t in rk for t in g.consumers[j]):
                    continue
                drop(k, j)
            if i in sk:
                if i not in held:
                    raise ScheduleError(f"stage {k} saves node {i}, which is not in memory")
                ev(SAVE, k, i, -1, 0, held[i])
        # backward_k
        n = g.nodes[bop.node]
        impl = bop.impls[sch.stage_impl[k]]
        for d in D:
            if d not in held:
                raise ScheduleError(f"backward operator {k} reads node {d}, which is not in memory")
        if not n.persist and bop.node not in grads:
            raise ScheduleError(f"backward operator {k} has no incoming gradient")
        acc = 0
        for p in _grad_inputs(g, bop):
            j = n.ins[p]
            if j in grads:
                acc |= 1 << p
            else:
                grads[j] = g.nbytes(j)
                ev(ALLOC, k, j, -1, T_GRAD, grads[j])
        if impl["ws"]:
            ev(ALLOC, k, k, -1, T_BWS, align(impl["ws"]))
        ev(RUN_BWD, k, k, sch.stage_impl[k], acc, 0)
        if num is not None:
            def getb(ref):
                return num.exts[ref] if ref <= 0 else num.x[ref]
            gy = None if n.persist else num.gr[n.id]
            din, dpar = net.backward_op(g, bop, impl["algo"], gy, getb, num.params, num.stats)
            for p, d in din.items():
                j = n.ins[p]
                if j > 0:
                    num.gr[j] = num.gr[j] + d if (acc >> p) & 1 else np.array(d, copy=True)
            num.pgrads.update(dpar)
        if impl["ws"]:
            ev(FREE, k, k, -1, T_BWS, align(impl["ws"]))
        if not n.persist and last_bop[bop.node] == k:
            ev(FREE, k, bop.node, -1, T_GRAD, grads.pop(bop.node))
            if num is not None:
                del num.gr[bop.node]
        for j in sorted(held):
            if j not in sk:
                drop(k, j)
    if held or grads or live != 0:
        raise ScheduleError(f"tensors left after the last stage: {sorted(held)} {sorted(grads)} live={live}")
    out = dict(events=events, peak=peak, fwd_peak=fwd_peak, recomputes=recomputes)
    if num is not None:
        out.update(loss=num.loss, grads=num.pgrads, stats=num.stats)
    return out


# ----------------------------------------------------------------------
def closed_form(graph_text, schedule_text):
    """Peak memory from the formulas alone.

    Returns dict(m_fwd{i}, m_bwd{k}, m_rec{(i,k)}, m_rec_dot{(i,k)}, m_rec_bar{(i,k)}, m_keep_bar{(i,k)},
    exact_peak, tight_peak, predicted_peak): `exact_peak` uses the true L_i^k of Section 3,
    `predicted_peak` the upper bound L-bar_i^k of Appendix B plus the
    no-recomputation term of Appendix C.2, `tight_peak` the same with Appendix B's
    tighter set L-dot_i^k (only operators up to the stage's own node can be recomputed
    before it, so only their inputs have to be counted as local).
    """
    g = OGraph(graph_text)
    sch = OSchedule(schedule_text, g)
    N, B = g.N, g.B
    sz = {i: g.nbytes(i) for i in g.nodes}

    def out_bytes(i, l, emitted):
        n = g.nodes[i]
        own = 0 if (n.fimpls[l]["inplace"] or n.persist) else sz[i]
        return own + sum(sz[c] for c in emitted)

    # ---- Eq. 1
    m_fwd = {}
    for i, n in g.nodes.items():
        if n.is_aux:
            continue
        l = sch.fwd_impl[i]
        emitted = [c for c in g.aux_children[i] if c in sch.fwd_save]
        L_i = {j for j in range(1, i) if any(t >= i for t in g.consumers[j])}
        S_i = {j for j in range(1, i) if j in sch.fwd_save}
        m_fwd[i] = align(n.fimpls[l]["ws"]) * (n.fimpls[l]["ws"] > 0) + out_bytes(i, l, emitted) + sum(sz[j] for j in L_i | S_i)

    # ---- gradient tensors: g_j is born at the highest stage that writes it, dies after the lowest stage of node j
    born, dies = {}, {}
    for k, b in g.bops.items():
        n = g.nodes[b.node]
        for p in _grad_inputs(g, b):
            j = n.ins[p]
            born[j] = max(born.get(j, 0), k)
        if not n.persist:
            dies[b.node] = min(dies.get(b.node, B + 1), k)

    def Lhat(k):
        return sum(sz[j] for j in born if born[j] > k >= dies[j])

    # ---- Eq. 5 and Eq. 3
    m_bwd, m_rec, m_rec_dot, m_rec_bar, m_keep_bar = {}, {}, {}, {}, {}
    for k in range(B, 0, -1):
        b = g.bops[k]
        impl = b.impls[sch.stage_impl[k]]
        D = set(_deps(g, sch, k))
        y_k = sum(sz[j] for j in born if born[j] == k)
        m_bwd[k] = (align(impl["ws"]) if impl["ws"] else 0) + y_k + Lhat(k) + sum(sz[j] for j in D | sch.s[k])
        enter = sch.saved_entering(k, B)
        rk = sch.r[k]
        for i in range(1, N + 1):
            n = g.nodes[i]
            later = sum(sz[j] for j in enter if j > i)
            if i in rk and not n.is_aux:
                l = rk[i]
                emitted = [c for c in g.aux_children[i] if c in rk]
                head = (align(n.fimpls[l]["ws"]) if n.fimpls[l]["ws"] else 0) + out_bytes(i, l, emitted) + Lhat(k)
                L_ik = {j for j in range(1, i) if any(t >= i and t in rk for t in g.consumers[j])}
                S_ik = {j for j in range(1, i) if j in sch.s[k]}
                D_lt = {j for j in D if j < i}
                m_rec[(i, k)] = head + sum(sz[j] for j in L_ik | S_ik | D_lt) + later
                Lbar = {j for j in range(1, i) if any(t >= i for t in g.consumers[j])}
                m_rec_bar[(i, k)] = head + sum(sz[j] for j in Lbar | S_ik | D_lt) + later
                Ldot = {j for j in range(1, i) if any(i <= t <= b.node for t in g.consumers[j])}
                m_rec_dot[(i, k)] = head + sum(sz[j] for j in Ldot | S_ik | D_lt) + later
            else:
                S_le = {j for j in range(1, i + 1) if j in sch.s[k]}
                D_le = {j for j in D if j <= i}
                m_keep_bar[(i, k)] = Lhat(k) + sum(sz[j] for j in S_le | D_le) + later
    exact = max(list(m_fwd.values()) + list(m_bwd.values()) + list(m_rec.values()))
    pred = max(list(m_fwd.values()) + list(m_bwd.values()) + list(m_rec_bar.values()) + list(m_keep_bar.values()))
    tight = max(list(m_fwd.values()) + list(m_bwd.values()) + list(m_rec_dot.values()) + list(m_keep_bar.values()))
    return dict(m_fwd=m_fwd, m_bwd=m_bwd, m_rec=m_rec, m_rec_dot=m_rec_dot, m_rec_bar=m_rec_bar, m_keep_bar=m_keep_bar,
                exact_peak=exact, tight_peak=tight, predicted_peak=pred)


def objective(graph_text, schedule_text):
    """Eq. 9: forward costs + backward costs + recomputation costs (summed over all i)."""
    g = OGraph(graph_text)
    sch = OSchedule(schedule_text, g)
    cost = 0.0
    for i, n in g.nodes.items():
        if not n.is_aux:
            cost += n.fimpls[sch.fwd_impl[i]]["cost"]
    for k, b in g.bops.items():
        cost += b.impls[sch.stage_impl[k]]["cost"]
        for i, l in sch.r[k].items():
            if l >= 0:
                cost += g.nodes[i].fimpls[l]["cost"]
    return cost
