"""The paper's joint optimisation as a 0-1 integer program (CPU only; SciPy's HiGHS solver).

Variables (Section 4, "Solver variables" of Appendix A):
    s^N_i, s^{k-1}_i   tensor i is held after the forward pass / after stage k
    r^k_i              tensor i is recomputed in stage k
    delta_{i,l}        forward implementation of node i;  delta^k_{i,l} the one of its recomputation in stage k
    delta-hat_{k,l}    implementation of backward operator k
    u_{k,j}            auxiliary: tensor j is present when backward_k runs (it is in S^{k-1} or a dependency of the
                       chosen implementation) -- the linearisation of the products delta-hat_{k,l} * s^{k-1}_j of
                       Eq. 10 / Eq. 11 (Appendix C.4 does it with one auxiliary variable per product; one per
                       (k, j) bounded below by both factors' sums is equivalent here because memory only has to
                       stay below the budget)

Objective: Eq. 9 (forward + backward + recomputation cost).  Constraints: one implementation each; Eq. 7 (a
recomputation's inputs are held or recomputed; only held or recomputed tensors are saved); Eq. 8 (dependencies of the
chosen backward implementation); the memory constraints of Appendix C.2 -- forward Eq. 1, backward Eq. 10, recomputation
with the L-bar bound of Appendix B (active when r^k_i = 1, through a big-M term) and the no-recomputation form; the
in-place rules of Appendix C.3 with the in-place implementation's selector in the role of q^k_i.  Stage structure,
intermediate (aux) nodes and what lies outside the accounting follow the executor's reading (one stage per backward
operator, aux nodes only with their creator, persistent nodes never saved or recomputed, a held tensor is not
recomputed).

`solve` returns a `schedules.Schedule`; the executor's own lowering (`monet_plan_load`) and the oracle's validator
accept or reject it like any other schedule, and their predicted peak is the quantity bounded here.
"""
from __future__ import annotations

import numpy as np
from scipy import sparse
from scipy.optimize import Bounds, LinearConstraint, milp

from .graphs import Graph
from .schedules import Schedule


def _align(b, a=256):
    return (int(b) + a - 1) // a * a


def node_bytes(g: Graph, i):
    n = g.nodes[i - 1]
    count = 1
    for d in n.shape:
        count *= d
    return _align({"mask": 8, "poolidx": 1}.get(n.op, 4) * count)


class _Vars:
    def __init__(self):
        self.n = 0
        self.integer = []
        self.cost = []

    def new(self, integer=True, cost=0.0):
        self.integer.append(1 if integer else 0)
        self.cost.append(cost)
        self.n += 1
        return self.n - 1


class _Rows:
    """Sparse rows lo <= a.x <= hi."""

    def __init__(self):
        self.r, self.c, self.v, self.lo, self.hi = [], [], [], [], []

    def add(self, terms, lo=-np.inf, hi=np.inf):
        row = len(self.lo)
        acc = {}
        for col, val in terms:
            acc[col] = acc.get(col, 0.0) + val
        for col, val in acc.items():
            if val != 0.0:
                self.r.append(row)
                self.c.append(col)
                self.v.append(val)
        self.lo.append(lo)
        self.hi.append(hi)


def solve(g: Graph, budget_bytes, tau=None, time_limit=120.0, mip_rel_gap=0.0, allow_inplace=True):
    """Cheapest schedule whose predicted peak (the L-bar bound) stays within `budget_bytes`.

    `tau` optionally maps ("f", node, l) / ("r", node, l) / ("b", k, l) to a cost; missing entries fall back to
    the graph's own cost fields.  Returns (schedule, objective value, solver status string); schedule is None
    if the program is infeasible or no solution was found in time."""
    N, B = len(g.nodes), len(g.bops)
    tau = tau or {}
    sz = {i: node_bytes(g, i) for i in range(1, N + 1)}
    is_aux = {i: g.is_aux(i) for i in range(1, N + 1)}
    persist = {i: bool(g.nodes[i - 1].attrs.get("persist")) for i in range(1, N + 1)}
    ins = {i: [j for j in g.nodes[i - 1].ins if j > 0] for i in range(1, N + 1)}
    consumers = {i: [] for i in range(1, N + 1)}       # aux nodes are not consumers
    aux_children = {i: [] for i in range(1, N + 1)}
    for i in range(1, N + 1):
        if is_aux[i]:
            aux_children[ins[i][0]].append(i)
        else:
            for j in ins[i]:
                consumers[j].append(i)
    fk = {b["k"]: b["node"] for b in g.bops}
    kind = {b["k"]: b["kind"] for b in g.bops}

    def fcost(i, l, phase):
        return float(tau.get((phase, i, l), tau.get(("f", i, l), g.fimpls[i][l]["cost"])))

    def inplace(i, l):
        return bool(g.fimpls[i][l].get("inplace"))

    def inplace_possible(i):          # static part of Appendix C.3
        j = ins[i][0] if ins[i] else 0
        return j > 0 and not is_aux[j] and sz[j] == sz[i]

    V, R = _Vars(), _Rows()
    # ---- variables
    sv = {}                                               # sv[k][i]: S^k (k = B: after the forward pass)
    for k in range(0, B + 1):
        sv[k] = {i: V.new() for i in range(1, N + 1) if not persist[i]}
    dfw = {}                                              # delta_{i,l}
    for i in range(1, N + 1):
        if not is_aux[i]:
            dfw[i] = [V.new(cost=fcost(i, l, "f")) for l in range(len(g.fimpls[i]))]
    dbw = {k: [V.new(cost=float(tau.get(("b", k, l), g.bimpls[k][l]["cost"]))) for l in range(len(g.bimpls[k]))]
           for k in range(1, B + 1)}
    rv, drc, uv = {}, {}, {}
    for k in range(1, B + 1):
        rv[k], drc[k], uv[k] = {}, {}, {}
        for i in range(1, N + 1):
            if persist[i]:
                continue
            allowed = i <= fk[k] or (is_aux[i] and ins[i][0] == fk[k])     # Appendix B: nothing beyond the stage's own node
            if allowed:
                rv[k][i] = V.new()
                if not is_aux[i]:
                    drc[k][i] = [V.new(cost=fcost(i, l, "r")) for l in range(len(g.fimpls[i]))]
            uv[k][i] = V.new(integer=False)

    def S(k, i):                                         # s of S^k, 0 where no variable exists
        return [(sv[k][i], 1.0)] if i in sv[k] else []

    def Rk(k, i):
        return [(rv[k][i], 1.0)] if i in rv[k] else []

    # ---- exactly one implementation; recomputation implementation iff recomputed
    for i in dfw:
        R.add([(v, 1.0) for v in dfw[i]], 1.0, 1.0)
    for k in dbw:
        R.add([(v, 1.0) for v in dbw[k]], 1.0, 1.0)
    for k in range(1, B + 1):
        for i, vs in drc[k].items():
            R.add([(v, 1.0) for v in vs] + [(rv[k][i], -1.0)], 0.0, 0.0)

    # ---- forward pass: in-place rules (Appendix C.3) and memory (Eq. 1)
    Lstat = {i: [j for j in range(1, i) if not persist[j] and any(t >= i for t in consumers[j])] for i in range(1, N + 1)}
    for i in dfw:
        for l in range(len(g.fimpls[i])):
            if not inplace(i, l):
                continue
            j = ins[i][0] if ins[i] else 0
            ok = allow_inplace and inplace_possible(i) and all(t == i for t in consumers[j])
            if not ok:
                R.add([(dfw[i][l], 1.0)], 0.0, 0.0)
            else:
                R.add([(dfw[i][l], 1.0)] + S(B, j), hi=1.0)          # the overwritten input is not saved
        terms = [(dfw[i][l], float(_align(g.fimpls[i][l]["ws"]) if g.fimpls[i][l]["ws"] else 0)) for l in range(len(g.fimpls[i]))]
        const = 0.0
        if not persist[i]:
            const += sz[i]
            terms += [(dfw[i][l], -float(sz[i])) for l in range(len(g.fimpls[i])) if inplace(i, l)]
        for c in aux_children[i]:
            terms += [(v, float(sz[c]) * w) for v, w in S(B, c)]
        Lset = set(Lstat[i])
        const += sum(sz[j] for j in Lset)
        for j in range(1, i):
            if j not in Lset and not persist[j]:
                terms += [(v, float(sz[j]) * w) for v, w in S(B, j)]
        R.add(terms, hi=float(budget_bytes) - const)
    # aux tensors exist only where their creator ran: in the forward pass always, so s^N of an aux node is free

    # ---- gradient tensors (constants of the graph)
    born, dies = {}, {}
    for b in g.bops:
        k, n = b["k"], g.nodes[b["node"] - 1]
        if not b["kind"].endswith("_wgrad"):
            srcs = [0] if b["kind"] == "softmaxce_bwd" else [p for p, j in enumerate(n.ins) if j > 0]
            for p in srcs:
                j = n.ins[p]
                if j > 0:
                    born[j] = max(born.get(j, 0), k)
        if not persist[b["node"]]:
            dies[b["node"]] = min(dies.get(b["node"], B + 1), k)
    Lhat = {k: sum(sz[j] for j in born if born[j] > k >= dies.get(j, 0)) for k in range(1, B + 1)}
    ynew = {k: sum(sz[j] for j in born if born[j] == k) for k in range(1, B + 1)}
    BIG = float(sum(sz.values()) + max([_align(d["ws"]) for i in g.fimpls for d in g.fimpls[i]] + [0]) + max(Lhat.values()) + max(ynew.values()))

    # ---- stages
    for k in range(1, B + 1):
        node_k = fk[k]
        deps = [[d for d in g.bimpls[k][l]["deps"] if d > 0] for l in range(len(g.bimpls[k]))]
        for i in range(1, N + 1):
            if persist[i]:
                continue
            # a held tensor is not recomputed; only held or recomputed tensors are saved (Eq. 7, second part)
            if i in rv[k]:
                R.add(Rk(k, i) + S(k, i), hi=1.0)
            R.add(S(k - 1, i) + [(v, -w) for v, w in S(k, i)] + [(v, -w) for v, w in Rk(k, i)], hi=0.0)
            # u_{k,i} >= s^{k-1}_i and >= the selectors of the implementations that depend on i
            for v, w in S(k - 1, i):
                R.add([(uv[k][i], 1.0), (v, -w)], lo=0.0)
            sel = [(dbw[k][l], 1.0) for l in range(len(deps)) if i in deps[l]]
            if sel:
                R.add([(uv[k][i], 1.0)] + [(v, -w) for v, w in sel], lo=0.0)
                # Eq. 8: a dependency of the chosen implementation is saved or recomputed
                R.add(S(k - 1, i) + Rk(k, i) + [(v, -w) for v, w in sel], lo=0.0)
        for i in rv[k]:
            if is_aux[i]:       # Appendix D: an intermediate tensor is only written while its creator runs
                R.add(Rk(k, i) + [(v, -w) for v, w in Rk(k, ins[i][0])], hi=0.0)
                continue
            # Eq. 7, first part: inputs of a recomputation are held or recomputed
            for j in ins[i]:
                if persist[j]:
                    R.add([(rv[k][i], 1.0)], hi=0.0)
                    continue
                R.add([(rv[k][i], 1.0)] + [(v, -w) for v, w in S(k - 1, j)] + [(v, -w) for v, w in Rk(k, j)], hi=0.0)
            # in-place recomputation (Appendix C.3): the input is recomputed in this stage, not saved, not a
            # dependency of the backward operator, and no later recomputation of the stage reads it
            for l in range(len(g.fimpls[i])):
                if not inplace(i, l):
                    continue
                q = drc[k][i][l]
                j = ins[i][0] if ins[i] else 0
                if not (allow_inplace and inplace_possible(i) and j in rv[k]):
                    R.add([(q, 1.0)], 0.0, 0.0)
                    continue
                R.add([(q, 1.0), (rv[k][j], -1.0)], hi=0.0)
                R.add([(q, 1.0)] + S(k - 1, j), hi=1.0)
                for ld in range(len(deps)):
                    if j in deps[ld]:
                        R.add([(q, 1.0), (dbw[k][ld], 1.0)], hi=1.0)
                for t in consumers[j]:      # an earlier consumer has read it already; a later one would read the overwritten buffer
                    if t > i and t in rv[k]:
                        R.add([(q, 1.0), (rv[k][t], 1.0)], hi=1.0)
        # backward memory (Eq. 10)
        terms = [(dbw[k][l], float(_align(g.bimpls[k][l]["ws"]) if g.bimpls[k][l]["ws"] else 0)) for l in range(len(deps))]
        terms += [(uv[k][i], float(sz[i])) for i in uv[k]]
        R.add(terms, hi=float(budget_bytes) - ynew[k] - Lhat[k])
        # recomputation memory, L-bar bound (Eq. 11 with Appendix B / C.2)
        for i in range(1, N + 1):
            if persist[i]:
                continue
            later = [(v, float(sz[j]) * w) for j in range(i + 1, N + 1) if not persist[j] for v, w in S(k, j)]
            # no recomputation of i: what is held or needed up to i, what entered the stage beyond i
            keep = [(uv[k][j], float(sz[j])) for j in range(1, i + 1) if j in uv[k]]
            R.add(keep + later, hi=float(budget_bytes) - Lhat[k])
            if i not in rv[k] or is_aux[i]:
                continue
            Lset = set(Lstat[i])
            const = Lhat[k] + sum(sz[j] for j in Lset)
            terms = [(drc[k][i][l], float(_align(g.fimpls[i][l]["ws"]) if g.fimpls[i][l]["ws"] else 0) - (sz[i] if inplace(i, l) else 0.0))
                     for l in range(len(g.fimpls[i]))]
            terms += [(rv[k][i], float(sz[i]) + BIG)]
            terms += [(rv[k][c], float(sz[c])) for c in aux_children[i] if c in rv[k]]
            terms += [(uv[k][j], float(sz[j])) for j in range(1, i) if j in uv[k] and j not in Lset]
            R.add(terms + later, hi=float(budget_bytes) - const + BIG)
    A = sparse.csr_matrix((R.v, (R.r, R.c)), shape=(len(R.lo), V.n))
    res = milp(c=np.array(V.cost), constraints=LinearConstraint(A, np.array(R.lo), np.array(R.hi)),
               integrality=np.array(V.integer), bounds=Bounds(np.zeros(V.n), np.ones(V.n)),
               options=dict(time_limit=float(time_limit), mip_rel_gap=float(mip_rel_gap), disp=False))
    status = res.message
    if res.x is None:
        return None, None, status
    x = np.rint(res.x).astype(int)

    sch = Schedule(N, B)
    for i in range(1, N + 1):
        sch.fwd_impl[i] = -1 if is_aux[i] else int(np.argmax([res.x[v] for v in dfw[i]]))
        if not persist[i] and x[sv[B][i]]:
            sch.fwd_save.add(i)
    for k in range(1, B + 1):
        sch.stage_impl[k] = int(np.argmax([res.x[v] for v in dbw[k]]))
        for i in rv[k]:
            if x[rv[k][i]]:
                sch.r[k][i] = -1 if is_aux[i] else int(np.argmax([res.x[v] for v in drc[k][i]]))
        sch.s[k] = {i for i in sv[k - 1] if x[sv[k - 1][i]]}
    return sch, float(res.fun), status
