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

The memory rows use running sums per stage (continuous P_i >= P_{i-1} + |i| u_{k,i}, Q_i >= Q_{i+1} + |i+1| s^k_{i+1}),
which keeps every row at a handful of entries; sizes are in MiB.  `recompute_blocks` optionally removes the
recomputation variables outside a window of builder blocks, which is what makes a 225-node network solvable in minutes.

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
        self.ub = []

    def new(self, integer=True, cost=0.0, ub=1.0):
        self.integer.append(1 if integer else 0)
        self.cost.append(cost)
        self.ub.append(ub)
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


def solve(g: Graph, budget_bytes, tau=None, time_limit=120.0, mip_rel_gap=0.0, allow_inplace=True, recompute_blocks=None,
          tight_local=False):
    """Cheapest schedule whose predicted peak (the L-bar bound; with `tight_local` Appendix B's tighter L-dot bound,
    which counts as local to a recomputation before stage k only the inputs of operators up to the stage's own node)
    stays within `budget_bytes`.

    `tau` optionally maps ("f", node, l) / ("r", node, l) / ("b", k, l) to a cost; missing entries fall back to
    the graph's own cost fields.  `recompute_blocks` = w restricts the program: stage k may recompute only nodes of
    the builder's block that holds the stage's own node and of the w blocks before it (every solution of the
    restricted program is one of the full program; large networks become solvable in minutes).  Returns (schedule,
    objective value, solver status string); schedule is None if the program is infeasible or no solution was found
    in time."""
    N, B = len(g.nodes), len(g.bops)
    tau = tau or {}
    MB = 1.0 / (1 << 20)                 # memory rows are written in MiB: coefficients of order 1 .. 1e5
    sz = {i: node_bytes(g, i) * MB for i in range(1, N + 1)}
    budget = float(budget_bytes) * MB

    def wsb(d):
        return float(_align(d["ws"])) * MB if d["ws"] else 0.0

    blk, nb = {}, 0                      # block index of every node; nodes outside the builder's blocks form their own
    in_block = {i: b for b, (_, ids) in enumerate(g.blocks) for i in ids}
    last = None
    for i in range(1, N + 1):
        cur = in_block.get(i, ("solo", i))
        if cur != last and not g.is_aux(i):
            nb += 1
            last = cur
        blk[i] = nb
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
            if allowed and (recompute_blocks is None or blk[i] >= blk[fk[k]] - recompute_blocks):
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
        terms = [(dfw[i][l], wsb(g.fimpls[i][l])) for l in range(len(g.fimpls[i]))]
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
        R.add(terms, hi=budget - const)
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
    BIG = float(sum(sz.values()) + max([wsb(d) for i in g.fimpls for d in g.fimpls[i]] + [0]) + max(Lhat.values()) + max(ynew.values()))
    total = float(sum(sz.values()))

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
        # Running sums keep the memory rows sparse: P[i] >= sum of u_{k,j} |j| over j <= i (what is present up to
        # node i), Q[i] >= sum of s^k_j |j| over j > i (what entered the stage beyond i).  Memory is only bounded from
        # above, so ">=" defines them well enough.
        P, Q = {0: None}, {N: None}
        for i in range(1, N + 1):
            if i in uv[k]:
                P[i] = V.new(integer=False, ub=total)
                R.add([(P[i], 1.0), (uv[k][i], -sz[i])] + ([(P[i - 1], -1.0)] if P[i - 1] is not None else []), lo=0.0)
            else:
                P[i] = P[i - 1]
        for i in range(N - 1, -1, -1):
            nxt = S(k, i + 1)
            if nxt:
                Q[i] = V.new(integer=False, ub=total)
                R.add([(Q[i], 1.0)] + [(v, -sz[i + 1] * w) for v, w in nxt] + ([(Q[i + 1], -1.0)] if Q[i + 1] is not None else []), lo=0.0)
            else:
                Q[i] = Q[i + 1]

        def run(var):
            return [(var, 1.0)] if var is not None else []

        # backward memory (Eq. 10)
        terms = [(dbw[k][l], wsb(g.bimpls[k][l])) for l in range(len(deps))]
        R.add(terms + run(P[N]), hi=budget - ynew[k] - Lhat[k])
        # recomputation memory, L-bar bound (Eq. 11 with Appendix B / C.2)
        for i in range(1, N + 1):
            if persist[i]:
                continue
            # no recomputation of i: what is held or needed up to i, what entered the stage beyond i
            R.add(run(P[i]) + run(Q[i]), hi=budget - Lhat[k])
            if i not in rv[k] or is_aux[i]:
                continue
            Lset = set(Lstat[i])
            if tight_local:
                Lset = {j for j in Lset if any(i <= t <= fk[k] for t in consumers[j])}
            const = Lhat[k] + sum(sz[j] for j in Lset)
            terms = [(drc[k][i][l], wsb(g.fimpls[i][l]) - (sz[i] if inplace(i, l) else 0.0)) for l in range(len(g.fimpls[i]))]
            terms += [(rv[k][i], sz[i] + BIG)]
            terms += [(rv[k][c], sz[c]) for c in aux_children[i] if c in rv[k]]
            # present before i, apart from the tensors the L-bar bound counts as constants
            terms += run(P[i - 1]) + [(uv[k][j], -sz[j]) for j in Lset if j in uv[k]]
            R.add(terms + run(Q[i]), hi=budget - const + BIG)
    A = sparse.csr_matrix((R.v, (R.r, R.c)), shape=(len(R.lo), V.n))
    res = milp(c=np.array(V.cost), constraints=LinearConstraint(A, np.array(R.lo), np.array(R.hi)),
               integrality=np.array(V.integer), bounds=Bounds(np.zeros(V.n), np.array(V.ub)),
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


def main():
    """Solve one of the full-size workloads and write the schedule as text (header lines start with '#')."""
    import argparse
    import os
    import time
    from . import graphs, schedules
    from paper_2010_14501_amd import costs, monet
    ap = argparse.ArgumentParser(description=main.__doc__)
    makers = {"resnet50_b184": lambda: graphs.resnet50(batch=184), "vgg16_b176": lambda: graphs.vgg16_bn(batch=176),
              "unet_b11": lambda: graphs.unet(batch=11), "mobilenetv2_b272": lambda: graphs.mobilenet_v2(batch=272),
              "googlenet_b320": lambda: graphs.googlenet(batch=320)}
    ap.add_argument("--workload", default="resnet50_b184", choices=sorted(makers))
    ap.add_argument("--budget", type=float, required=True, help="fraction of the store-everything predicted peak")
    ap.add_argument("--recompute-blocks", type=int, default=0, help="-1: unrestricted")
    ap.add_argument("--time-limit", type=float, default=900.0)
    ap.add_argument("--gap", type=float, default=0.02)
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    g = makers[args.workload]()
    tau = costs.read_table(os.path.join(root, "workloads", "measured", f"costs_{args.workload}.txt"))
    gt = g.text()
    store = monet.Plan(gt, schedules.store_everything_schedule(g).text()).predicted_peak
    t0 = time.time()
    sch, obj, status = solve(g, int(args.budget * store), tau=tau, time_limit=args.time_limit, mip_rel_gap=args.gap,
                             recompute_blocks=None if args.recompute_blocks < 0 else args.recompute_blocks)
    secs = time.time() - t0
    if sch is None:
        raise SystemExit(f"no schedule after {secs:.0f} s: {status}")
    plan = monet.Plan(gt, sch.text())
    head = [f"# python -m workloads.ilp --workload {args.workload} --budget {args.budget} --recompute-blocks {args.recompute_blocks}"
            f" --time-limit {args.time_limit:g} --gap {args.gap:g} --out {args.out}",
            f"# budget {args.budget * store / 1e9:.3f} GB = {args.budget:g} x store-everything; objective (Eq. 9, measured costs) {obj:.2f} ms;"
            f" predicted peak {plan.predicted_peak / 1e9:.3f} GB; solved in {secs:.0f} s: {status}"]
    with open(args.out, "w") as fh:
        fh.write("\n".join(head) + "\n" + sch.text())
    print("\n".join(head))


if __name__ == "__main__":
    main()
