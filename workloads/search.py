"""A small schedule search over block-level decisions (CPU only; stands in for the paper's solver
on networks too large for brute force).

The paper minimises total time (its objective, Eq. 9: forward + backward + recomputation cost)
under a peak-memory budget by an integer program over per-tensor bits.  Here the decision is
coarser -- per block one of three levels -- and the search is greedy, but both sides of the
trade-off are the real ones: the peak is the exact peak of the lowered plan (Eq. 1 / Eq. 5 / Eq. 3
evaluated by the executor's own lowering) and the time is the sum of measured operator costs of the
recomputation events of that plan (the third term of Eq. 9; the first two do not depend on the
decision once the operator variants are fixed).

    level 0  the block keeps nothing (it is recomputed from the nearest kept tensor before it)
    level 1  the block keeps its output
    level 2  the block keeps its output and every own tensor its backward operators read
"""
from .schedules import DEFAULT_VARIANTS, block_checkpoint_set, block_output_set, choose_bimpls, schedule_for_saved_set


def saved_set(g, levels, variants=None):
    variants = DEFAULT_VARIANTS if variants is None else variants
    bimpl = choose_bimpls(g, variants)
    F = block_output_set(g, {b for b, l in enumerate(levels) if l >= 1})
    F |= block_checkpoint_set(g, bimpl, {b for b, l in enumerate(levels) if l >= 2})
    return F


def evaluate(g, graph_text, levels, tau, lower, variants=None):
    """(schedule, exact peak bytes, recomputation ms).  `lower(graph_text, schedule_text)` returns an object
    with .exact_peak and .trace_tuples() (the executor's plan); `tau` maps ("r"|"f", node, impl) to ms."""
    sch = schedule_for_saved_set(g, saved_set(g, levels, variants), variants)
    plan = lower(graph_text, sch.text())
    ms = 0.0
    for kind, _stage, node, impl, _aux, _bytes, _live in plan.trace_tuples():
        if kind == 3:     # RUN_RECOMPUTE
            ms += tau.get(("r", node, impl), tau.get(("f", node, impl), 0.0))
    return sch, plan.exact_peak, ms


def greedy(g, tau, budget_bytes, lower, variants=None, start_level=1, log=None):
    """Raise block levels while the peak stays within the budget, each time taking the raise that saves
    the most recomputation time per byte of peak it costs (raises that cost no peak go first); if the
    start point itself is over budget, first lower levels, cheapest time per byte saved first.
    Returns (levels, schedule, peak, recomputation ms)."""
    gt = g.text()
    nb = len(g.blocks)
    levels = [start_level] * nb
    sch, peak, ms = evaluate(g, gt, levels, tau, lower, variants)
    while peak > budget_bytes:
        best = None
        for b in range(nb):
            if levels[b] == 0:
                continue
            trial = list(levels)
            trial[b] -= 1
            try:
                s2, p2, m2 = evaluate(g, gt, trial, tau, lower, variants)
            except Exception:
                continue
            if p2 >= peak:
                continue
            score = (m2 - ms) / (peak - p2)
            if best is None or score < best[0]:
                best = (score, trial, s2, p2, m2)
        if best is None:
            raise ValueError("budget cannot be met by block-level decisions")
        _, levels, sch, peak, ms = best
        if log:
            log(f"lower -> peak {peak / 1e9:.3f} GB, recompute {ms:.2f} ms")
    while True:
        best = None
        for b in range(nb):
            if levels[b] == 2:
                continue
            trial = list(levels)
            trial[b] += 1
            try:
                s2, p2, m2 = evaluate(g, gt, trial, tau, lower, variants)
            except Exception:
                continue
            if p2 > budget_bytes or m2 >= ms:
                continue
            score = (ms - m2) / max(p2 - peak, 1)
            if best is None or score > best[0]:
                best = (score, trial, s2, p2, m2)
        if best is None:
            break
        _, levels, sch, peak, ms = best
        if log:
            log(f"raise -> peak {peak / 1e9:.3f} GB, recompute {ms:.2f} ms")
    return levels, sch, peak, ms
