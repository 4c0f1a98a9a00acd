"""Brute-force schedule choice for tiny graphs (test infrastructure).

Stands in for the paper's 0-1 integer program (Section 4) where the graph is
small enough to enumerate: every subset of checkpointed blocks, crossed with
the operator-variant toggles, is expanded to a full schedule, checked for
feasibility (Eq. 7, Eq. 8, Appendix C.3), priced with the objective (Eq. 9)
and bounded with the memory constraints (Eq. 4, using the L-bar bound as the
paper's experiments do).  The cheapest schedule within the budget M wins.
"""
import itertools

from workloads import schedules

from . import schedule as osch


def brute_force(g, budget, variant_sets=None):
    """Return (cost, predicted_peak, checkpoint_blocks, variant_name, schedule_text) or None."""
    gt = g.text()
    if variant_sets is None:
        variant_sets = {"lean": schedules.DEFAULT_VARIANTS, "standard": schedules.STANDARD_VARIANTS}
    nb = len([b for b in g.blocks])
    best = None
    for bits in itertools.product([0, 1], repeat=nb):
        C = {b for b in range(nb) if bits[b]}
        for vname, variants in variant_sets.items():
            try:
                st = schedules.tiny_chain_schedule(g, C, variants).text()
                osch.interpret(gt, st)
            except (ValueError, osch.ScheduleError):
                continue
            peak = osch.closed_form(gt, st)["predicted_peak"]
            if peak > budget:
                continue
            cost = osch.objective(gt, st)
            cand = (cost, peak, sorted(C), vname, st)
            if best is None or cand[:2] < best[:2]:
                best = cand
    return best
