"""The 0-1 integer program of Section 4 (workloads/ilp.py) on graphs small enough to solve in seconds.

Every solution is checked by parties that share no code with the program: the oracle's validator (Eq. 7, Eq. 8,
Appendix C.3 / D), its closed-form memory model (the predicted peak is the quantity the program bounds), its
objective (Eq. 9) and the executor's own lowering; optimality is checked against the brute-force search over
checkpointed-block subsets, whose schedules are a subset of the program's feasible set."""
import pytest

from oracle import schedule as osch
from oracle import search as osearch
from workloads import graphs, ilp, schedules
import paper_2010_14501_amd as M


def check(g, sch, budget, obj):
    gt, st = g.text(), sch.text()
    og = osch.OGraph(gt)
    osch.validate(og, osch.OSchedule(st, og))
    cf = osch.closed_form(gt, st)
    plan = M.Plan(gt, st)
    assert cf["predicted_peak"] == plan.predicted_peak <= budget
    assert cf["exact_peak"] == plan.exact_peak == osch.interpret(gt, st)["peak"]
    assert abs(osch.objective(gt, st) - obj) <= 1e-9 * obj
    return plan


def test_tiny_chain_program_against_brute_force():
    g = graphs.tiny_chain()
    gt = g.text()
    store = M.Plan(gt, schedules.store_everything_schedule(g).text()).predicted_peak
    costs = []
    for frac in (1.0, 0.8, 0.6, 0.45):
        budget = int(frac * store)
        sch, obj, status = ilp.solve(g, budget, time_limit=120)
        assert sch is not None, (frac, status)
        check(g, sch, budget, obj)
        bf = osearch.brute_force(g, budget)
        if bf is not None:
            assert obj <= bf[0] * (1 + 1e-9), (frac, obj, bf[:4])
        costs.append(obj)
    assert costs == sorted(costs) and costs[0] < costs[-1]            # less memory never makes the step cheaper
    # with the whole store-everything footprint available nothing is recomputed
    sch, obj, _ = ilp.solve(g, store)
    assert not any(sch.r[k] for k in sch.r)


def test_program_reports_infeasibility():
    g = graphs.tiny_chain()
    sch, obj, status = ilp.solve(g, 20000)          # less than a single activation plus its gradient
    assert sch is None


def test_program_uses_the_cost_table_it_is_given():
    """Making one backward variant free must make the program choose it wherever the budget allows."""
    g = graphs.tiny_chain()
    store = M.Plan(g.text(), schedules.store_everything_schedule(g).text()).predicted_peak
    tau = {}
    for b in g.bops:
        if b["kind"] == "relu_bwd":
            for l, d in enumerate(g.bimpls[b["k"]]):
                tau[("b", b["k"], l)] = 0.0 if d["algo"] == "from_input" else 1e9
    sch, obj, _ = ilp.solve(g, store, tau=tau)
    for b in g.bops:
        if b["kind"] == "relu_bwd":
            assert g.bimpls[b["k"]][sch.stage_impl[b["k"]]]["algo"] == "from_input"
    og = osch.OGraph(g.text())
    osch.validate(og, osch.OSchedule(sch.text(), og))


def test_small_resnet_program_beats_the_block_heuristic():
    g = graphs.resnet50(batch=2, hw=32, classes=10, widths=(8, 16), depths=(1, 1), stem=8)
    gt = g.text()
    block = M.Plan(gt, schedules.block_output_schedule(g).text())
    budget = block.predicted_peak
    sch, obj, status = ilp.solve(g, budget, time_limit=240, mip_rel_gap=0.02)
    assert sch is not None, status
    check(g, sch, budget, obj)
    assert obj <= osch.objective(gt, schedules.block_output_schedule(g).text()) * (1 + 1e-9)


def test_program_trades_convolution_workspace_for_time():
    """Two 3x3 layers with 128 channels offer five forward / input-gradient implementations (plain, reduction split,
    Winograd with 2x2 output tiles, with 4x4 tiles through a workspace and with 4x4 tiles in one kernel) of differing
    workspace and cost.  With memory to spare the program takes the cheapest form everywhere (the one-kernel Winograd,
    which also needs less workspace than the other 4x4 form and so dominates it); as the budget shrinks it falls back to
    the smaller 2x2 form, to the split form, then to the workspace-free one (Appendix D's trade-off), and the objective
    never improves."""
    g = graphs.tiny_chain(batch=2, hw=8, channels=128, blocks=2)
    gt = g.text()
    store = M.Plan(gt, schedules.store_everything_schedule(g).text()).predicted_peak
    seen, costs = [], []
    for frac in (4.0, 0.45, 0.25, 0.11):
        budget = int(frac * store)
        sch, obj, status = ilp.solve(g, budget, time_limit=120)
        assert sch is not None, (frac, status)
        check(g, sch, budget, obj)
        algos = [g.fimpls[n.id][sch.fwd_impl[n.id]]["algo"] for n in g.nodes if n.op == "conv"]
        algos += [g.bimpls[b["k"]][sch.stage_impl[b["k"]]]["algo"] for b in g.bops if b["kind"] == "conv_dgrad"]
        seen.append(algos)
        costs.append(obj)
    assert all(a == "winograd4f" for a in seen[0])
    assert all(a == "winograd" for a in seen[1])
    assert all(a == "igemm_splitk" for a in seen[2])
    assert all(a == "igemm" for a in seen[3])
    assert costs == sorted(costs)


def test_block_window_restricts_the_program_without_leaving_it():
    """`recompute_blocks` = w only removes recomputation variables: every solution is still a valid schedule within
    the budget, it can never be cheaper than the unrestricted optimum, and a wider window is never worse."""
    g = graphs.tiny_chain(blocks=5)
    gt = g.text()
    budget = M.Plan(gt, schedules.block_output_schedule(g).text()).predicted_peak
    objs = []
    for w in (0, 1, None):
        sch, obj, status = ilp.solve(g, budget, time_limit=120, recompute_blocks=w)
        assert sch is not None, (w, status)
        check(g, sch, budget, obj)
        if w is not None:       # nothing outside the window is recomputed
            blocks = {i: b for b, (_, ids) in enumerate(g.blocks) for i in ids}
            for b in g.bops:
                own = blocks.get(b["node"])
                for i in sch.r[b["k"]]:
                    if own is not None and i in blocks:
                        assert own - w <= blocks[i] <= own, (w, b["k"], i)
        objs.append(obj)
    assert objs[0] >= objs[1] * (1 - 1e-9) >= objs[2] * (1 - 2e-9)
    # keeping block outputs and recomputing inside blocks is itself block-local, so w = 0 is at least as good
    assert objs[0] <= osch.objective(gt, schedules.block_output_schedule(g).text()) * (1 + 1e-9)


def test_committed_full_size_solutions_are_valid_schedules_within_their_budgets():
    """The full-size schedules the program found (kept as text; bench.py runs them as `<workload>_ilp_<budget>`) pass
    the oracle's validator and the executor's lowering, and their predicted peaks are within the budgets their
    headers state."""
    import glob
    import os
    import re
    import bench
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    files = sorted(glob.glob(os.path.join(root, "workloads", "measured", "ilp_*.sched")))
    assert len(files) >= 6
    for path in files:
        stem = os.path.basename(path)[len("ilp_"):-len(".sched")]
        base, frac = stem.rsplit("_", 1)
        g, sch, batch, desc = bench.build_workload(f"{base}_ilp_{frac}")
        gt, st = g.text(), sch.text()
        og = osch.OGraph(gt)
        osch.validate(og, osch.OSchedule(st, og))
        plan = M.Plan(gt, st)
        budget_gb = float(re.search(r"budget ([0-9.]+) GB", desc).group(1))
        assert plan.predicted_peak <= budget_gb * 1e9 * (1 + 1e-3), path
        assert plan.exact_peak <= plan.predicted_peak
        store = M.Plan(gt, schedules.store_everything_schedule(g).text()).predicted_peak
        assert plan.predicted_peak < (float(frac) + 0.005) * store, path
        assert sum(1 for e in plan.trace_tuples() if e[0] == M.RUN_RECOMPUTE) > 0


def test_program_with_the_tighter_local_bound():
    """Appendix B's L-dot bound as an option of the program: every solution of the L-bar program stays feasible, so
    the optimum (both programs solved to optimality) can only improve; the solution's tight predicted peak (closed
    form of the oracle, and the planner's) stays within the budget and above the exact peak."""
    g = graphs.resnet50(batch=2, hw=32, classes=10, widths=(4, 8, 8, 16), depths=(1, 1, 1, 1), stem=4)
    gt = g.text()
    budget = int(0.7 * M.Plan(gt, schedules.store_everything_schedule(g).text()).predicted_peak)
    loose, obj_loose, status = ilp.solve(g, budget, time_limit=200)
    tight, obj_tight, status_t = ilp.solve(g, budget, time_limit=200, tight_local=True)
    assert loose is not None and tight is not None and "successfully" in status and "successfully" in status_t, (status, status_t)
    st = tight.text()
    og = osch.OGraph(gt)
    osch.validate(og, osch.OSchedule(st, og))
    cf = osch.closed_form(gt, st)
    plan = M.Plan(gt, st)
    assert cf["exact_peak"] == plan.exact_peak <= cf["tight_peak"] == plan.predicted_peak_tight <= budget
    assert plan.predicted_peak_tight <= plan.predicted_peak
    assert abs(osch.objective(gt, st) - obj_tight) <= 1e-9 * obj_tight
    assert obj_tight <= obj_loose * (1 + 1e-9), (obj_tight, obj_loose)
