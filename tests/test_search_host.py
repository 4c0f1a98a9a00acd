"""Host-side checks of the block-level schedule search and of the cost-table text format (no GPU):
the search works on the executor's own lowering (exact peak) and on a cost table; here the table is
synthetic (the graph's flop-based cost fields)."""
import os

import pytest

from workloads import graphs, schedules, search
from paper_2010_14501_amd import costs
import paper_2010_14501_amd as M


def small_resnet():
    return graphs.resnet50(batch=2, hw=32, classes=10, widths=(4, 8, 8, 16), depths=(2, 2, 1, 1), stem=4)


def synthetic_tau(g):
    tau = {}
    for i, impls in g.fimpls.items():
        for l, d in enumerate(impls):
            tau[("f", i, l)] = tau[("r", i, l)] = d["cost"] * 1e-9
    for k, impls in g.bimpls.items():
        for l, d in enumerate(impls):
            tau[("b", k, l)] = d["cost"] * 1e-9
    return tau


def test_search_respects_the_budget_and_uses_slack():
    g = small_resnet()
    tau = synthetic_tau(g)
    gt = g.text()
    store = M.Plan(gt, schedules.store_everything_schedule(g, schedules.DEFAULT_VARIANTS).text()).exact_peak
    _, lean_peak, lean_ms = search.evaluate(g, gt, [1] * len(g.blocks), tau, M.Plan)
    assert lean_ms > 0 and lean_peak < store
    last = None
    for frac in (0.6, 0.8, 1.0):
        budget = int(lean_peak + frac * (store - lean_peak))
        levels, sch, peak, ms = search.greedy(g, tau, budget, M.Plan)
        assert peak <= budget
        plan = M.Plan(gt, sch.text())                       # the returned schedule is the evaluated one
        assert plan.exact_peak == peak
        assert ms <= lean_ms
        if last is not None:
            assert ms <= last + 1e-12                       # more memory never costs time
        last = ms
    assert last < 0.5 * lean_ms
    # a budget below the block-output schedule forces blocks to keep nothing
    low_levels, _, low_peak, low_ms = search.greedy(g, tau, int(0.97 * lean_peak), M.Plan)
    assert low_peak <= 0.97 * lean_peak and 0 in low_levels and low_ms > 0
    with pytest.raises(ValueError):
        search.greedy(g, tau, 1024, M.Plan)


def test_cost_table_text_roundtrip(tmp_path):
    g = graphs.tiny_chain()
    tau = synthetic_tau(g)
    lines = costs.table_lines(g, tau)
    assert any(l.startswith("b 1 conv_wgrad") for l in lines) and any(l.startswith("r ") for l in lines)
    path = os.path.join(tmp_path, "t.txt")
    with open(path, "w") as fh:
        fh.write("# header\n" + "\n".join(lines) + "\n")
    back = costs.read_table(path)
    assert set(back) == set(tau)
    assert all(abs(back[k] - tau[k]) <= 1e-6 + 1e-6 * abs(tau[k]) for k in tau)
    costs.apply_to_graph(g, back)
    assert g.fimpls[1][0]["cost"] == pytest.approx(back[("f", 1, 0)] * 1e3)


def test_committed_cost_table_covers_every_implementation_of_resnet50():
    g = graphs.resnet50(batch=184)
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "workloads", "measured", "costs_resnet50_b184.txt")
    tau = costs.read_table(path)
    for k, impls in g.bimpls.items():
        for l in range(len(impls)):
            assert ("b", k, l) in tau, (k, l)
    for i, impls in g.fimpls.items():
        algos = {d["algo"] for d in impls}
        for l, d in enumerate(impls):
            if d["algo"] == "inplace" and "oop" in algos:
                continue            # same kernel as the out-of-place record
            assert ("f", i, l) in tau or ("f", i, 1 - l) in tau, (i, l)
