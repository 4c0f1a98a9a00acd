"""Host-side checks of libmonet.so that need no GPU: every declared symbol is exported, and the
plan lowering (event trace, exact and predicted peak, feasibility errors) agrees with the oracle's
literal interpreter of the paper's forward/backward algorithms, record by record."""
import itertools
import os
import re

import pytest

from oracle import schedule as osch
from workloads import graphs, schedules
import paper_2010_14501_amd as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = M.load_library()
    names = set()
    for hdr in ("monet.h", "monet_kernels.h"):
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(monet_[a-z0-9_]+)\s*\(", text))
    assert len(names) >= 25
    for n in sorted(names):
        assert hasattr(lib, n), n


def check_against_oracle(g, sch):
    gt, st = g.text(), sch.text()
    want = osch.interpret(gt, st)
    cf = osch.closed_form(gt, st)
    plan = M.Plan(gt, st)
    assert plan.trace_tuples() == want["events"]
    assert plan.exact_peak == want["peak"] == cf["exact_peak"]
    assert plan.predicted_peak == cf["predicted_peak"]
    assert plan.exact_peak <= plan.predicted_peak_tight == cf["tight_peak"] <= plan.predicted_peak
    assert plan.arena_bytes - plan.persistent_bytes >= plan.exact_peak
    return plan


def test_trace_matches_oracle_on_all_tiny_schedules():
    g = graphs.tiny_chain()
    for bits in itertools.product([0, 1], repeat=4):
        C = {b for b in range(4) if bits[b]}
        check_against_oracle(g, schedules.tiny_chain_schedule(g, C))
        check_against_oracle(g, schedules.tiny_chain_schedule(g, C, schedules.STANDARD_VARIANTS))
    check_against_oracle(g, schedules.store_everything_schedule(g))


def test_trace_matches_oracle_on_resnet_shapes():
    g = graphs.resnet50(batch=2, hw=32, classes=10, widths=(4, 8, 8, 16), depths=(2, 2, 1, 1), stem=4)
    for sch in (schedules.store_everything_schedule(g),
                schedules.store_everything_schedule(g, schedules.DEFAULT_VARIANTS),
                schedules.block_output_schedule(g)):
        check_against_oracle(g, sch)


@pytest.mark.parametrize("net", ["vgg", "unet", "mbv2", "googlenet"])
def test_trace_matches_oracle_on_the_other_network_families(net):
    if net == "vgg":
        g = graphs.vgg16_bn(batch=2, hw=32, classes=10, widths=(8, 16, 16, 32, 32), fc=64)
    elif net == "unet":
        g = graphs.unet(batch=2, h=32, w=48, classes=2, base=8, depth=4)
    elif net == "googlenet":
        g = graphs.googlenet(batch=2, hw=32, classes=10, stem=(8, 8, 16),
                             inceptions=(("a", 8, (8, 12), (4, 8), 4), "pool", ("b", 12, (8, 16), (4, 8), 8)))
    else:
        g = graphs.mobilenet_v2(batch=2, hw=32, classes=10, stem=8, last=64,
                                stages=((1, 8, 1, 1), (6, 12, 2, 2), (6, 16, 2, 2), (6, 24, 1, 1)))
    bimpl = schedules.choose_bimpls(g, schedules.DEFAULT_VARIANTS)
    keep = {b for b in range(len(g.blocks)) if b % 2 == 0} | {len(g.blocks) - 1}
    alternate = schedules.expand(g, schedules.block_checkpoint_set(g, bimpl, keep), bimpl)
    recomputes = []
    for sch in (schedules.store_everything_schedule(g),
                schedules.store_everything_schedule(g, schedules.DEFAULT_VARIANTS),
                schedules.block_output_schedule(g), alternate):
        plan = check_against_oracle(g, sch)
        recomputes.append(sum(1 for e in plan.trace_tuples() if e[0] == M.RUN_RECOMPUTE))
    assert recomputes[0] == recomputes[1] == 0 and recomputes[2] > 0 and recomputes[3] > 0


def test_full_size_plans_of_the_other_network_families():
    """VGG-16 b176, UNet b11 at 416x608, MobileNetV2 b272 and the inception network b320 lower at their full
    sizes; recomputing block internals cuts the peak well below store-everything."""
    for g in (graphs.vgg16_bn(), graphs.unet(), graphs.mobilenet_v2(), graphs.googlenet()):
        lean = M.Plan(g.text(), schedules.block_output_schedule(g).text())
        store = M.Plan(g.text(), schedules.store_everything_schedule(g).text())
        assert lean.exact_peak <= lean.predicted_peak
        assert lean.exact_peak < 0.75 * store.exact_peak
        assert lean.arena_bytes - lean.persistent_bytes <= 1.3 * lean.exact_peak


def test_full_resnet50_plan_fragmentation_is_small():
    g = graphs.resnet50(batch=184)
    sch = schedules.block_output_schedule(g)
    plan = M.Plan(g.text(), sch.text())
    dynamic = plan.arena_bytes - plan.persistent_bytes
    assert plan.exact_peak <= plan.predicted_peak
    assert plan.exact_peak <= dynamic <= 1.25 * plan.exact_peak
    store = M.Plan(g.text(), schedules.store_everything_schedule(g).text())
    assert plan.exact_peak < 0.6 * store.exact_peak


def _small_nets():
    yield graphs.tiny_chain()
    yield graphs.resnet50(batch=2, hw=32, classes=10, widths=(8, 16, 16, 32), depths=(2, 2, 2, 2), stem=8)
    yield graphs.googlenet(batch=2, hw=32, classes=10, stem=(8, 8, 16),
                           inceptions=(("a", 8, (8, 12), (4, 8), 4), "pool", ("b", 12, (8, 16), (4, 8), 8)))
    yield graphs.mobilenet_v2(batch=2, hw=32, classes=10, stem=8, last=64, stages=((1, 8, 1, 1), (6, 12, 2, 2), (6, 12, 1, 1)))


def test_live_tensors_never_share_arena_bytes():
    """At every launch the tensors the plan holds (forward and gradient) occupy pairwise disjoint byte ranges,
    except an in-place result, which sits exactly on its input.  The allocator hands freed blocks out again late
    and whole near BatchNorm / add / ReLU launches; that must never put two live tensors on the same bytes."""
    checked = 0
    for g in _small_nets():
        for sch in (schedules.store_everything_schedule(g), schedules.block_output_schedule(g)):
            plan = M.Plan(g.text(), sch.text())
            launch_events = [i for i, e in enumerate(plan.trace()) if e["kind"] in (M.RUN_FWD, M.RUN_RECOMPUTE, M.RUN_BWD)]
            for ev in launch_events:
                spans = []
                for n in g.nodes:
                    for is_grad in (False, True):
                        off = plan.tensor_offset(ev, n.id, is_grad)
                        if off >= 0:
                            count = 1
                            for d in n.shape:
                                count *= d
                            nbytes = {"mask": 8, "poolidx": 1}.get(n.op, 4) * count      # 64-bit mask words, 8-bit tap indices
                            spans.append((off, off + nbytes, n.id, is_grad))
                spans.sort()
                for (a0, a1, an, ag), (b0, b1, bn, bg) in zip(spans, spans[1:]):
                    assert a1 <= b0 or (a0 == b0 and a1 == b1 and not ag and not bg), (ev, (an, ag, a0, a1), (bn, bg, b0, b1))
                checked += len(spans)
    assert checked > 10000


def test_graph_builder_workspaces_are_the_library_s():
    """The workspace a graph declares for a reduction-split convolution is what the kernel library asks for: all of
    it for `splits` ranges on every tile, and for splits = 1 exactly the size with which the library cuts the ragged
    last round (a smaller one would cut less, a larger one would be wasted peak memory)."""
    from paper_2010_14501_amd import monet
    seen = 0
    for g in (graphs.resnet50(batch=184), graphs.vgg16_bn(), graphs.unet(), graphs.mobilenet_v2(), graphs.googlenet()):
        by_id = {n.id: n for n in g.nodes}
        for n in g.nodes:
            if n.op != "conv" or n.ins[0] <= 0:
                continue
            N, H, W, C = by_id[n.ins[0]].shape
            K, a = n.shape[-1], n.attrs
            shape = (N, H, W, C, K, a["R"], a["S"], a["stride"], a["pad"])
            for b in g.bops:
                if b["node"] == n.id and b["kind"] == "conv_wgrad":
                    for impl in g.bimpls[b["k"]]:
                        if impl["algo"] in ("winograd", "winograd4"):
                            need = monet.call("monet_conv_winograd_wgrad_workspace_bytes", N, H, W, C, K, 2 if impl["algo"] == "winograd" else 4)
                            assert impl["ws"] == (need + 255) // 256 * 256, (g.params[n.pars[0]][1], impl, need)
                            seen += 1
            impls = [(0, i) for i in g.fimpls[n.id]]
            impls += [(1, i) for b in g.bops if b["node"] == n.id and b["kind"] == "conv_dgrad" for i in g.bimpls[b["k"]]]
            for which, impl in impls:
                if impl["algo"] in ("winograd", "winograd4"):
                    need = monet.call("monet_conv_winograd_workspace_bytes", N, H, W, C, K, 2 if impl["algo"] == "winograd" else 4)
                    assert impl["ws"] == (need + 255) // 256 * 256, (g.params[n.pars[0]][1], which, impl, need)
                    seen += 1
                if impl["algo"] != "igemm_splitk":
                    continue
                need = monet.call("monet_conv_workspace_bytes", which, *shape, impl["splits"])
                assert impl["ws"] == (need + 255) // 256 * 256 and need > 0, (g.params[n.pars[0]][1], which, impl, need)
                seen += 1
    assert seen > 60


def _edit(text, drop=None, add=None):
    lines = text.splitlines()
    if drop is not None:
        assert drop in lines, drop
        lines.remove(drop)
    if add is not None:
        lines.append(add)
    return "\n".join(lines) + "\n"


def test_infeasible_schedules_are_rejected_with_the_constraint_named():
    g = graphs.tiny_chain()
    gt = g.text()
    st = schedules.tiny_chain_schedule(g, {0, 2}).text()
    cases = [
        (_edit(st, drop="r 15 16 impl=-1"), "Eq.8"),
        (_edit(st, drop="s 15 11"), "Eq.7"),
        (_edit(st, add="s 12 5"), "Eq.7"),
        (_edit(st, add="r 16 16 impl=-1"), "Appendix D"),
        (_edit(_edit(st, drop="r 15 15 impl=0"), add="r 15 15 impl=1"), "C.3"),
        (st.replace("fwd 3 impl=0 save=1", "fwd 3 impl=1 save=1"), "C.3"),
        (_edit(st, add="r 16 2 impl=0"), "already held"),
        (_edit(st, add="r 2 5 impl=0"), "Appendix B"),
    ]
    for bad, needle in cases:
        with pytest.raises(M.MonetError) as ei:
            M.Plan(gt, bad)
        assert ei.value.code == -2 and needle in str(ei.value), (needle, str(ei.value))
        with pytest.raises(osch.ScheduleError):     # the oracle rejects the same schedules
            osch.interpret(gt, bad)


def test_bad_text_is_a_graph_error():
    g = graphs.tiny_chain()
    st = schedules.tiny_chain_schedule(g, {0, 2}).text()
    with pytest.raises(M.MonetError) as ei:
        M.Plan("not a graph\n", st)
    assert ei.value.code == -1
    with pytest.raises(M.MonetError) as ei:
        M.Plan(g.text().replace("deps=4 ", "deps=3 "), st)      # declared dependency differs from the kernel's
    assert ei.value.code == -1


def test_step_without_arena_is_refused():
    g = graphs.tiny_chain()
    plan = M.Plan(g.text(), schedules.tiny_chain_schedule(g, {0, 2}).text())
    with pytest.raises(M.MonetError) as ei:
        plan.step(None, [0], [0] * plan.num_params, [0] * plan.num_params)
    assert ei.value.code == -3
    with pytest.raises(M.MonetError) as ei:
        plan.bind_arena(256, 1024)
    assert ei.value.code == -3
