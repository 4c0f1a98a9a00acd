"""Measured operator costs: the paper's profiled tables tau_i^l / tau-hat_k^l (Section 4, Appendix D
"Implementation": every implementation of every operator is timed once, with its workspace c, and
the solver works from those tables).

The operators are timed where they run: a whole training step is executed under a schedule with
the fused launches switched off, every launch bracketed by a HIP event pair, and each launch record
names the forward node (or backward operator) and the implementation index it ran.  Several
schedules with different implementation choices cover all implementations.  Recomputation gets a
table of its own ("r"): a recomputed BatchNorm reuses its statistics and is cheaper than the first
forward.

Text table, one record per line:

    f|r|b <node or k> <op or kind> <impl index> <algo> ws=<bytes> ms=<milliseconds>

    python -m paper_2010_14501_amd.costs --workload resnet50_b184 --out workloads/measured/costs_resnet50_b184.txt
"""
import argparse
import os
import sys

import numpy as np


def measure(graph_text, schedule_texts, exts, params, steps=3):
    """{("f"|"r"|"b", id, impl): median ms} over `steps` timed steps of each schedule."""
    from .runner import StepRunner
    samples = {}
    for st in schedule_texts:
        run = StepRunner(graph_text, st, exts, params)
        run.plan.set_fusion(False)
        info = run.plan.launches()
        run.step()
        run.plan.set_timing(True)
        for _ in range(steps):
            run.step()
            ms = run.plan.read_timing()
            for (label, kind, ident, impl, _f, _b), t in zip(info, ms):
                key = ("b" if kind == 4 else ("f" if kind == 2 else "r"), int(ident), int(impl))
                samples.setdefault(key, []).append(float(t))
        run.plan.set_timing(False)
        del run
    return {k: float(np.median(v)) for k, v in samples.items()}


def table_lines(g, tau):
    """`g` is a graph description with .nodes, .fimpls, .bops, .bimpls (workloads.graphs.Graph)."""
    out = []
    for (phase, ident, impl), ms in sorted(tau.items(), key=lambda kv: (kv[0][0], kv[0][1], kv[0][2])):
        if phase == "b":
            kind = g.bops[ident - 1]["kind"]
            d = g.bimpls[ident][impl]
        else:
            kind = g.nodes[ident - 1].op
            d = g.fimpls[ident][impl]
        out.append(f"{phase} {ident} {kind} {impl} {d['algo']} ws={int(d['ws'])} ms={ms:.6f}")
    return out


def read_table(path):
    tau = {}
    with open(path) as fh:
        for line in fh:
            f = line.split()
            if len(f) < 7 or f[0] not in ("f", "r", "b"):
                continue
            tau[(f[0], int(f[1]), int(f[3]))] = float(f[6].split("=")[1])
    return tau


def apply_to_graph(g, tau):
    """Write the measured times (microseconds) into the cost fields of the graph's implementation records,
    where measured; the forward table fills fimpl costs, the backward table bimpl costs."""
    for (phase, ident, impl), ms in tau.items():
        if phase == "f":
            g.fimpls[ident][impl]["cost"] = ms * 1e3
        elif phase == "b":
            g.bimpls[ident][impl]["cost"] = ms * 1e3
    return g


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50_b184")
    ap.add_argument("--out", required=True)
    ap.add_argument("--steps", type=int, default=3)
    args = ap.parse_args()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    from workloads import graphs, schedules, tensors
    makers = {"resnet50_b184": lambda: graphs.resnet50(batch=184), "vgg16_b176": lambda: graphs.vgg16_bn(batch=176),
              "unet_b11": lambda: graphs.unet(batch=11), "mobilenetv2_b272": lambda: graphs.mobilenet_v2(batch=272),
              "googlenet_b320": lambda: graphs.googlenet(batch=320), "tiny_chain": graphs.tiny_chain}
    g = makers[args.workload]()
    exts, params = tensors.make_inputs(g, seed=0)
    lean, std = schedules.DEFAULT_VARIANTS, schedules.STANDARD_VARIANTS
    plain = dict(std, conv_wgrad="direct", tconv_wgrad="direct", conv_dgrad="igemm", conv_fwd="igemm",
                 relu_bwd="from_input", relu6_bwd="from_input")
    scheds = [schedules.block_output_schedule(g, lean),            # lean variants + recomputation
              schedules.store_everything_schedule(g, lean),        # every ReLU backward from its mask
              schedules.store_everything_schedule(g, std),         # standard variants, split convolutions
              schedules.store_everything_schedule(g, plain),       # workspace-free convolutions, ReLU from input
              schedules.block_output_schedule(g, schedules.IGEMM_VARIANTS),   # split implicit GEMM where Winograd is preferred
              schedules.block_output_schedule(g, schedules.WINOGRAD2_VARIANTS),   # Winograd with 2x2 output tiles where offered
              schedules.block_output_schedule(g, schedules.WINOGRAD_WS_VARIANTS),   # 4x4 tiles through the workspace where the one-kernel form is preferred
              schedules.block_output_schedule(g, schedules.IM2COL_VARIANTS)]   # explicit patch matrix + GEMM for every filter larger than 1x1
    tau = measure(g.text(), [s.text() for s in scheds], exts, params, args.steps)
    lines = [f"# operator cost table, workload {args.workload}, one MI355X, fp32; times are medians of {args.steps} steps",
             f"# python -m paper_2010_14501_amd.costs --workload {args.workload} --out {args.out}"] + table_lines(g, tau)
    with open(args.out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print(f"wrote {len(tau)} records to {args.out}")


if __name__ == "__main__":
    main()
