#!/usr/bin/env python3
"""Throughput of the schedule-executed training step on one MI355X.

A step is one pass of the whole hot path -- forward pass with greedy freeing and checkpoint
saving, then the backward pass with recomputation -- of the ResNet-50-shaped network at batch
184 (synthetic N(0,1) images, He-normal weights, uniform labels) under the block-output
schedule with the lean operator variants, through libmonet.so.  Inputs, weights and the arena
are resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50_b184|vgg16_b176|unet_b11|mobilenetv2_b272|googlenet_b320|tiny_chain, or one of these with _store_everything, _store_everything_lean, _block_outputs, _igemm, _ilp_<budget>]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3      # 256 CUs x 256 flop/clk x 2.4 GHz
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of a kernel class come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled by what the same
# counters read for a plain copy; counters cannot be read from inside this process, so the figure is the one recorded in
# profiles/step_<workload>_hbm_traffic.txt (written by `python -m paper_2010_14501_amd.profsum traffic`), null if that
# workload was not profiled.


def recorded_traffic(workload, label):
    from paper_2010_14501_amd import profsum
    return profsum.read_traffic(os.path.join(ROOT, "profiles", f"step_{workload}_hbm_traffic.txt"), label)


def _stored_schedule(path, batch):
    """A schedule the 0-1 program found (python -m workloads.ilp), kept as text beside the cost table it was priced with."""
    from workloads import schedules
    with open(path) as fh:
        lines = fh.read().splitlines()
    head = " ".join(l[1:].strip() for l in lines if l.startswith("#"))
    body = "\n".join(l for l in lines if not l.startswith("#")) + "\n"
    return schedules.StoredSchedule(body), batch, "0-1 integer program: " + head


def build_workload(name, variants=None):
    from workloads import graphs, schedules
    if name.endswith("_igemm"):          # the same workload with every convolution on the implicit GEMM (no Winograd form)
        g, sch, batch, desc = build_workload(name[:-len("_igemm")], schedules.IGEMM_VARIANTS)
        return g, sch, batch, desc + "; implicit-GEMM convolutions only"
    lean_variants = schedules.DEFAULT_VARIANTS if variants is None else variants
    if name == "resnet50_b184":
        g = graphs.resnet50(batch=184)
        return g, schedules.block_output_schedule(g, lean_variants), 184, "keep block outputs, recompute block internals; BN backward from output, ReLU backward from 1-bit mask, in-place BN/ReLU, split-K weight gradient, Winograd F(4x4, 3x3) for the 3x3 / stride-1 layers"
    if name.startswith("resnet50_b184_"):        # same network under another schedule
        g = graphs.resnet50(batch=184)
        kind = name[len("resnet50_b184_"):]
        if kind == "store_everything":
            return g, schedules.store_everything_schedule(g), 184, "store everything, standard variants (plain back-propagation)"
        if kind == "keep_masks":
            # block outputs plus the 1-bit sign masks of every ReLU: a recomputed convolution -> BatchNorm -> ReLU chain then
            # needs no mask again, and the ReLU rides in the convolution's epilogue with the BatchNorm
            F = schedules.block_output_set(g) | {n.id for n in g.nodes if g.is_aux(n.id) and g.nodes[n.ins[0] - 1].op in ("relu", "relu6")}
            return g, schedules.schedule_for_saved_set(g, F, lean_variants), 184, "keep block outputs and all ReLU sign masks, recompute the rest; lean variants"
        if kind == "store_everything_lean":
            return g, schedules.store_everything_schedule(g, lean_variants), 184, "store everything the lean variants read"
        if kind.startswith("budget_"):
            # block-level greedy search on the measured operator costs, peak budget = fraction of store-everything
            from workloads import search
            from paper_2010_14501_amd import costs, monet
            frac = float(kind[len("budget_"):])
            tau = costs.read_table(os.path.join(ROOT, "workloads", "measured", "costs_resnet50_b184.txt"))
            store = monet.Plan(g.text(), schedules.store_everything_schedule(g).text()).exact_peak
            levels, sch, peak, ms = search.greedy(g, tau, frac * store, monet.Plan, variants=lean_variants)
            return g, sch, 184, (f"greedy block-level search, budget {frac:.2f} x store-everything peak "
                                 f"({frac * store / 1e9:.2f} GB); block levels {''.join(map(str, levels))}; "
                                 f"predicted recomputation {ms:.1f} ms; lean variants")
        if kind.startswith("ilp_"):
            return (g,) + _stored_schedule(os.path.join(ROOT, "workloads", "measured", f"ilp_resnet50_b184_{kind[len('ilp_'):]}.sched"), 184)
        raise SystemExit(f"unknown workload {name}")
    lean = "; lean operator variants"
    nets = {"vgg16_b176": (lambda: graphs.vgg16_bn(batch=176), 176, schedules.vgg_alternate_schedule,
                           "every second convolution triple recomputed"),
            "unet_b11": (lambda: graphs.unet(batch=11), 11, schedules.unet_skip_schedule,
                         "forward pass keeps the skip tensors only"),
            "mobilenetv2_b272": (lambda: graphs.mobilenet_v2(batch=272), 272, schedules.mobilenet_depthwise_schedule,
                                 "depthwise triples recomputed"),
            "googlenet_b320": (lambda: graphs.googlenet(batch=320), 320, schedules.googlenet_alternate_schedule,
                               "every second block (stem stage / inception module) recomputed")}
    for base, (make, batch, named, desc) in nets.items():
        if name.startswith(base + "_ilp_"):
            g = make()
            path = os.path.join(ROOT, "workloads", "measured", f"ilp_{base}_{name[len(base) + 5:]}.sched")
            return (g,) + _stored_schedule(path, batch)
        if name == base:
            g = make()
            return g, named(g, lean_variants), batch, desc + lean
        if name == base + "_block_outputs":
            g = make()
            return g, schedules.block_output_schedule(g, lean_variants), batch, "keep block outputs, recompute block internals" + lean
        if name == base + "_store_everything":
            g = make()
            return g, schedules.store_everything_schedule(g), batch, "store everything, standard variants"
        if name == base + "_store_everything_lean":
            g = make()
            return g, schedules.store_everything_schedule(g, lean_variants), batch, "store everything the lean variants read"
    if name == "tiny_chain":
        g = graphs.tiny_chain()
        return g, schedules.tiny_chain_schedule(g, {0, 2}, lean_variants), 2, "checkpoint blocks {0,2}, recompute {1,3}; lean variants"
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(workload):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import network as onet
    from workloads import graphs, tensors
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    if workload.startswith("resnet50_b184"):
        batch = 32
        g = graphs.resnet50(batch=batch)
        sample = "same ResNet-50 graph at batch 32 (224x224, 1000 classes), one store-everything fp64 step"
    elif workload.startswith("vgg16_b176"):
        batch = 4
        g = graphs.vgg16_bn(batch=batch)
        sample = "same VGG-16 graph at batch 4 (224x224), one store-everything fp64 step"
    elif workload.startswith("unet_b11"):
        batch = 1
        g = graphs.unet(batch=batch, h=208, w=304)
        sample = "same UNet graph at batch 1 and half resolution (208x304), one store-everything fp64 step"
    elif workload.startswith("mobilenetv2_b272"):
        batch = 16
        g = graphs.mobilenet_v2(batch=batch)
        sample = "same MobileNetV2 graph at batch 16 (224x224), one store-everything fp64 step"
    elif workload.startswith("googlenet_b320"):
        batch = 32
        g = graphs.googlenet(batch=batch)
        sample = "same inception graph at batch 32 (224x224), one store-everything fp64 step"
    else:
        batch = 2
        g = graphs.tiny_chain()
        sample = "tiny chain at full size, one store-everything fp64 step"
    exts, params = tensors.make_inputs(g, seed=0)
    oe, op = tensors.oracle_inputs(exts, params)
    gt = g.text()
    t0 = time.perf_counter()
    onet.store_everything_step(gt, oe, op)
    dt = time.perf_counter() - t0
    return {"value": batch / dt, "unit": "images/s", "cores": int(threads), "kind": "oracle", "sample": sample,
            "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50_b184")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="run only a plain device copy of this many MiB (counter calibration) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (the step has no collectives); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py: no GPU visible; the training step exists only as gfx950 kernels")
    if args.copy_calibration:
        # plain copy of known size: what FETCH_SIZE / WRITE_SIZE read for it scales the counters of the step
        from paper_2010_14501_amd import monet
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.randn(n, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            monet.call("monet_copy", None, src.data_ptr(), dst.data_ptr(), n)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 20
        print(json.dumps({"copy_bytes_read": 4 * n, "copy_bytes_written": 4 * n, "launches": 20, "gbs": 8 * n / dt / 1e9}))
        return
    from workloads import tensors
    from paper_2010_14501_amd.runner import StepRunner

    g, sch, batch, sched_desc = build_workload(args.workload)
    exts, params = tensors.make_inputs(g, seed=0)
    run = StepRunner(g.text(), sch.text(), exts, params)
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        run.step(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    peak = 0
    for _ in range(args.steps):
        peak = run.step(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    loss = run.loss_value()

    out = {
        "metric": "train images/s at schedule peak-mem budget (ResNet-50 b184)" if args.workload == "resnet50_b184"
        else "train images/s at schedule peak-mem budget",
        "value": batch * args.steps / dt,
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "batch": batch, "schedule": sched_desc,
                   "nodes": len(g.nodes), "backward_ops": len(g.bops)},
        "peak_gb": peak / 1e9,
        "predicted_peak_gb": run.plan.predicted_peak / 1e9,
        "arena_gb": run.plan.arena_bytes / 1e9,
        "loss": loss,
    }

    # what the step launches, per class (static: from the plan's launch list)
    info = run.plan.launches(issued=True)
    static = {}
    for (label, kind, _id, impl, flops, nbytes, issued) in info:
        c = static.setdefault(label, {"launches": 0, "flops": 0.0, "bytes": 0.0, "issued": 0.0})
        c["launches"] += 1
        c["flops"] += flops
        c["bytes"] += nbytes
        c["issued"] += issued
    out["launch_classes"] = static

    if not args.no_roofline:
        # second pass over the same steps with a pair of HIP events around every operator launch
        import numpy as np
        run.plan.set_timing(True)
        tot = np.zeros(len(info))
        n_timed = max(3, min(args.steps, 10))
        for _ in range(n_timed):
            run.step(stream)
            tot += run.plan.read_timing()
        run.plan.set_timing(False)
        tot /= n_timed                                   # ms per launch, averaged over steps
        classes = {k: dict(v, ms=0.0) for k, v in static.items()}
        for (label, *_), ms in zip(info, tot):
            classes[label]["ms"] += float(ms)
        for c in classes.values():
            c["tflops"] = c["flops"] / (c["ms"] * 1e-3) / 1e12 if c["ms"] > 0 else 0.0
            c["issued_tflops"] = c["issued"] / (c["ms"] * 1e-3) / 1e12 if c["ms"] > 0 else 0.0
            c["gbs"] = c["bytes"] / (c["ms"] * 1e-3) / 1e9 if c["ms"] > 0 else 0.0

        def mfma_entry(c):
            # held against the peak: the flop the kernels put on the matrix cores (a Winograd form issues 1/4 to 1/2.25 of
            # the direct form's); `algorithmic` is the direct form's flop per second, the figure the metric counts
            return {"bound": "mfma", "achieved": c["issued_tflops"], "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": c["issued_tflops"] / MFMA_F32_PEAK_TFLOPS, "algorithmic": c["tflops"]}

        dom = max(classes, key=lambda k: classes[k]["ms"])
        d = classes[dom]
        if d["flops"] > 0:
            roof = mfma_entry(d)
        else:
            roof = {"bound": "hbm", "achieved": d["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": d["gbs"] / HBM_PEAK_GBS}
        roof.update({"kernel": dom, "launches_per_step": d["launches"], "avg_launch_ms": d["ms"] / d["launches"],
                     "traffic": recorded_traffic(args.workload, dom),
                     "algorithmic_bytes_per_launch": d["bytes"] / d["launches"]})
        # every convolution class beside the dominant one (implicit GEMM and Winograd forms, all three modes)
        roof["conv_classes"] = {k: dict(mfma_entry(v), ms=round(v["ms"], 3), launches=v["launches"],
                                        traffic=recorded_traffic(args.workload, k))
                                for k, v in classes.items() if k.startswith("conv_") and v["flops"] > 0}
        out["roofline"] = roof
        out["classes"] = {k: {"launches": v["launches"], "ms": round(v["ms"], 4), "tflops": round(v["tflops"], 2),
                              "issued_tflops": round(v["issued_tflops"], 2), "gbs": round(v["gbs"], 1)}
                          for k, v in sorted(classes.items(), key=lambda kv: -kv[1]["ms"])}
        out["timed_ms_per_step"] = float(tot.sum())

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
