"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2010_14501_amd.profsum stats    <kernel_stats.csv> --title T --cmd CMD --out FILE [--top 40]
    python -m paper_2010_14501_amd.profsum traffic  --fetch F.csv --write W.csv --fetch-copy FC.csv --write-copy WC.csv
                                                    --copy-mib 1024 --bench-json B.json --title T --cmd CMD... --out FILE
    python -m paper_2010_14501_amd.profsum counters <counter_collection.csv>... --title T --cmd CMD... --out FILE [--match conv_tile]

`stats` reads the `*_kernel_stats.csv` of `rocprofv3 --kernel-trace --stats`; `traffic` and `counters` read the
`*_counter_collection.csv` files of `rocprofv3 --pmc` runs (one row per dispatch and counter).  `traffic` scales
FETCH_SIZE / WRITE_SIZE (KiB per dispatch) by what the same counters read for a plain copy of known size, lists the
kernels by bytes moved, and writes one `traffic` line per kernel group (the kernels behind a launch class of bench.py)
with the bytes per launch; bench.py reads those lines for `roofline.traffic`.
"""
import argparse
import collections
import csv
import json
import re


def short(name):
    name = name.replace("monet::(anonymous namespace)::", "").replace("monet::", "").replace("void ", "")
    return name.split("(")[0].strip()


# launch classes of bench.py -> the kernels their launches consist of (regular expressions on the short kernel name).
# conv_tile_kernel<MODE, WM, WN, VEC, USE>: MODE 0 forward, 1 input gradient, 2 filter gradient; USE 0 implicit GEMM,
# 1 / 2 / 3 the batched GEMMs of a Winograd forward pass / input gradient / filter gradient.  Linear and transposed
# convolution layers run on the same kernels, so their launches are counted with the class that shares the kernel.
GROUPS = [
    (("conv_fwd", "linear_fwd", "tconv_dgrad"), [r"^conv_tile_kernel<0, \d+, \d+, \w+, 0>$"]),
    (("conv_dgrad", "linear_dgrad", "tconv_fwd"), [r"^conv_tile_kernel<1, \d+, \d+, \w+, 0>$"]),
    (("conv_wgrad", "linear_wgrad", "tconv_wgrad"), [r"^conv_tile_kernel<2, \d+, \d+, \w+, 0>$"]),
    (("conv_fwd_winograd",), [r"^wino4?_filter_kernel<false>$", r"^wino4?_input_kernel<0>$", r"^conv_tile_kernel<0, \d+, \d+, \w+, 1>$",
                              r"^wino4?_output_kernel<false>$", r"^wino4_fused_kernel<false"]),
    (("conv_dgrad_winograd",), [r"^wino4?_filter_kernel<true>$", r"^wino4?_input_kernel<1>$", r"^conv_tile_kernel<0, \d+, \d+, \w+, 2>$",
                                r"^wino4?_output_kernel<true>$", r"^wino4_fused_kernel<true"]),
    (("conv_wgrad_winograd",), [r"^wino4?_input_kernel<2>$", r"^wino4?_dy_kernel$", r"^conv_tile_kernel<2, \d+, \d+, \w+, 3>$",
                                r"^wino4?_filter_back_kernel$"]),
    (("bn_bwd", "relu_bn_bwd", "relu_add_bn_bwd"), [r"^bn_bwd_"]),
    (("bn_relu_fwd", "bn_add_relu_fwd", "bn_relu_apply", "bn_add_relu_apply", "add_relu_fwd"), [r"^fwd_chain_kernel"]),
    (("dwconv_fwd", "dwconv_dgrad"), [r"^dw3_row_kernel", r"^dw3_dgrad_s2_kernel", r"^dw_fwd_kernel", r"^dw_dgrad_kernel"]),
]


def load_counters(path):
    """{(kernel, counter): [dispatches, sum]}"""
    agg = collections.defaultdict(lambda: [0, 0.0])
    with open(path) as fh:
        for r in csv.DictReader(fh):
            a = agg[(short(r["Kernel_Name"]), r["Counter_Name"])]
            a[0] += 1
            a[1] += float(r["Counter_Value"])
    return agg


def cmd_stats(a):
    with open(a.csv[0]) as fh:
        rows = list(csv.DictReader(fh))
    lines = [f"# {a.title}", "", "Command (run from the repo root on the MI355X box):", ""] + [f"    {c}" for c in a.cmd] + [
        "", "rocprofv3 kernel statistics (all launches of the run: warm-up, timed steps and the per-launch-timed pass):", "",
        f"{'kernel':<92} {'calls':>6} {'total ms':>10} {'avg us':>10} {'%':>6} {'min us':>9} {'max us':>9}"]
    for r in rows[:a.top]:
        lines.append(f"{short(r['Name']):<92} {int(r['Calls']):>6} {int(r['TotalDurationNs']) / 1e6:>10.3f} "
                     f"{float(r['AverageNs']) / 1e3:>10.2f} {float(r['Percentage']):>6.2f} {int(r['MinNs']) / 1e3:>9.2f} "
                     f"{int(r['MaxNs']) / 1e3:>9.2f}")
    open(a.out, "w").write("\n".join(lines) + "\n")


def cmd_traffic(a):
    fetch, write = load_counters(a.fetch), load_counters(a.write)
    fc, wc = load_counters(a.fetch_copy), load_counters(a.write_copy)
    copy_kib = a.copy_mib * 1024.0

    def factor(agg, counter):
        n, v = max((x for (k, c), x in agg.items() if c == counter), key=lambda x: x[1])
        return (v / n) / copy_kib, v / n
    ff, fraw = factor(fc, "FETCH_SIZE")
    wf, wraw = factor(wc, "WRITE_SIZE")
    bench = json.load(open(a.bench_json))
    steps = bench["steps"] + bench["warmup"]
    per_kernel = {}
    for (k, c), (n, v) in fetch.items():
        if c == "FETCH_SIZE":
            per_kernel[k] = [n, v * 1024.0 / ff, 0.0]
    for (k, c), (n, v) in write.items():
        if c == "WRITE_SIZE":
            per_kernel.setdefault(k, [n, 0.0, 0.0])[2] = v * 1024.0 / wf
    lines = [f"# {a.title}", "", "Commands (run from the repo root on the MI355X box; one counter per run):", ""]
    lines += [f"    {c}" for c in a.cmd]
    lines += ["", f"Calibration: a plain copy of {a.copy_mib} MiB (reads and writes that much per launch) reads",
              f"FETCH_SIZE = {fraw:.0f} KiB and WRITE_SIZE = {wraw:.0f} KiB per dispatch,",
              f"so FETCH_SIZE is divided by {ff:.4f} and WRITE_SIZE by {wf:.4f} below.", "",
              f"{'kernel':<64} {'dispatches':>10} {'read MB':>10} {'written MB':>11}   (per dispatch, calibrated; {steps} steps)"]
    for k, (n, rd, wr) in sorted(per_kernel.items(), key=lambda kv: -(kv[1][1] + kv[1][2]))[:a.top]:
        lines.append(f"{k:<64} {n:>10} {rd / n / 1e6:>10.1f} {wr / n / 1e6:>11.1f}")
    lines += ["", "Per launch class of bench.py (bytes of all kernels of the group over the steps profiled, divided by the group's",
              "launches in those steps; `algorithmic` = each operand and the output once, as bench.py counts it):", ""]
    classes = bench["launch_classes"]
    for labels, pats in GROUPS:
        launches = sum(classes.get(l, {}).get("launches", 0) for l in labels) * steps
        ks = [k for k in per_kernel if any(re.search(p, k) for p in pats)]
        if not launches or not ks:
            continue
        rd = sum(per_kernel[k][1] for k in ks)
        wr = sum(per_kernel[k][2] for k in ks)
        alg = sum(classes[l]["bytes"] for l in labels if l in classes) * steps / launches
        lines.append(f"traffic {'+'.join(l for l in labels if l in classes)} launches={launches} read_mb={rd / launches / 1e6:.1f} "
                     f"written_mb={wr / launches / 1e6:.1f} bytes_per_launch={(rd + wr) / launches:.0f} algorithmic={alg:.0f} "
                     f"ratio={(rd + wr) / launches / alg:.2f}")
    open(a.out, "w").write("\n".join(lines) + "\n")


def cmd_counters(a):
    agg = collections.defaultdict(dict)
    disp = {}
    for path in a.csv:
        for (k, c), (n, v) in load_counters(path).items():
            if a.match and not re.search(a.match, k):
                continue
            agg[k][c] = v
            disp[k] = n
    names = sorted({c for v in agg.values() for c in v})
    lines = [f"# {a.title}", "", "Commands (run from the repo root on the MI355X box; one counter group per run):", ""]
    lines += [f"    {c}" for c in a.cmd]
    lines += ["", "Counter sums over all dispatches of the kernel in the run (counters are per shader engine / XCD summed by rocprofv3):", ""]
    for k in sorted(agg, key=lambda k: -max(agg[k].values())):
        lines.append(f"{k}   ({disp[k]} dispatches)")
        for c in names:
            if c in agg[k]:
                lines.append(f"    {c:<32} {agg[k][c]:.6g}")
        v = agg[k]
        if "SQ_BUSY_CU_CYCLES" in v and "SQ_VALU_MFMA_BUSY_CYCLES" in v and v["SQ_BUSY_CU_CYCLES"] > 0:
            lines.append(f"    {'MFMA busy / CU busy':<32} {v['SQ_VALU_MFMA_BUSY_CYCLES'] / v['SQ_BUSY_CU_CYCLES']:.3f}")
        if "GRBM_GUI_ACTIVE" in v and v["GRBM_GUI_ACTIVE"] > 0:
            # GRBM_GUI_ACTIVE is summed over the 8 XCDs: / 8 = cycles the kernel's dispatches were on the chip; x 256 CUs (x 4 SIMDs)
            chip = v["GRBM_GUI_ACTIVE"] / 8.0
            if "SQ_BUSY_CU_CYCLES" in v:
                lines.append(f"    {'CU busy / (cycles x 256 CUs)':<32} {v['SQ_BUSY_CU_CYCLES'] / (chip * 256):.3f}")
            if "SQ_VALU_MFMA_BUSY_CYCLES" in v:
                lines.append(f"    {'MFMA busy / (cycles x 1024 SIMDs)':<32} {v['SQ_VALU_MFMA_BUSY_CYCLES'] / (chip * 1024):.3f}")
        if "SQ_INSTS_VALU" in v and "SQ_INSTS_VALU_MFMA_MOPS_F32" in v and v["SQ_INSTS_VALU_MFMA_MOPS_F32"] > 0:
            # one 32x32x2 fp32 instruction = 4096 flop = 8 counted units of 512 flop; SQ_INSTS_VALU counts matrix instructions too
            mfma = v["SQ_INSTS_VALU_MFMA_MOPS_F32"] / 8.0
            lines.append(f"    {'other vector instr. / MFMA instr.':<32} {(v['SQ_INSTS_VALU'] - mfma) / mfma:.2f}")
        if "SQ_WAVE_CYCLES" in v and "SQ_WAIT_INST_ANY" in v and v["SQ_WAVE_CYCLES"] > 0:
            lines.append(f"    {'any wait / wave cycles':<32} {v['SQ_WAIT_INST_ANY'] / v['SQ_WAVE_CYCLES']:.3f}")
        if "SQ_WAVE_CYCLES" in v and "SQ_WAIT_INST_LDS" in v and v["SQ_WAVE_CYCLES"] > 0:
            lines.append(f"    {'LDS wait / wave cycles':<32} {v['SQ_WAIT_INST_LDS'] / v['SQ_WAVE_CYCLES']:.3f}")
        if "SQ_LDS_BANK_CONFLICT" in v and "SQ_LDS_IDX_ACTIVE" in v and v["SQ_LDS_IDX_ACTIVE"] > 0:
            lines.append(f"    {'LDS conflict / LDS active':<32} {v['SQ_LDS_BANK_CONFLICT'] / v['SQ_LDS_IDX_ACTIVE']:.3f}")
    open(a.out, "w").write("\n".join(lines) + "\n")


def read_traffic(path, label):
    """bytes per launch recorded for the kernel group that contains `label`, or None."""
    try:
        with open(path) as fh:
            for line in fh:
                p = line.split()
                if len(p) > 2 and p[0] == "traffic" and label in p[1].split("+"):
                    for item in p[2:]:
                        if item.startswith("bytes_per_launch="):
                            return float(item.split("=")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["stats", "traffic", "counters"])
    ap.add_argument("csv", nargs="*")
    ap.add_argument("--title", default="")
    ap.add_argument("--cmd", action="append", default=[])
    ap.add_argument("--out", required=True)
    ap.add_argument("--top", type=int, default=40)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--fetch-copy")
    ap.add_argument("--write-copy")
    ap.add_argument("--copy-mib", type=int, default=1024)
    ap.add_argument("--bench-json")
    ap.add_argument("--match", default="")
    a = ap.parse_args()
    {"stats": cmd_stats, "traffic": cmd_traffic, "counters": cmd_counters}[a.what](a)


if __name__ == "__main__":
    main()
