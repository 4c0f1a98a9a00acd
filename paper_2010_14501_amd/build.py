"""Builds libmonet.so (host planner + gfx950 kernels) in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmonet.so")
SOURCES = ["plan.cpp", "api.cpp", "elementwise.hip", "bn.hip", "fused.hip", "depthwise.hip", "conv.hip", "winograd.hip", "winograd_fused.hip", "im2col.hip", "pointwise.hip", "stem.hip"]
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-result", "-Wno-unknown-attributes",
]


def build(verbose=True):
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src + ".o")
        cmd = ["hipcc", "-c", "-x", "hip", os.path.join(CSRC, src), "-o", obj] + FLAGS
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip()]
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n" + out, file=sys.stderr)
        elif verbose and lines:
            print(f"[build] {src}:\n" + "\n".join(lines[:40]))
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    if verbose:
        print(f"[build] wrote {LIB}")
    return LIB


if __name__ == "__main__":
    build()
