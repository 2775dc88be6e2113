"""Builds libarkv.so (host C++ + gfx950 HIP kernels) in-tree with hipcc.

`python -m paper_2603_08727_amd.build --phase-trace` builds libarkv_trace.so beside it: the same sources with
-DARKV_PHASE_TRACE (in-kernel timestamps at the kernels' phase boundaries, read by phase_trace.py)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libarkv.so")
LIB_TRACE = os.path.join(HERE, "libarkv_trace.so")
LIB_MEASURE = os.path.join(HERE, "libarkv_measure.so")   # bandwidth measurement kernels, not part of the product
MEASURE_SOURCES = ["arkv_measure.hip"]
SOURCES = ["arkv_host.cpp", "arkv_decode.hip", "arkv_tailor.hip", "arkv_prefill.hip", "arkv_attn.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def build(verbose: bool = True, phase_trace: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build", "trace" if phase_trace else "product")
    flags = FLAGS + (["-DARKV_PHASE_TRACE"] if phase_trace else [])
    lib = LIB_TRACE if phase_trace else LIB
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    mobjs = [os.path.join(objdir, src + ".o") for src in MEASURE_SOURCES]
    for src, obj in zip(MEASURE_SOURCES, mobjs):
        cmd = [hipcc, *flags, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        objs.append(obj)
        cmd = [hipcc, *flags, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib]
    subprocess.run(cmd, check=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *mobjs, "-o", LIB_MEASURE], check=True)
    return lib


if __name__ == "__main__":
    print(build(phase_trace="--phase-trace" in sys.argv[1:]))
