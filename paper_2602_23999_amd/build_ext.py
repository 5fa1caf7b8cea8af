"""Builds librabitq_hip.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librabitq_hip.so")
PROBE = os.path.join(HERE, "stream_probe")
# (source, extra defines, object name)
UNITS = [("api.hip", [], "api.o"), ("gemm.hip", [], "gemm.o"), ("stages.hip", [], "stages.o"),
         ("scan_dispatch.hip", [], "scan_dispatch.o"), ("build.hip", [], "build.o"),
         ("scan.hip", ["-DRQ_PART=0"], "scan0.o"), ("scan.hip", ["-DRQ_PART=1"], "scan1.o"),
         ("scan.hip", ["-DRQ_PART=2"], "scan2.o"),
         ("estimate_mfma.hip", [], "estimate_mfma.o")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature" not in l)
    if out.strip():
        print(out, flush=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd))


def build(verbose: bool = True, jobs: int = 7) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("RQ_EXTRA_FLAGS", "").split()  # e.g. -DRQ_STATS for development counters
    os.makedirs(OBJ, exist_ok=True)
    cmds = [[hipcc, *FLAGS, *extra, *defs, "-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ, obj)]
            for src, defs, obj in UNITS]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[os.path.join(OBJ, o) for _, _, o in UNITS], "-o", LIB],
         verbose)
    # stand-alone driver of the streaming-regime scan (for counter runs under rocprofv3 without Python in the process)
    _run([hipcc, *FLAGS, os.path.join(CSRC, "stream_probe.hip"), "-L", HERE, "-lrabitq_hip", "-Wl,-rpath,$ORIGIN",
          "-o", PROBE], verbose)
    return LIB


if __name__ == "__main__":
    build()
