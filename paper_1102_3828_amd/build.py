"""Build the HIP libraries for gfx950 in-tree (hipcc; no GPU needed to compile)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libivfadcr.so")
SYNTH_SRC = os.path.join(ROOT, "synthdata", "gen.hip")
SYNTH_LIB = os.path.join(ROOT, "synthdata", "libsynthgen.so")

SOURCES = ["index.hip", "gemm.hip", "select.hip", "scan.hip", "rerank.hip", "encode.hip", "search.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    return r.stderr


def build(verbose: bool = False) -> None:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(CSRC, "_build")
    os.makedirs(objdir, exist_ok=True)
    jobs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        jobs.append([hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        logs = list(ex.map(_run, jobs))
    if verbose:
        for l in logs:
            if l.strip():
                print(l, file=sys.stderr)
    objs = [j[-1] for j in jobs]
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    if os.path.exists(SYNTH_SRC):
        _run([hipcc, *FLAGS, "-shared", SYNTH_SRC, "-o", SYNTH_LIB])


if __name__ == "__main__":
    build(verbose=True)
    print("built", LIB)
