"""Builds libdeeprebirth.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdeeprebirth.so")
CEILINGS_LIB = os.path.join(HERE, "libdr_ceilings.so")      # measuring aids for bench.py --ceilings; not linked into the library
SOURCES = ["api.hip", "conv_f32.hip", "conv_bf16.hip", "conv_bf16_dma.hip", "conv_bf16_patch.hip", "conv_bf16_rows.hip", "pointwise.hip", "pointwise_nhwc.hip", "train.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         # hipcc may otherwise pair fp32 operations into packed instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build_library(verbose=False, jobs=4):
    """Compiles every source (always) and links the shared library.  Returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _wait(procs, verbose)
    _wait(procs, verbose)
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    tmp = CEILINGS_LIB + ".tmp%d" % os.getpid()
    p = subprocess.run([hipcc] + FLAGS + ["-shared", os.path.join(CSRC, "ceilings.hip"), "-o", tmp], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if p.returncode != 0:
        sys.stderr.write(p.stdout)
        raise RuntimeError("hipcc failed on ceilings.hip")
    os.replace(tmp, CEILINGS_LIB)
    return LIB


def _wait(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        keep = [l for l in out.splitlines() if "packed-fp32-ops" not in l and "not a recognized feature" not in l]
        if p.returncode != 0:
            sys.stderr.write("\n".join(keep) + "\n")
            raise RuntimeError("hipcc failed on %s" % src)
        if verbose and keep:
            print("\n".join(keep), flush=True)


if __name__ == "__main__":
    print(build_library(verbose=True))
