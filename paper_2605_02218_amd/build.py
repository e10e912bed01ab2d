"""Builds libcovspec.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcovspec.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["covspec_api.hip", "gemm.hip", "gemm64.hip", "elementwise.hip", "select.hip", "eigen.hip", "subspace.hip", "greedy.hip", "verify.hip", "draft.hip", "stream.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    """Compile every source and link the shared library; always rebuilds.  COVSPEC_HIPCC_FLAGS (optional, space
    separated) adds compiler flags, e.g. a -D that selects a kernel variant for a measurement."""
    os.makedirs(OBJDIR, exist_ok=True)
    hipcc = _hipcc()
    flags = FLAGS + os.environ.get("COVSPEC_HIPCC_FLAGS", "").split()
    objs = [os.path.join(OBJDIR, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(10, len(SOURCES))) as ex:
        outs = list(ex.map(one, zip(SOURCES, objs)))
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]))
    if verbose:
        sys.stdout.write("\n".join(o for o in outs if o.strip()) + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
