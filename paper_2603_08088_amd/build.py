"""Build libeagletv.so (hipcc, gfx950) in-tree.  Run as ``python -m paper_2603_08088_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libeagletv.so")
PROBE_LIB = os.path.join(HERE, "libeagletv_probe.so")   # measurement aids (include/eagletv_probe.h), separate on purpose
SOURCES = ["api.hip", "mask.hip", "attention.hip", "posterior.hip", "commit.hip", "lmhead.hip", "branch.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc(sources, target, verbose, extra=()):
    # extern "C" entry points are exported explicitly; everything else stays hidden
    cmd = [HIPCC] + FLAGS + ["-DETV_BUILDING"] + list(extra) + [os.path.join(CSRC, s) for s in sources] + ["-o", target]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False, extra=()) -> str:
    _hipcc(SOURCES, LIB, verbose, extra)
    _hipcc(["probe.hip"], PROBE_LIB, verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
