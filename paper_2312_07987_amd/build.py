"""Builds libswitchhead.so (the C-ABI library of include/switchhead.h) in-tree with hipcc
for gfx950.  `python -m paper_2312_07987_amd.build` or build() from Python."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libswitchhead.so")
OBJ = os.path.join(os.path.dirname(HERE), "_build")
SOURCES = ["host.hip", "routing.hip", "small.hip", "simt.hip", "mfma_gemm.hip", "mfma_pp.hip", "mfma_attn.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _run(cmd):
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), p.stdout, p.stderr))


def build(verbose=False, jobs=6):
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()
    objs = []
    cmds = []
    for s in SOURCES:
        o = os.path.join(OBJ, s.replace(".hip", ".o"))
        objs.append(o)
        cmds.append([cc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", o])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(_run, cmds))
    _run([cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
