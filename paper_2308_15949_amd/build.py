"""Builds liblaud.so (gfx950 HIP kernels + C ABI) in-tree with hipcc.

    python -m paper_2308_15949_amd.build

Every source is compiled to an object of its own (in parallel), then linked; objects live in
csrc/_build/ (ignored by git).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "liblaud.so")
SOURCES = ["laud_api.hip", "laud_mask.hip", "laud_chanmask.hip", "laud_static.hip", "laud_se.hip", "laud_gemm.hip",
           "laud_probe.hip", "laud_tail.hip", "laud_head.hip"]
# packed-fp32 code generation is switched off for device code (the host pass warns that it
# does not know the feature; that is harmless).
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))
    if verbose and err.strip():
        print(err)


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build())
