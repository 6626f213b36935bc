"""Builds libsla2.so (the C-ABI library of HIP kernels) for gfx950, in-tree.

    python -m paper_2602_12675_amd.build

hipcc cross-compiles without a GPU.  Objects go to _build/ (not committed); the
shared library lands next to this file, where the ctypes binding looks for it.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsla2.so")

SOURCES = ["sla2_api.cpp", "sla2_pool.hip", "sla2_router.hip", "sla2_router_soft.hip", "sla2_static.hip", "sla2_f32.hip", "sla2_bwd.hip", "sla2_bwd_mfma.hip", "sla2_mfma.hip", "sla2_dense.hip"]

# packed-fp32 instructions are switched off on purpose (known-bad forms on this hardware)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument", "-Wall"]


def _compile(src: str, obj: str, verbose: bool) -> None:
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if verbose and err:
        print(err, file=sys.stderr)


def build_library(verbose: bool = True) -> str:
    out = os.path.join(ROOT, "_build")
    os.makedirs(out, exist_ok=True)
    objs = [os.path.join(out, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        list(ex.map(lambda so: _compile(so[0], so[1], verbose), zip(SOURCES, objs)))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library())
