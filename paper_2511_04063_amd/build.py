"""Builds libdartqr.so (the HIP library) in-tree for gfx950 with hipcc.

    python -m paper_2511_04063_amd.build [--incremental]

Every source is compiled to an object file under ``_build/`` (one hipcc process each, in parallel) and the objects are
linked into ``paper_2511_04063_amd/libdartqr.so``.  ``--incremental`` skips sources whose object is newer than the
source and every header; the default compiles everything.
"""

from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libdartqr.so")
OBJ_DIR = os.path.join(ROOT, "_build")

SOURCES = ["dq_api.hip", "gemm_f32.hip", "gemm_bf16.hip", "qr_kernels.hip", "qr_cholpanel.hip", "elementwise.hip",
           "heads_kernels.hip", "objective_kernels.hip", "cayley_kernels.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]

_NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stdout}\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = True, extra_flags=(), incremental: bool = False) -> str:
    """Compile every HIP source and link paper_2511_04063_amd/libdartqr.so; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs = []
    objects = []
    for src in SOURCES:
        spath = os.path.join(CSRC, src)
        opath = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        objects.append(opath)
        fresh = (incremental and not extra_flags and os.path.exists(opath)
                 and os.path.getmtime(opath) > max(os.path.getmtime(spath), newest_header))
        if not fresh:
            jobs.append([hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", spath,
                         "-o", opath])
    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", "8"))))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objects, "-o", LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(incremental="--incremental" in sys.argv[1:]))
