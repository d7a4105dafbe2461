"""Builds libdllm_hcsa.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2512_17077_amd.build        # compile everything, always

The library links only against the HIP runtime; there is no torch in its ABI.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
BUILD_DIR = os.path.join(_HERE, "_build")
LIB_PATH = os.path.join(_HERE, "libdllm_hcsa.so")

SOURCES = ["api.hip", "checks.hip", "select_kernels.hip", "pack_kernels.hip", "attend_f32.hip",
           "attend_sparse_bf16.hip", "attend_dense_bf16.hip"]
# the same sources with the device-side precondition checks compiled in (a debugging aid, see include/dllm_hcsa.h)
LIB_PATH_CHECKED = os.path.join(_HERE, "libdllm_hcsa_checked.so")
CHECKED_FLAGS = ["-DDLLM_CHECK_PRECONDITIONS"]

# packed-fp32 VALU forms are switched off for all device code
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-I", INCLUDE, "-I", CSRC]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; libdllm_hcsa.so cannot be built")


def _compile(src: str, extra=(), subdir: str = "") -> str:
    os.makedirs(os.path.join(BUILD_DIR, subdir), exist_ok=True)
    obj = os.path.join(BUILD_DIR, subdir, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False, extra=(), checked: bool = True) -> str:
    """Compiles the library, and (checked=True) its twin with the precondition checks, always from scratch."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    jobs = [(s, tuple(extra), "") for s in SOURCES]
    if checked:
        jobs += [(s, tuple(extra) + tuple(CHECKED_FLAGS), "checked") for s in SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda j: _compile(*j), jobs))
    n = len(SOURCES)
    for lib, part in ((LIB_PATH, objs[:n]), (LIB_PATH_CHECKED, objs[n:])):
        if part:
            subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *part], check=True)
            if verbose:
                print("built", lib)
    return LIB_PATH


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
