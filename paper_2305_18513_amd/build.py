"""Builds ``libslimfit.so`` (the C-ABI library) for gfx950 with hipcc, in-tree.

    python -m paper_2305_18513_amd.build            # rebuild

hipcc cross-compiles without a GPU.  The flags keep fp32 arithmetic IEEE
(no FMA contraction, no fast-math; denormals are preserved by default on
gfx9) and switch packed-fp32 instruction selection off.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libslimfit.so")
OBJ_DIR = os.path.join(PKG, "_build")

SOURCES = ("api.hip", "quant.hip", "layer_delta.hip", "prune.hip", "prune_short.hip", "prune_global.hip", "layernorm.hip", "probe.hip")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", INCLUDE, "-I", CSRC,
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the library cannot be built")
    return exe


def _compile(src: str, extra_flags=(), obj_dir: str = OBJ_DIR) -> str:
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compile every source and link the shared library.  Always rebuilds.

    ``extra_flags`` (e.g. ``-DSLIMFIT_QUANT_UNROLL=2``) and ``out`` exist for
    tuning sweeps; the defaults build the library the binding loads.
    """
    obj_dir = OBJ_DIR if out == LIB else out + ".obj"
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(lambda s: _compile(s, tuple(extra_flags), obj_dir), SOURCES))
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build_library()
