"""Builds libpolarquant.so (the HIP kernels and their C ABI) for gfx950, in-tree.

`python -m paper_2502_00527_amd.build` compiles every source under csrc/ with
hipcc; it cross-compiles without a GPU.  The flags matter for correctness:
floating-point contraction is off (the encoder's fp32/fp64 operation chains are
part of the definition of the codes; fused multiply-adds are written out where
wanted), and packed-fp32 instructions are disabled.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libpolarquant.so")
SOURCES = ["pq_api.hip", "pq_encode.hip", "pq_values.hip", "pq_decode.hip", "pq_decode_partials.hip",
           "pq_decode_partials_ga.hip", "pq_decode_roles.hip", "pq_decode_roles_grid.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libpolarquant needs the ROCm toolchain")
    return exe


def _filter(text: str) -> str:
    return "\n".join(l for l in text.splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compiles every translation unit (in parallel) and links libpolarquant.so."""
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    procs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, *extra_flags, *inc, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, proc in procs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + _filter(out))
        if verbose and _filter(out).strip():
            print(_filter(out))
        objs.append(obj)
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + _filter(res.stdout + res.stderr))
    return LIB_PATH


if __name__ == "__main__":
    build()
    sys.exit(0)
