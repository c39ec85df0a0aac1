"""Builds libasyncspade.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libasyncspade.so")
OBJ = os.path.join(HERE, "_build")
DEMO = os.path.join(HERE, "abi_demo")
SOURCES = ["api.hip", "predict.hip", "score.hip", "topk.hip", "select_rows.hip", "select_fused.hip", "attn.hip", "attn_mfma.hip",
           "cache_ops.hip"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("build step failed: " + " ".join(cmd))
    if verbose and err.strip():
        print(err)


def build(verbose: bool = True) -> str:
    """Compiles every source to an object (in parallel, always from scratch) and links the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-DAS_BUILDING_LIBRARY",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
             "-fno-gpu-sanitize", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc] + flags + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize",
          "-Wl,--version-script=" + os.path.join(CSRC, "exports.map"), "-o", LIB] + objs, verbose)
    # a plain-C caller of the ABI: C99 host code through gcc, linked against the library and the HIP runtime
    _run(["gcc", "-std=c99", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
          "-I", "/opt/rocm/include", os.path.join(CSRC, "abi_demo.c"), "-o", DEMO, "-L", HERE, "-lasyncspade",
          "-Wl,-rpath,$ORIGIN", "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"], verbose)
    return LIB


if __name__ == "__main__":
    build()
