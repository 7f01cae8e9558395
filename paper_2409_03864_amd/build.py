"""Builds libtsg.so (the C-ABI library) in-tree with hipcc for gfx950.

    python paper_2409_03864_amd/build.py [--force]

Run it as a file (or through __graft_entry__.build()): importing the package itself
requires the library to exist already.
"""
from __future__ import annotations

import os
import subprocess
import sys
import time
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtsg.so")
# (the slowest units first: the build is as long as its longest chain of units)
SOURCES = ["gemm_f32_conv.hip", "gemm_f32_conv_b.hip", "gemm_bf16_conv.hip", "gemm_bf16_conv_b.hip",
           "gemm_bf16_row.hip", "gemm_bf16_col.hip", "gemm_f32_row.hip", "gemm_f32_col.hip",
           "gemm_bf16_row_bt.hip", "gemm_bf16_col_bt.hip", "gemm_f32_row_bt.hip", "gemm_f32_col_bt.hip",
           "api.cpp", "reduce.hip", "ceiling.hip"]
PUBLIC_HEADER = os.path.join(HERE, "..", "include", "tsg.h")


def _deps(src: str):
    """Headers a source includes: the kernel units see their own kernel header, the C-ABI layer
    and the reduce see the public header."""
    deps = [os.path.join(CSRC, "tsg_internal.h")]
    if src.startswith("gemm_"):
        deps += [os.path.join(CSRC, h) for h in ("gemm_kernel.h", "gemm_elem.h", "gemm_tiles.h")]
    else:
        deps.append(PUBLIC_HEADER)
    return deps

# packed-fp32 instruction selection is switched off for all device code
HIPCC_FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-fno-gpu-rdc",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str, force: bool) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(OBJ, src + ".o")
    if force or _stale(obj, [path] + _deps(src)):
        cmd = [_hipcc()] + HIPCC_FLAGS + ["-x", "hip", "-c", path, "-o", obj]
        t0 = time.time()
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if os.environ.get("TSG_BUILD_VERBOSE"):
            print("  %-24s %6.1f s" % (src, time.time() - t0), file=sys.stderr, flush=True)
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB, objs):
        cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
