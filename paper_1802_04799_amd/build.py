"""Builds libtvg.so (HIP, gfx950 only) next to this file with hipcc.

Run as ``python -m paper_1802_04799_amd.build``; ``build(force=True)`` recompiles
every source.  The library is built in-tree so that it travels with the
repository snapshot to the GPU machine.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtvg.so")
SOURCES = ["api.cpp", "conv_igemm.hip", "conv3x3_patch.hip", "conv3x3_dbuf.hip", "conv7x7s2_stem.hip", "conv1x1.hip", "dwconv.hip", "dwpw.hip", "pool.hip", "probe.hip", "conv_f32_small.hip", "conv3x3_winograd.hip", "conv1x1_deep.hip"]
HEADERS = [os.path.join(CSRC, "tvg_internal.h"), os.path.join(CSRC, "tvg_device.h"),
           os.path.join(ROOT, "include", "tvg.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-x", "hip",
         # packed-fp32 instruction forms are disabled for every device function
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        cmd = [HIPCC] + FLAGS + ["-c", path, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if warn.strip():
            sys.stderr.write(warn + "\n")
    return obj


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB, objs):
        cmd = [HIPCC, "-shared", "--offload-arch=gfx950", "-o", LIB] + objs + \
              ["-Wl,-rpath,/opt/rocm/lib"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv, verbose=True)
