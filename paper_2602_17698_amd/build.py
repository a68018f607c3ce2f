"""Builds libscalebits.so (gfx950) in-tree with hipcc: one object per .hip file, then a link.

Variants (compile-time switches of the arithmetic, one library each):
  ""   -> libscalebits.so      cost = sum s * d^2
  "l1" -> libscalebits_l1.so   cost = sum s * |d|   (-DSBITS_COST_POWER=1)
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
VARIANTS = {"": [], "l1": ["-DSBITS_COST_POWER=1"]}
SOURCES = ["api.hip", "reorder.hip", "cost.hip", "fused.hip", "alloc.hip", "pack.hip", "mpgemm.hip", "dequant.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-ffp-contract=off",                       # no implicit FMA: only the fmaf() the method names
         "-Xarch_device", "-fno-honor-nans",        # device code only: inputs are finite by contract,
                                                    # spares the NaN-quieting ops around min/max
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + INCLUDE, "-I" + CSRC, "-Wall", "-Wno-unused-function"]


def lib_path(variant: str = "") -> str:
    return os.path.join(HERE, "libscalebits%s.so" % ("_" + variant if variant else ""))


def _compile(src: str, force: bool, variant: str) -> str:
    objdir = os.path.join(HERE, "_build" + ("_" + variant if variant else ""))
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    deps.append(os.path.join(INCLUDE, "scalebits.h"))
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC, *FLAGS, *VARIANTS[variant], "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout)
        raise RuntimeError("hipcc failed on " + src)
    return obj


def build(force: bool = False, variant: str = "") -> str:
    LIB = lib_path(variant)
    os.makedirs(os.path.join(HERE, "_build" + ("_" + variant if variant else "")), exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, variant), SOURCES))
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(o) for o in objs):
        tmp = LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


def build_all(force: bool = False) -> list:
    return [build(force, v) for v in VARIANTS]


if __name__ == "__main__":
    for path in build_all(force="--force" in sys.argv):
        print(path)
