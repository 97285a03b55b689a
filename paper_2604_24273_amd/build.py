"""Builds libbitrl.so (gfx950) from csrc/ with hipcc, in-tree.

`python -m paper_2604_24273_amd.build` compiles every source each time it is
called; the tests, the smoke check and the benchmark only call it when no
library is present.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libbitrl.so")

SOURCES = ["api.hip", "quantize_weights.hip", "act_quant.hip", "gemm.hip", "gemv.hip", "attention.hip", "attention_mfma.hip", "misc.hip", "ppo.hip", "int8_weights.hip", "serialize.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr[-8000:]))
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp"
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr[-8000:])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


MICRO = os.path.join(PKG, "microbench")


def build_microbench(verbose: bool = False) -> None:
    """Stand-alone probes (pure MFMA rate, HBM stream) under microbench/bin/."""
    out = os.path.join(MICRO, "bin")
    os.makedirs(out, exist_ok=True)
    for name in ("mfma_i8_peak", "stream_copy"):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-o", os.path.join(out, name), os.path.join(MICRO, name + ".hip")]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (name, r.stderr[-4000:]))
        if verbose:
            print("built", os.path.join(out, name))


if __name__ == "__main__":
    build(verbose=True)
    build_microbench(verbose=True)
    sys.exit(0)
