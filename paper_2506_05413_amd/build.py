"""Builds libsmoothrot.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2506_05413_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libsmoothrot.so")

SOURCES = ["sr_api.hip", "fwht_quant.hip", "calib_fold.hip", "gemm_prefill.hip", "gemm_f6.hip", "gemm_decode.hip", "kv_quant.hip", "linear_decode.hip", "ceilings.hip"]

# packed-fp32 instructions are switched off on purpose (device code only)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _check_asm_loads() -> None:
    """The staged rotation kernels load rows with inline-assembly loads whose destination registers must not be
    touched before the matching wait (csrc/check_asm_loads.py): verified on the device assembly of this build."""
    asm = os.path.join(OBJ, "fwht_quant.s")
    dev_flags = [f for f in FLAGS if f not in ("-fPIC", "-fvisibility=hidden")]
    r = subprocess.run([_hipcc(), *dev_flags, "-S", "--cuda-device-only", os.path.join(CSRC, "fwht_quant.hip"), "-o", asm],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed for fwht_quant.hip:\n" + r.stderr[-2000:])
    r = subprocess.run([sys.executable, os.path.join(CSRC, "check_asm_loads.py"), asm], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("inline-assembly load check failed:\n" + r.stdout + r.stderr)


def build(verbose: bool = True) -> str:
    """Compile every HIP source and link the shared library; returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        check = ex.submit(_check_asm_loads)
        objs = list(ex.map(_compile, SOURCES))
        check.result()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
