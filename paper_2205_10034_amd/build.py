"""Builds libmoesys_hip.so (gfx950) in-tree with hipcc.

``python -m paper_2205_10034_amd.build`` compiles every translation unit under
``csrc/`` and links the shared library next to this file.  Nothing is built at
import time: tests, the smoke check and the bench load what is already there.
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
LIB = os.path.join(HERE, "libmoesys_hip.so")
# the same library with the grouped GEMM's phase timing compiled in (see gemm_profile.py); diagnostics only
PROF_LIB = os.path.join(HERE, "libmoesys_hip_prof.so")

SOURCES = ["api.cpp", "gate.hip", "dispatch.hip", "combine.hip", "ffn.hip", "grouped_gemm_bf16.hip",
           "grouped_wgrad_bf16.hip", "expert_gemv_bf16.hip", "backward.hip", "layer.hip", "ring.cpp", "expert_cache.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-ignored-optimization-argument",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(src: str, suffix: str = "", defines=()) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + suffix + ".o")
    cmd = [HIPCC] + FLAGS + ["-D" + d for d in defines] + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err:
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        prof = ex.submit(_compile, "grouped_gemm_bf16.hip", "_prof", ("MOESYS_GEMM_PROFILE",))
        peaks = ex.submit(_compile, "peaks.hip")  # machine peaks: diagnostics, linked into the timing build only
        objs = list(ex.map(_compile, SOURCES))
        prof_obj, peaks_obj = prof.result(), peaks.result()
    prof_objs = [prof_obj if o.endswith("grouped_gemm_bf16.o") else o for o in objs] + [peaks_obj]
    for lib, these in ((LIB, objs), (PROF_LIB, prof_objs)):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + these
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print(f"built {lib}")
    return LIB


if __name__ == "__main__":
    build()
