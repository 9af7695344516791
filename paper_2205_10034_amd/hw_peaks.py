"""Peaks of the machine as measured by small kernels of this repository.

``python -m paper_2205_10034_amd.hw_peaks`` prints the streaming copy and read rates (HBM), the rate of a
loop of nothing but bf16 MFMAs together with the shader clock it ran at, and the conflict-free LDS read
rate.  They put the roofline fractions quoted for the kernels into context: the published peaks (8 TB/s,
2.5 PFLOP/s at 2.4 GHz) stay the denominators of record.  Uses the phase-timing build of the library.
"""
from __future__ import annotations

import ctypes
import os
import sys

from . import binding
from .build import PROF_LIB


def main() -> int:
    if not os.path.exists(PROF_LIB):
        print(f"{PROF_LIB} is not built: run `python -m paper_2205_10034_amd.build`", file=sys.stderr)
        return 2
    binding.use_library(PROF_LIB)
    L = binding.lib()
    out = (ctypes.c_double * 8)()
    L.moe_hw_peaks.argtypes = [ctypes.POINTER(ctypes.c_double)]
    st = L.moe_hw_peaks(out)
    if st != 0:
        print("moe_hw_peaks failed:", L.moe_last_error().decode(), file=sys.stderr)
        return 1
    cus = int(out[5])
    print(f"compute units: {cus}")
    print(f"streaming copy, 1 GiB -> 1 GiB: {out[0]:8.0f} GB/s read+written   ({out[0] / 8000:.2f} of 8 TB/s)")
    print(f"streaming read, 1 GiB:          {out[1]:8.0f} GB/s                ({out[1] / 8000:.2f} of 8 TB/s)")
    print(f"one cold read of 256 MiB:       {out[6]:8.0f} GB/s                ({out[6] / 8000:.2f} of 8 TB/s; one launch, events around it)")
    print(f"bf16 MFMA 32x32x16 loop:        {out[2]:8.1f} TFLOP/s at a shader clock of {out[3]:.0f} MHz "
          f"({out[2] / 2500:.2f} of 2.5 PFLOP/s; {out[2] * 1e12 / (cus * 4 * out[3] * 1e6):.0f} flop per clock per SIMD)")
    print(f"LDS 16-byte reads, conflict-free layout: {out[4]:6.1f} B per shader clock per CU")
    return 0


if __name__ == "__main__":
    sys.exit(main())
