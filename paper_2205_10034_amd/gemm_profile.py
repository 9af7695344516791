"""Phase timing of the grouped GEMM kernels inside one MoE layer forward.

``python -m paper_2205_10034_amd.gemm_profile gpt large`` loads the phase-timing
build of the library (``libmoesys_hip_prof.so``, built with the product library),
runs one layer forward per named workload and prints, for each of the two grouped
GEMMs, where a wavefront's shader clocks go - multiplying between the K-step
barriers, waiting for its own operand loads, waiting at the barriers, in the
epilogues - and the shader clock frequency the kernel actually ran at (shader
clock counter against the 100 MHz reference counter).  Synthetic inputs of the
workload's shapes; nothing here is part of the product path.
"""
from __future__ import annotations

import ctypes
import os
import sys

import numpy as np
import torch

from . import binding
from .build import PROF_LIB

SLOTS = 16
WAVES = 8
CUS = 256


def run(name: str) -> None:
    import paper_2205_10034_amd as M
    from workloads import WORKLOADS, make_layer
    wl = WORKLOADS[name]
    layer = make_layer(wl)
    dev = "cuda"
    dt = torch.bfloat16
    x = torch.from_numpy(layer["x"]).to(dev).to(dt)
    t = {"w_router": torch.from_numpy(layer["w_router"]).to(dev)}
    if layer.get("b_router") is not None:
        t["b_router"] = torch.from_numpy(layer["b_router"]).to(dev)
    names = ("w1", "w2") if wl.act == "gelu" else ("w_gate_proj", "w_up", "w_down")
    for n in names:  # [E, in, out] -> [E, out, in]
        t[n] = torch.from_numpy(layer[n]).to(dev).to(dt).transpose(1, 2).contiguous()
    W = M.Weights(t, "output_major")
    cfg = M.MoEConfig.from_workload(wl)
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
    out = torch.empty_like(x)
    prof = torch.zeros(2 * CUS * WAVES * SLOTS, dtype=torch.int64, device=dev)
    L = binding.lib()
    L.moe_gemm_profile_set.argtypes = [ctypes.c_void_p]
    for _ in range(3):
        M.moe_layer_forward(cfg, W, x, None, out, ws)
    torch.cuda.synchronize()
    if L.moe_gemm_profile_set(prof.data_ptr()) != 0:
        raise RuntimeError("moe_gemm_profile_set failed")
    M.moe_layer_forward(cfg, W, x, None, out, ws)
    torch.cuda.synchronize()
    L.moe_gemm_profile_set(None)
    p = prof.cpu().numpy().reshape(2, CUS * WAVES, SLOTS).astype(np.float64)
    for g, nm in enumerate(("first GEMM", "second GEMM")):
        q = p[g]
        q = q[q[:, 5] > 0]  # wavefronts that ran at least one tile
        if not len(q):
            continue
        steps, tiles = q[:, 3], q[:, 5]
        life, ref = q[:, 9], q[:, 11] - q[:, 10]
        mhz = (life / np.maximum(ref, 1)).mean() * 100.0
        span_us = (q[:, 11].max() - q[:, 10].min()) / 100.0
        print(f"{name} {nm}: {len(q)} wavefronts, {steps.mean():.1f} K-steps and {tiles.mean():.2f} tiles each "
              f"(min {tiles.min():.0f}, max {tiles.max():.0f}); shader clock {mhz:.0f} MHz; "
              f"first start to last end {span_us:.1f} us")
        print(f"    wavefront lifetime [clocks]: mean {life.mean():.0f}  min {life.min():.0f}  max {life.max():.0f};  "
              f"start to first tile ready: mean {q[:, 8].mean():.0f}")
        total = life.mean()
        for i, lab in ((0, "multiply (barrier to wait)"), (1, "wait for own loads"), (2, "wait at K-step barrier"),
                       (4, "epilogue and tile switch"), (13, "  of it: last quarter K-step"), (14, "  of it: next tile's requests"), (12, "  of it: wait for first stage"), (7, "wait at tile-start barrier"), (6, "last epilogue")):
            v = q[:, i].mean()
            print(f"    {lab:28s} {v:12.0f} clocks  {100 * v / total:5.1f} %   per K-step {v / steps.mean():7.1f}   "
                  f"per tile {v / tiles.mean():9.1f}")
        print(f"    (inside multiply: finding the next tile, once per tile    {q[:, 15].mean() / tiles.mean():9.1f} clocks per tile)")
        half = len(q) // 2
        print("    per K-step, wavefronts 0-3 / 4-7 of a workgroup: multiply "
              f"{_by_wave(q, 0, 0):.0f} / {_by_wave(q, 0, 1):.0f}, barrier wait {_by_wave(q, 2, 0):.0f} / {_by_wave(q, 2, 1):.0f}")


def _by_wave(q: np.ndarray, col: int, upper: int) -> float:
    # rows are (workgroup, wavefront) in order; wavefront index = row mod 8 only when every workgroup ran,
    # so group by position inside each run of eight
    idx = np.arange(len(q)) % WAVES
    sel = (idx >= 4) if upper else (idx < 4)
    return float((q[sel, col] / np.maximum(q[sel, 3], 1)).mean())


def main(argv) -> int:
    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        return 2
    if not os.path.exists(PROF_LIB):
        print(f"{PROF_LIB} is not built: run `python -m paper_2205_10034_amd.build`", file=sys.stderr)
        return 2
    binding.use_library(PROF_LIB)
    for name in (argv or ["gpt"]):
        run(name)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
