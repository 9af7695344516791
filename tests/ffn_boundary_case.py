"""Grouped-GEMM tile boundaries: moe_expert_ffn on hand-made expert_offsets against the oracle.

Run by tests/test_gpu_tiles.py with the default tile capacity and with the capacity pinned to 256 and
to 320 rows through moe_set_tuning.  Row counts sit on and around every boundary of the token tiling: empty experts, 1 row,
one 64-row unit +-1, one tile +-1 for both capacities, several tiles with a short or an almost
full remainder.  Exits non-zero (or raises) on a mismatch.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np
import torch

import paper_2205_10034_amd as M
from oracle import moe_oracle as O
from workloads import WORKLOADS, make_layer
from gpu_util import alloc_ws, rel_fro, tdtype, to_dev, to_np, upload_weights

ROW_SETS = [
    [0, 1, 63, 64, 65, 0, 255, 256, 257, 319, 320, 321],
    [639, 0, 0, 641, 1, 513, 1279, 2],
    [1025, 1087, 1089, 0],
]


def run_case(rows, act, d_model, d_ff, seed, bias=True):
    E = len(rows)
    R = int(sum(rows))
    # a config whose capacity admits these counts: dropless, T*k = R
    wl = WORKLOADS["gpt"].scaled(T=max(R, 1), E=E, k=1, d_model=d_model, d_ff=d_ff, act=act, capacity_factor=0.0,
                                 seed=seed)
    L = make_layer(wl, with_bias=bias)
    cfg = M.MoEConfig.from_workload(wl)
    offsets_np = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    xd_np = L["x"][:R]
    ref = O.expert_ffn(xd_np.astype(np.float64), offsets_np, L, act)
    W = upload_weights(L, "bf16", nullable_bias=True)      # zero biases travel as NULL pointers
    xd = to_dev(xd_np, "bf16")
    yd = torch.full((max(R, 1), d_model), float("nan"), dtype=tdtype("bf16"), device="cuda")
    ws = alloc_ws(cfg, 2)
    offsets = torch.from_numpy(offsets_np).cuda()
    for rep in range(2):  # twice on one workspace: the tile counters must be back at zero for the second call
        yd.fill_(float("nan"))
        M.moe_expert_ffn(cfg, W, xd, offsets, yd, ws)
        torch.cuda.synchronize()
        got = to_np(yd[:R])
        assert np.isfinite(got).all(), f"rows {rows} {act}: rows left unwritten (call {rep})"
        for e in range(E):
            lo, hi = offsets_np[e], offsets_np[e + 1]
            if hi > lo:
                err = rel_fro(got[lo:hi], ref[lo:hi])
                assert err < 1e-2, f"rows {rows} {act} expert {e} ({hi - lo} rows) rel err {err} (call {rep})"
    print(f"ok rows={rows} act={act} d={d_model} f={d_ff} bias={bias}", flush=True)


def main():
    print("tile capacity override:", M.moe_get_tuning(M.MOE_TUNE_GEMM_TILE_ROWS) or "(default)", flush=True)
    for i, rows in enumerate(ROW_SETS):
        run_case(rows, "gelu", 256, 512, 100 + i)
    run_case(ROW_SETS[0], "swiglu", 256, 256, 200)
    run_case(ROW_SETS[1], "gelu", 192, 320, 201)   # narrow-tile kernels
    # K loops of one to five K-steps (the next tile is then resolved outside the K loop), wide and narrow tiles
    for i, (d_model, d_ff) in enumerate([(64, 256), (256, 64), (128, 256), (192, 256), (320, 256), (64, 64)]):
        run_case(ROW_SETS[0], "gelu", d_model, d_ff, 300 + i)
    run_case(ROW_SETS[2], "swiglu", 64, 128, 310)
    # without biases (NULL pointers): the kernels compiled without the bias staging
    run_case(ROW_SETS[0], "gelu", 256, 512, 320, bias=False)
    run_case(ROW_SETS[1], "gelu", 192, 320, 321, bias=False)
    run_case(ROW_SETS[0], "gelu", 64, 256, 322, bias=False)
    return 0


if __name__ == "__main__":
    sys.exit(main())
