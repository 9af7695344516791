"""Helpers for the GPU parity tests: upload a seeded workload, run stages through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_2205_10034_amd as M

from paper_2205_10034_amd.torch_util import (  # noqa: F401  (re-exported for the tests)
    EXPERT_MATS, alloc_ws, tdtype, to_dev, to_np, upload_weights, ws_view,
)


def run_layer(cfg: M.MoEConfig, W: M.Weights, x: torch.Tensor, residual=None):
    """moe_layer_forward; returns out and every intermediate read back from the workspace."""
    ws = alloc_ws(cfg)
    ws.zero_()
    out = torch.empty_like(x)
    M.moe_layer_forward(cfg, W, x, residual, out, ws)
    torch.cuda.synchronize()
    L = M.moe_workspace_layout(cfg)
    A = cfg.k * cfg.T
    dt = tdtype(cfg.dtype)
    r = {"out": to_np(out)}
    r["topk_idx"] = ws_view(ws, L["topk_idx"], A, torch.int32).cpu().numpy().reshape(cfg.T, cfg.k)
    r["topk_w"] = ws_view(ws, L["topk_w"], A, torch.float32).cpu().numpy().reshape(cfg.T, cfg.k)
    r["expert_counts"] = ws_view(ws, L["expert_counts"], cfg.E, torch.int32).cpu().numpy()
    r["expert_offsets"] = ws_view(ws, L["expert_offsets"], cfg.E + 1, torch.int32).cpu().numpy()
    r["assign_to_row"] = ws_view(ws, L["assign_to_row"], A, torch.int32).cpu().numpy()
    R = int(r["expert_offsets"][-1])
    r["row_to_assign"] = ws_view(ws, L["row_to_assign"], A, torch.int32).cpu().numpy()[:R]
    # (bf16: the xd segment is empty; with k = 1 so is yd)
    for name, nxt in (("xd", "h"), ("yd", "scratch")):
        if L[nxt] - L[name] >= L["r_max"] * cfg.d_model * ws_view(ws, 0, 1, dt).element_size() and L["r_max"]:
            r[name] = to_np(ws_view(ws, L[name], L["r_max"] * cfg.d_model, dt).reshape(L["r_max"], cfg.d_model)[:R])
    r["out_tensor"] = out
    return r


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    """||a-b||_F / ||b||_F (0 if both empty/zero)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    num = np.linalg.norm(a - b)
    return float(num / den) if den > 0 else float(num)

