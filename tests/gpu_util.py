"""Helpers for the GPU parity tests: upload a seeded workload, run stages through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_2205_10034_amd as M

EXPERT_MATS = ("w1", "w2", "w_gate_proj", "w_up", "w_down")


def tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 array of representable values -> device tensor of the storage dtype (exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(tdtype(dtype)).contiguous()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def upload_weights(L: dict, dtype: str, layout: str = "output_major", nullable_bias: bool = False) -> M.Weights:
    """Expert matrices arrive input-major ([E,in,out]); output-major copies are made on the device
    with the library's own transpose kernel."""
    t = {}
    for name in EXPERT_MATS:
        if name in L and L[name] is not None:
            src = to_dev(L[name], dtype)
            if layout == "output_major":
                dst = torch.empty((src.shape[0], src.shape[2], src.shape[1]), dtype=src.dtype, device="cuda")
                M.moe_transpose_expert_weights(src, dst)
                t[name] = dst
            else:
                t[name] = src
    for name in ("b1", "b2"):
        if name in L and L[name] is not None:
            if nullable_bias and not np.any(L[name]):
                continue
            t[name] = to_dev(L[name], dtype)
    t["w_router"] = to_dev(L["w_router"], "f32")
    if L.get("b_router") is not None:
        t["b_router"] = to_dev(L["b_router"], "f32")
    torch.cuda.synchronize()
    return M.Weights(t, layout)


def alloc_ws(cfg: M.MoEConfig, kind: int = 0) -> torch.Tensor:
    n = M.moe_workspace_bytes(cfg, kind)
    return torch.empty(n + 256, dtype=torch.uint8, device="cuda")[:n] if n else torch.empty(256, dtype=torch.uint8, device="cuda")


def ws_view(ws: torch.Tensor, off: int, count: int, dtype) -> torch.Tensor:
    nbytes = count * torch.empty((), dtype=dtype).element_size()
    return ws[off:off + nbytes].view(dtype)


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
    r["xd"] = to_np(ws_view(ws, L["xd"], L["r_max"] * cfg.d_model, dt).reshape(L["r_max"], cfg.d_model)[:R])
    r["yd"] = to_np(ws_view(ws, L["yd"], L["r_max"] * cfg.d_model, dt).reshape(L["r_max"], cfg.d_model)[:R])
    r["out_tensor"] = out
    return r


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    """||a-b||_F / ||b||_F (0 if both empty/zero)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    num = np.linalg.norm(a - b)
    return float(num / den) if den > 0 else float(num)
