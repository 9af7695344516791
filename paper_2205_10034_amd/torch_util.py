"""Device-memory plumbing around the binding: upload a layer's parameters, allocate and view a workspace.

torch supplies device memory only; nothing here computes any part of the layer (the one kernel call is the
library's own weight transpose, which prepares the output-major layout the bf16 kernels read).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as M

EXPERT_MATS = ("w1", "w2", "w_gate_proj", "w_up", "w_down")


def tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 array of representable values -> device tensor of the storage dtype (exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(tdtype(dtype)).contiguous()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def upload_weights(L: dict, dtype: str, layout: str = "output_major", nullable_bias: bool = False,
                   pack_router: bool = True) -> M.Weights:
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
                torch.cuda.synchronize()
                del src
            else:
                t[name] = src
    for name in ("b1", "b2"):
        if name in L and L[name] is not None:
            if nullable_bias and not np.any(L[name]):
                continue
            t[name] = to_dev(L[name], dtype)
    t["w_router"] = to_dev(L["w_router"], "f32")
    n = M.moe_router_pack_bytes(*t["w_router"].shape) if (dtype == "bf16" and pack_router) else 0
    if n:   # the gate's pre-split copy of the router (one-time preparation, like the transposes above)
        t["w_router_packed"] = torch.empty(n, dtype=torch.uint8, device="cuda")
        M.moe_pack_router(t["w_router"], t["w_router_packed"])
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
