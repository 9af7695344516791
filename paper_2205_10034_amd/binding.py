"""ctypes binding of libmoesys_hip.so: argument marshalling only.

Every function has the name and meaning of its C counterpart in
``include/moesys.h``.  Tensors are torch CUDA tensors (torch supplies device
memory and streams, nothing else); bf16 tensors are ``torch.bfloat16``.  If the
library has not been built the import of :func:`lib` fails loudly - there is no
CPU or eager fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libmoesys_hip.so")
_lib = None

MOE_F32, MOE_BF16 = 0, 1
MOE_ACT_GELU, MOE_ACT_SWIGLU = 0, 1
MOE_LAYOUT_INPUT_MAJOR, MOE_LAYOUT_OUTPUT_MAJOR = 0, 1
MOE_WS_LAYER, MOE_WS_DISPATCH, MOE_WS_FFN = 0, 1, 2
MOE_DROPLESS = 2 ** 31 - 1
STAGE_NAMES = ["gate", "dispatch", "gemm1", "gemm2", "combine"]


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__(f"{where}: status {status}: {detail}")
        self.status = status


class _Config(C.Structure):
    _fields_ = [("T", C.c_int32), ("d_model", C.c_int32), ("d_ff", C.c_int32), ("E", C.c_int32),
                ("k", C.c_int32), ("capacity_factor", C.c_float), ("renormalize", C.c_int32),
                ("act", C.c_int32), ("dtype", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p),
                ("w_gate_proj", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p),
                ("w_router", C.c_void_p), ("b_router", C.c_void_p), ("layout", C.c_int32),
                ("expert_elem_offset", C.c_void_p), ("w_router_packed", C.c_void_p)]


class _WsLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("topk_idx", "topk_w", "expert_counts", "expert_offsets",
                                          "assign_to_row", "row_to_assign", "xd", "h", "yd", "scratch",
                                          "tile_counters", "total")] + [("r_max", C.c_int64)]


RING_COPY_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p)
RING_EVCREATE_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.POINTER(C.c_void_p))
RING_EV_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_void_p)
RING_EV2_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p)
RING_ELAPSED_FN = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_float))


class RingBackend(C.Structure):
    _fields_ = [("user", C.c_void_p), ("copy_h2d_async", RING_COPY_FN), ("event_create", RING_EVCREATE_FN),
                ("event_destroy", RING_EV_FN), ("event_record", RING_EV2_FN), ("stream_wait_event", RING_EV2_FN),
                ("event_synchronize", RING_EV_FN), ("event_elapsed_ms", RING_ELAPSED_FN)]


def lib_path() -> str:
    return _LIB_PATH


def use_library(path: str) -> None:
    """Selects another build of the library (the phase-timing build) before the first call; diagnostics only."""
    global _LIB_PATH
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    _LIB_PATH = path


def lib() -> C.CDLL:
    """Loads the built library; raises if it is missing (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is not built: run `python -m paper_2205_10034_amd.build`")
        # torch brings its own copy of the HIP runtime; it has to be the first one in the process, so that
        # this library binds to the same runtime (and the same device context) as the tensors it is handed
        import torch  # noqa: F401
        L = C.CDLL(_LIB_PATH)
        L.moe_status_string.restype = C.c_char_p
        L.moe_status_string.argtypes = [C.c_int32]
        L.moe_last_error.restype = C.c_char_p
        L.moe_version.restype = C.c_int32
        L.moe_config_check.argtypes = [C.POINTER(_Config)]
        L.moe_capacity.argtypes = [C.POINTER(_Config)]
        L.moe_workspace_bytes.restype = C.c_size_t
        L.moe_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int32]
        L.moe_workspace_layout.argtypes = [C.POINTER(_Config), C.POINTER(_WsLayout)]
        vp = C.c_void_p
        L.moe_gate.argtypes = [C.POINTER(_Config)] + [vp] * 7
        L.moe_router_pack_bytes.restype = C.c_size_t
        L.moe_router_pack_bytes.argtypes = [C.c_int32, C.c_int32]
        L.moe_pack_router.argtypes = [vp, vp, C.c_int32, C.c_int32, vp]
        L.moe_gate_packed.argtypes = [C.POINTER(_Config)] + [vp] * 8
        L.moe_dispatch.argtypes = [C.POINTER(_Config)] + [vp] * 8 + [C.c_size_t, vp]
        L.moe_dispatch_static.argtypes = [C.POINTER(_Config)] + [vp] * 8
        L.moe_expert_ffn.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), vp, vp, vp, vp, C.c_size_t, vp]
        L.moe_combine.argtypes = [C.POINTER(_Config)] + [vp] * 6
        L.moe_layer_forward.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), vp, vp, vp, vp, C.c_size_t, vp]
        L.moe_layer_route.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), vp, vp, C.c_size_t, vp]
        L.moe_layer_experts.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), vp, vp, vp, vp, C.c_size_t, vp]
        L.moe_layer_forward_timed.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), vp, vp, vp, vp, C.c_size_t, vp, vp]
        L.moe_timer_create.argtypes = [C.POINTER(vp)]
        L.moe_timer_destroy.argtypes = [vp]
        L.moe_timer_read.argtypes = [vp, C.POINTER(C.c_float)]
        L.moe_transpose_expert_weights.argtypes = [vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        L.moe_ring_create.argtypes = [vp, C.c_size_t, C.c_int32, C.POINTER(vp), C.c_int32, C.c_size_t, vp,
                                      C.POINTER(RingBackend), C.POINTER(vp)]
        L.moe_ring_acquire.argtypes = [vp, C.c_int32, vp, C.POINTER(vp)]
        L.moe_ring_release.argtypes = [vp, C.c_int32, vp]
        L.moe_ring_stats.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_double)]
        L.moe_ring_destroy.argtypes = [vp]
        L.moe_expert_cache_create.argtypes = [C.POINTER(vp), C.c_int32, C.c_float, C.c_float, C.c_int32]
        L.moe_expert_cache_destroy.argtypes = [vp]
        L.moe_expert_cache_begin_batch.argtypes = [vp]
        L.moe_expert_cache_schedule.argtypes = [vp, C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                                C.POINTER(C.c_int64)]
        L.moe_expert_cache_lookup.argtypes = [vp, C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        L.moe_expert_cache_stats.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.moe_combine_backward.argtypes = [C.POINTER(_Config)] + [vp] * 7
        L.moe_expert_ffn_backward_workspace_bytes.restype = C.c_size_t
        L.moe_expert_ffn_backward_workspace_bytes.argtypes = [C.POINTER(_Config)]
        L.moe_expert_ffn_backward.argtypes = [C.POINTER(_Config), C.POINTER(_Weights)] + [vp] * 11 + [C.c_int32, vp, C.c_size_t, vp]
        L.moe_layer_backward_workspace_bytes.restype = C.c_size_t
        L.moe_layer_backward_workspace_bytes.argtypes = [C.POINTER(_Config)]
        L.moe_layer_backward.argtypes = ([C.POINTER(_Config), C.POINTER(_Weights)] + [vp] * 5 + [C.c_float, vp, C.c_size_t] +
                                         [vp] * 7 + [C.c_int32, vp, C.c_size_t, vp])
        L.moe_gate_aux_loss.argtypes = [C.POINTER(_Config), vp, vp, C.c_float, vp, vp, vp, vp]
        L.moe_expert_wgrad.argtypes = [vp, vp, vp, vp, C.c_int32, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int64, vp]
        L.moe_expert_pool_create.argtypes = [vp, C.c_size_t, C.c_size_t, C.POINTER(vp), C.c_int32, C.c_int32, C.c_size_t,
                                             C.c_float, C.c_float, C.c_int32, vp, C.POINTER(vp)]
        L.moe_expert_pool_prepare.argtypes = [vp, C.c_int32, vp, C.c_int32, vp, vp]
        L.moe_expert_pool_prefetch.argtypes = [vp, C.c_int32, vp, vp, C.POINTER(C.c_int32)]
        L.moe_expert_pool_stats.argtypes = [vp] + [C.POINTER(C.c_uint64)] * 5
        L.moe_expert_pool_destroy.argtypes = [vp]
        L.moe_set_tuning.argtypes = [C.c_int32, C.c_int32]
        L.moe_get_tuning.argtypes = [C.c_int32, C.POINTER(C.c_int32)]
        _lib = L
    return _lib


def _check(st: int, where: str) -> None:
    if st != 0:
        raise MoEError(st, where, lib().moe_last_error().decode())


@dataclass
class MoEConfig:
    T: int
    d_model: int
    d_ff: int
    E: int
    k: int
    capacity_factor: float = 0.0
    renormalize: bool = False
    act: str = "gelu"
    dtype: str = "bf16"

    def c(self) -> _Config:
        return _Config(self.T, self.d_model, self.d_ff, self.E, self.k, float(self.capacity_factor),
                       int(bool(self.renormalize)), {"gelu": 0, "swiglu": 1}[self.act],
                       {"f32": 0, "bf16": 1}[self.dtype])

    @staticmethod
    def from_workload(wl, **kw) -> "MoEConfig":
        d = dict(T=wl.T, d_model=wl.d_model, d_ff=wl.d_ff, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                 renormalize=wl.renormalize, act=wl.act, dtype=wl.dtype)
        d.update(kw)
        return MoEConfig(**d)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return t.data_ptr()


def _need(t, nbytes: int, what: str) -> None:
    """The library takes plain pointers and trusts the configuration for what lies behind them: a tensor of the wrong
    dtype or shape (bfloat16 tensors under a float32 configuration, say) would be read or written past its end on the
    device.  Every tensor the binding knows the size of is therefore checked here, on the host, before the call."""
    if t is None or isinstance(t, int):
        return
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise ValueError(f"{what} holds {have} bytes, the configuration needs {nbytes} (wrong dtype or shape?)")


def _esize(cfg) -> int:
    return {"f32": 4, "bf16": 2}[cfg.dtype]


def _need_tokens(cfg, **tensors) -> None:
    for name, t in tensors.items():
        _need(t, cfg.T * cfg.d_model * _esize(cfg), name)


def _need_routing(cfg, topk_idx=None, topk_w=None, probs=None, assign_to_row=None, row_to_assign=None,
                  expert_counts=None, expert_offsets=None) -> None:
    A = cfg.k * cfg.T
    _need(topk_idx, 4 * A, "topk_idx")
    _need(topk_w, 4 * A, "topk_w")
    _need(probs, 4 * cfg.T * cfg.E, "probs")
    _need(assign_to_row, 4 * A, "assign_to_row")
    _need(expert_counts, 4 * cfg.E, "expert_counts")
    _need(expert_offsets, 4 * (cfg.E + 1), "expert_offsets")


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


class Weights:
    """Device pointers of one layer's parameters (keeps the tensors alive)."""

    def __init__(self, tensors: Dict[str, "object"], layout: str = "output_major"):
        self.tensors = dict(tensors)
        self.layout = layout
        g = lambda n: _ptr(self.tensors.get(n))
        self.c = _Weights(g("w1"), g("b1"), g("w2"), g("b2"), g("w_gate_proj"), g("w_up"), g("w_down"),
                          g("w_router"), g("b_router"),
                          MOE_LAYOUT_OUTPUT_MAJOR if layout == "output_major" else MOE_LAYOUT_INPUT_MAJOR,
                          g("expert_elem_offset"), g("w_router_packed"))

    def need(self, cfg) -> None:
        """Raises ValueError if a parameter tensor is smaller than `cfg` says (see _need)."""
        t, s = self.tensors, _esize(cfg)
        E, d, f = cfg.E, cfg.d_model, cfg.d_ff
        _need(t.get("w_router"), 4 * d * E, "w_router")
        _need(t.get("b_router"), 4 * E, "b_router")
        _need(t.get("w_router_packed"), moe_router_pack_bytes(d, E) if t.get("w_router_packed") is not None else 0,
              "w_router_packed")
        _need(t.get("expert_elem_offset"), 8 * E, "expert_elem_offset")
        if t.get("expert_elem_offset") is None:  # (with per-expert offsets the matrices are pools of any size)
            for n in ("w1", "w2", "w_gate_proj", "w_up", "w_down"):
                _need(t.get(n), E * d * f * s, n)
            _need(t.get("b1"), E * f * s, "b1")
            _need(t.get("b2"), E * d * s, "b2")


MOE_TUNE_GEMM_TILE_ROWS, MOE_TUNE_FEW_TOKEN_KERNELS, MOE_TUNE_GATE_TOKENS, MOE_TUNE_GEMM_MFMA = 0, 1, 2, 3


def moe_set_tuning(key: int, value: int) -> None:
    _check(lib().moe_set_tuning(key, value), "moe_set_tuning")


def moe_get_tuning(key: int) -> int:
    v = C.c_int32()
    _check(lib().moe_get_tuning(key, C.byref(v)), "moe_get_tuning")
    return v.value


def moe_capacity(cfg: MoEConfig) -> int:
    c = cfg.c()
    v = lib().moe_capacity(C.byref(c))
    if v < 0:
        _check(lib().moe_config_check(C.byref(c)), "moe_capacity")
    return v


def moe_workspace_bytes(cfg: MoEConfig, kind: int = MOE_WS_LAYER) -> int:
    c = cfg.c()
    v = lib().moe_workspace_bytes(C.byref(c), kind)
    if v == 0:
        _check(lib().moe_config_check(C.byref(c)), "moe_workspace_bytes")
    return v


def moe_workspace_layout(cfg: MoEConfig) -> Dict[str, int]:
    c, L = cfg.c(), _WsLayout()
    _check(lib().moe_workspace_layout(C.byref(c), C.byref(L)), "moe_workspace_layout")
    return {n: getattr(L, n) for n, _ in _WsLayout._fields_}


def moe_gate(cfg, x, w_router, b_router, topk_idx, topk_w, probs=None, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x)
    _need(w_router, 4 * cfg.d_model * cfg.E, "w_router")
    _need(b_router, 4 * cfg.E, "b_router")
    _need_routing(cfg, topk_idx=topk_idx, topk_w=topk_w, probs=probs)
    _check(lib().moe_gate(C.byref(c), _ptr(x), _ptr(w_router), _ptr(b_router), _ptr(topk_idx), _ptr(topk_w),
                          _ptr(probs), _stream(stream)), "moe_gate")


def moe_router_pack_bytes(d_model: int, E: int) -> int:
    return lib().moe_router_pack_bytes(d_model, E)


def moe_pack_router(w_router, packed, stream=None):
    """packed <- w_router [d_model, E] (float32) split into bfloat16 pieces in the gate's operand order."""
    d, E = w_router.shape
    _check(lib().moe_pack_router(_ptr(w_router), _ptr(packed), d, E, _stream(stream)), "moe_pack_router")


def moe_gate_packed(cfg, x, w_router, b_router, w_router_packed, topk_idx, topk_w, probs=None, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x)
    _need(w_router, 4 * cfg.d_model * cfg.E, "w_router")
    _need(b_router, 4 * cfg.E, "b_router")
    _need(w_router_packed, moe_router_pack_bytes(cfg.d_model, cfg.E), "w_router_packed")
    _need_routing(cfg, topk_idx=topk_idx, topk_w=topk_w, probs=probs)
    _check(lib().moe_gate_packed(C.byref(c), _ptr(x), _ptr(w_router), _ptr(b_router), _ptr(w_router_packed), _ptr(topk_idx),
                                 _ptr(topk_w), _ptr(probs), _stream(stream)), "moe_gate_packed")


def moe_dispatch(cfg, x, topk_idx, expert_counts, expert_offsets, assign_to_row, row_to_assign, xd, ws,
                 stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x)
    _need_routing(cfg, topk_idx=topk_idx, assign_to_row=assign_to_row, row_to_assign=None, expert_counts=expert_counts,
                  expert_offsets=expert_offsets)
    _check(lib().moe_dispatch(C.byref(c), _ptr(x), _ptr(topk_idx), _ptr(expert_counts), _ptr(expert_offsets),
                              _ptr(assign_to_row), _ptr(row_to_assign), _ptr(xd), _ptr(ws),
                              ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "moe_dispatch")


def moe_dispatch_static(cfg, x, topk_idx, expert_counts, expert_offsets, assign_to_row, row_to_assign, xd, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x)
    _need_routing(cfg, topk_idx=topk_idx, assign_to_row=assign_to_row, expert_counts=expert_counts,
                  expert_offsets=expert_offsets)
    _check(lib().moe_dispatch_static(C.byref(c), _ptr(x), _ptr(topk_idx), _ptr(expert_counts), _ptr(expert_offsets),
                                     _ptr(assign_to_row), _ptr(row_to_assign), _ptr(xd), _stream(stream)),
           "moe_dispatch_static")


def moe_expert_ffn(cfg, weights: Weights, xd, expert_offsets, yd, ws, stream=None):
    c = cfg.c()
    weights.need(cfg)
    _need_routing(cfg, expert_offsets=expert_offsets)
    _check(lib().moe_expert_ffn(C.byref(c), C.byref(weights.c), _ptr(xd), _ptr(expert_offsets), _ptr(yd), _ptr(ws),
                                ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "moe_expert_ffn")


def moe_combine(cfg, yd, assign_to_row, topk_w, residual, out, stream=None):
    c = cfg.c()
    _need_tokens(cfg, residual=residual, out=out)
    _need_routing(cfg, topk_w=topk_w, assign_to_row=assign_to_row)
    _check(lib().moe_combine(C.byref(c), _ptr(yd), _ptr(assign_to_row), _ptr(topk_w), _ptr(residual), _ptr(out),
                             _stream(stream)), "moe_combine")


def moe_layer_forward(cfg, weights: Weights, x, residual, out, ws, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x, residual=residual, out=out)
    weights.need(cfg)
    _check(lib().moe_layer_forward(C.byref(c), C.byref(weights.c), _ptr(x), _ptr(residual), _ptr(out), _ptr(ws),
                                   ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "moe_layer_forward")


def moe_layer_route(cfg, weights: Weights, x, ws, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x)
    weights.need(cfg)
    _check(lib().moe_layer_route(C.byref(c), C.byref(weights.c), _ptr(x), _ptr(ws),
                                 ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "moe_layer_route")


def moe_layer_experts(cfg, weights: Weights, x, residual, out, ws, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x, residual=residual, out=out)
    weights.need(cfg)
    _check(lib().moe_layer_experts(C.byref(c), C.byref(weights.c), _ptr(x), _ptr(residual), _ptr(out), _ptr(ws),
                                   ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "moe_layer_experts")


def moe_combine_backward(cfg, d_out, yd, assign_to_row, topk_w, d_yd, d_topk_w, stream=None):
    c = cfg.c()
    _check(lib().moe_combine_backward(C.byref(c), _ptr(d_out), _ptr(yd), _ptr(assign_to_row), _ptr(topk_w), _ptr(d_yd),
                                      _ptr(d_topk_w), _stream(stream)), "moe_combine_backward")


def moe_expert_ffn_backward_workspace_bytes(cfg) -> int:
    c = cfg.c()
    return lib().moe_expert_ffn_backward_workspace_bytes(C.byref(c))


def _grad_dtype(*tensors) -> int:
    """MOE_F32 or MOE_BF16 from the element size of the weight-gradient tensors (which must agree)."""
    sizes = {t.element_size() for t in tensors if t is not None}
    if len(sizes) > 1:
        raise ValueError("the weight gradients must have one element type")
    return MOE_BF16 if sizes == {2} else MOE_F32


def moe_expert_ffn_backward(cfg, weights: Weights, w1_input_major, w2_input_major, xd, h, d_yd, expert_offsets, d_xd,
                            d_w1, d_b1, d_w2, d_b2, ws, stream=None):
    c = cfg.c()
    _check(lib().moe_expert_ffn_backward(C.byref(c), C.byref(weights.c), _ptr(w1_input_major), _ptr(w2_input_major),
                                         _ptr(xd), _ptr(h), _ptr(d_yd), _ptr(expert_offsets), _ptr(d_xd), _ptr(d_w1),
                                         _ptr(d_b1), _ptr(d_w2), _ptr(d_b2), _grad_dtype(d_w1, d_w2), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)), "moe_expert_ffn_backward")


def moe_layer_backward_workspace_bytes(cfg) -> int:
    c = cfg.c()
    return lib().moe_layer_backward_workspace_bytes(C.byref(c))


def moe_layer_backward(cfg, weights: Weights, w1_input_major, w2_input_major, x, d_out, add_to_d_x, fwd_ws, d_x,
                       d_w_router, d_b_router, d_w1, d_b1, d_w2, d_b2, ws, stream=None, aux_loss_coef: float = 0.0):
    c = cfg.c()
    _need_tokens(cfg, x=x, d_out=d_out, add_to_d_x=add_to_d_x, d_x=d_x)
    weights.need(cfg)
    _need(d_w_router, 4 * cfg.d_model * cfg.E, "d_w_router")
    _need(d_b_router, 4 * cfg.E, "d_b_router")
    _check(lib().moe_layer_backward(C.byref(c), C.byref(weights.c), _ptr(w1_input_major), _ptr(w2_input_major), _ptr(x),
                                    _ptr(d_out), _ptr(add_to_d_x), aux_loss_coef, _ptr(fwd_ws),
                                    fwd_ws.numel() * fwd_ws.element_size(),
                                    _ptr(d_x), _ptr(d_w_router), _ptr(d_b_router), _ptr(d_w1), _ptr(d_b1), _ptr(d_w2),
                                    _ptr(d_b2), _grad_dtype(d_w1, d_w2), _ptr(ws), ws.numel() * ws.element_size(),
                                    _stream(stream)),
           "moe_layer_backward")


def moe_gate_aux_loss(cfg, probs, topk_idx, coef: float, expert_fraction, mean_prob, loss, stream=None):
    c = cfg.c()
    _check(lib().moe_gate_aux_loss(C.byref(c), _ptr(probs), _ptr(topk_idx), coef, _ptr(expert_fraction), _ptr(mean_prob),
                                   _ptr(loss), _stream(stream)), "moe_gate_aux_loss")


def moe_expert_wgrad(a, b, expert_offsets, c, max_rows_per_expert: int, stream=None, a_column_sums=None):
    """c[e] = a[rows of e]^T @ b[rows of e]; a [R,N1], b [R,N2] bf16, c [E,N1,N2] float32 or bfloat16; a_column_sums
    [E,N1] float32 (optional): sum over the rows of e of a."""
    E, N1, N2 = c.shape
    _check(lib().moe_expert_wgrad(_ptr(a), _ptr(b), _ptr(expert_offsets), _ptr(c), _grad_dtype(c), _ptr(a_column_sums), E, N1, N2,
                                  max_rows_per_expert, _stream(stream)), "moe_expert_wgrad")


class StageTimer:
    def __init__(self):
        self.h = C.c_void_p()
        _check(lib().moe_timer_create(C.byref(self.h)), "moe_timer_create")

    def read(self) -> List[float]:
        arr = (C.c_float * len(STAGE_NAMES))()
        _check(lib().moe_timer_read(self.h, arr), "moe_timer_read")
        return list(arr)

    def close(self):
        if self.h:
            lib().moe_timer_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_layer_forward_timed(cfg, weights: Weights, x, residual, out, ws, timer: StageTimer, stream=None):
    c = cfg.c()
    _need_tokens(cfg, x=x, residual=residual, out=out)
    weights.need(cfg)
    _check(lib().moe_layer_forward_timed(C.byref(c), C.byref(weights.c), _ptr(x), _ptr(residual), _ptr(out),
                                         _ptr(ws), ws.numel() * ws.element_size(), _stream(stream), timer.h),
           "moe_layer_forward_timed")


def moe_transpose_expert_weights(src, dst, stream=None):
    """dst[e,c,r] = src[e,r,c] for a 3-D tensor [E, rows, cols]."""
    import torch
    E, rows, cols = src.shape
    dt = MOE_BF16 if src.dtype == torch.bfloat16 else MOE_F32
    _check(lib().moe_transpose_expert_weights(_ptr(src), _ptr(dst), E, rows, cols, dt, _stream(stream)),
           "moe_transpose_expert_weights")


class Ring:
    """moe_ring_* wrapper.  ``host_layers`` are pinned host tensors (or raw addresses with a custom backend)."""

    def __init__(self, dev_base, budget_bytes: int, n_sections: int, host_layers: Sequence, layer_bytes: int,
                 copy_stream=None, backend: Optional[RingBackend] = None):
        self._keep = (dev_base, list(host_layers), copy_stream, backend)
        ptrs = (C.c_void_p * len(host_layers))(*[h if isinstance(h, int) else h.data_ptr() for h in host_layers])
        self.h = C.c_void_p()
        cs = None if copy_stream is None else (copy_stream if isinstance(copy_stream, int) else copy_stream.cuda_stream)
        base = dev_base if isinstance(dev_base, int) else dev_base.data_ptr()
        _check(lib().moe_ring_create(base, budget_bytes, n_sections, ptrs, len(host_layers), layer_bytes, cs,
                                     C.byref(backend) if backend is not None else None, C.byref(self.h)),
               "moe_ring_create")

    def acquire(self, layer: int, compute_stream=None) -> int:
        p = C.c_void_p()
        s = compute_stream if isinstance(compute_stream, int) else _stream(compute_stream)
        _check(lib().moe_ring_acquire(self.h, layer, s, C.byref(p)), "moe_ring_acquire")
        return p.value

    def release(self, layer: int, compute_stream=None) -> None:
        s = compute_stream if isinstance(compute_stream, int) else _stream(compute_stream)
        _check(lib().moe_ring_release(self.h, layer, s), "moe_ring_release")

    def stats(self):
        b, n, ms = C.c_uint64(), C.c_uint64(), C.c_double()
        _check(lib().moe_ring_stats(self.h, C.byref(b), C.byref(n), C.byref(ms)), "moe_ring_stats")
        return {"bytes_copied": b.value, "copies": n.value, "copy_ms": ms.value}

    def close(self):
        if self.h:
            lib().moe_ring_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ExpertCache:
    """moe_expert_cache_* wrapper: the frequency-based residency policy (host only)."""

    def __init__(self, slots: int, threshold: float, beta: float, decay_steps: int):
        self.h = C.c_void_p()
        _check(lib().moe_expert_cache_create(C.byref(self.h), slots, threshold, beta, decay_steps),
               "moe_expert_cache_create")

    def begin_batch(self) -> None:
        _check(lib().moe_expert_cache_begin_batch(self.h), "moe_expert_cache_begin_batch")

    def schedule(self, item: int):
        """-> (slot, hit, evicted item or -1)"""
        slot, hit, gone = C.c_int32(), C.c_int32(), C.c_int64()
        _check(lib().moe_expert_cache_schedule(self.h, item, C.byref(slot), C.byref(hit), C.byref(gone)),
               "moe_expert_cache_schedule")
        return slot.value, bool(hit.value), gone.value

    def lookup(self, item: int):
        """-> (slot or -1, hit count)"""
        slot, hits = C.c_int32(), C.c_double()
        _check(lib().moe_expert_cache_lookup(self.h, item, C.byref(slot), C.byref(hits)), "moe_expert_cache_lookup")
        return slot.value, hits.value

    def stats(self):
        h, m, e = C.c_uint64(), C.c_uint64(), C.c_uint64()
        _check(lib().moe_expert_cache_stats(self.h, C.byref(h), C.byref(m), C.byref(e)), "moe_expert_cache_stats")
        return {"hits": h.value, "misses": m.value, "evictions": e.value}

    def close(self):
        if self.h:
            lib().moe_expert_cache_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ExpertPool:
    """moe_expert_pool_* wrapper.  ``host_blobs``: pinned host tensors, one per (layer, expert), layer-major."""

    def __init__(self, dev_pool, slot_bytes: int, host_blobs: Sequence, n_layers: int, E: int, blob_bytes: int,
                 threshold: float, beta: float, decay_steps: int, copy_stream=None):
        self._keep = (dev_pool, list(host_blobs), copy_stream)
        ptrs = (C.c_void_p * len(host_blobs))(*[h.data_ptr() for h in host_blobs])
        self.h = C.c_void_p()
        cs = None if copy_stream is None else copy_stream.cuda_stream
        _check(lib().moe_expert_pool_create(dev_pool.data_ptr(), dev_pool.numel() * dev_pool.element_size(), slot_bytes,
                                            ptrs, n_layers, E, blob_bytes, threshold, beta, decay_steps, cs,
                                            C.byref(self.h)), "moe_expert_pool_create")

    def prepare(self, layer: int, counts_dev, elem_bytes: int, dev_offsets, compute_stream=None) -> None:
        _check(lib().moe_expert_pool_prepare(self.h, layer, _ptr(counts_dev), elem_bytes, _ptr(dev_offsets),
                                             _stream(compute_stream)), "moe_expert_pool_prepare")

    def prefetch(self, layer: int, counts_dev, stream=None) -> int:
        """Enqueue the copies of the guessed experts of ``layer`` that are not resident; returns how many."""
        n = C.c_int32()
        _check(lib().moe_expert_pool_prefetch(self.h, layer, _ptr(counts_dev), _stream(stream), C.byref(n)),
               "moe_expert_pool_prefetch")
        return n.value

    def stats(self):
        v = [C.c_uint64() for _ in range(5)]
        _check(lib().moe_expert_pool_stats(self.h, *[C.byref(x) for x in v]), "moe_expert_pool_stats")
        return dict(zip(("bytes_copied", "copies", "hits", "misses", "evictions"), [x.value for x in v]))

    def close(self):
        if self.h:
            lib().moe_expert_pool_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
