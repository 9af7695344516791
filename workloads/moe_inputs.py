"""Seeded synthetic inputs for the MoE-layer forward pass.

The paper measures on trained GPT-MoE and multi-task (UFO) models whose weights
and data are not public (Section 5.2, Section 5.3.1); the five workloads below
stand in for them with random tensors of the same shape class:

* ``tiny``      - correctness case, fp32 everywhere.
* ``gpt``       - GPT-style MoE layer (shape class of Table 2), top-2, capacity 1.25.
* ``skew``      - unbalanced multi-task routing (Section 4.1's load imbalance),
                  top-1, dropless, Zipf(1.2) log-prior on the router bias.
* ``large``     - large SwiGLU experts, top-2, capacity factor 1.0.
* ``ring``      - one layer of the 24-layer stack used for ring memory
                  offloading (Section 3.3.2), 64 experts, top-2, dropless.

Recipe (identical for every workload): draw standard normals in float32 from
``numpy.random.default_rng(seed)`` in a fixed order, scale by the stated
standard deviation, then round once to the storage type (float32 or bfloat16,
round-to-nearest-even).  Arrays handed out are float32 holding exactly
representable values of the storage type, so the GPU path and the oracle see
the same numbers.  No arithmetic of the MoE layer itself lives here.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class MoEWorkload:
    name: str
    T: int                 # tokens
    d_model: int
    d_ff: int
    E: int                 # experts
    k: int                 # experts chosen per token
    capacity_factor: float  # <= 0 means dropless
    renormalize: bool      # top-k weights divided by their sum
    act: str               # "gelu" | "swiglu"
    dtype: str             # "f32" | "bf16": storage type of x, expert weights, outputs
    seed: int
    router_bias: str = "none"   # "none" | "zipf"
    zipf_s: float = 1.2
    zipf_scale: float = 1.0     # multiplies the log-prior bias
    w2_std_scale: float = 1.0   # extra factor on the second matrix's std (ring stack)
    n_layers: int = 1

    def scaled(self, **kw) -> "MoEWorkload":
        return replace(self, **kw)


WORKLOADS: Dict[str, MoEWorkload] = {
    "tiny": MoEWorkload("tiny", 256, 128, 512, 4, 1, 1.25, False, "gelu", "f32", 0),
    "gpt": MoEWorkload("gpt", 8192, 1024, 4096, 16, 2, 1.25, True, "gelu", "bf16", 1),
    "skew": MoEWorkload("skew", 16384, 768, 3072, 8, 1, 0.0, False, "gelu", "bf16", 2,
                        router_bias="zipf"),
    "skew40": MoEWorkload("skew40", 16384, 768, 3072, 8, 1, 0.0, False, "gelu", "bf16", 2,
                          router_bias="zipf", zipf_scale=0.65),
    "large": MoEWorkload("large", 32768, 4096, 14336, 8, 2, 1.0, True, "swiglu", "bf16", 3),
    "ring": MoEWorkload("ring", 4096, 2048, 8192, 64, 2, 0.0, True, "gelu", "bf16", 4000,
                        w2_std_scale=1.0 / np.sqrt(2.0 * 24.0), n_layers=24),
}


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bfloat16 bit patterns, round-to-nearest-even (NaN-free inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16, returned as float32."""
    return (bf16_bits(a).astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(a.shape)


def zipf_masses(E: int, s: float) -> np.ndarray:
    """Normalised Zipf weights (e+1)^-s, e = 0..E-1 (float64)."""
    w = np.arange(1, E + 1, dtype=np.float64) ** (-s)
    return w / w.sum()


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_round(a)
    return np.ascontiguousarray(a, dtype=np.float32)


def _normal(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return _store(a, dtype)


def make_layer(wl: MoEWorkload, seed: Optional[int] = None, with_bias: bool = False,
               x: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Draw one MoE layer's inputs and parameters.

    Returns float32 arrays: ``x[T,d]``, ``w_router[d,E]``, ``b_router[E]`` and
    either ``w1[E,d,f], b1[E,f], w2[E,f,d], b2[E,d]`` (GELU) or
    ``w_gate_proj[E,d,f], w_up[E,d,f], w_down[E,f,d]`` (SwiGLU).  Values of
    ``x`` and of the expert tensors are representable in ``wl.dtype``; the
    router tensors are float32.  Biases are zero unless ``with_bias`` (tests
    use non-zero biases so that a dropped bias term is visible).
    """
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    T, d, f, E = wl.T, wl.d_model, wl.d_ff, wl.E
    out: Dict[str, np.ndarray] = {}
    xs = _normal(rng, (T, d), 1.0, wl.dtype)
    out["x"] = xs if x is None else _store(x, wl.dtype)
    out["w_router"] = _normal(rng, (d, E), d ** -0.5, "f32")
    if wl.router_bias == "zipf":
        out["b_router"] = (wl.zipf_scale * np.log(zipf_masses(E, wl.zipf_s))).astype(np.float32)
    else:
        out["b_router"] = np.zeros(E, dtype=np.float32)
    bstd = 0.5 if with_bias else 0.0
    if wl.act == "gelu":
        out["w1"] = _normal(rng, (E, d, f), d ** -0.5, wl.dtype)
        out["w2"] = _normal(rng, (E, f, d), f ** -0.5 * wl.w2_std_scale, wl.dtype)
        out["b1"] = _normal(rng, (E, f), bstd, wl.dtype)
        out["b2"] = _normal(rng, (E, d), bstd, wl.dtype)
    elif wl.act == "swiglu":
        out["w_gate_proj"] = _normal(rng, (E, d, f), d ** -0.5, wl.dtype)
        out["w_up"] = _normal(rng, (E, d, f), d ** -0.5, wl.dtype)
        out["w_down"] = _normal(rng, (E, f, d), f ** -0.5 * wl.w2_std_scale, wl.dtype)
    else:
        raise ValueError(f"unknown activation {wl.act!r}")
    return out


class RingStackPool:
    """The ring workload's stack of GELU MoE layers, drawn lazily.

    Drawing 24 independent 4 GiB layers costs minutes of host time, so the stack draws ONE pool of
    standard normals of a layer's size plus ``n_layers`` extra elements and gives layer ``l`` the
    window starting at element ``l`` (every layer sees N(0,1) marginals; consecutive layers are
    shifted copies): ``w1`` of layer l is ``pool[l : l + n1]`` as ``[E, d, f]`` times ``d^-1/2``,
    ``w2`` is ``pool[n1 + l : n1 + l + n1]`` as ``[E, f, d]`` times ``f^-1/2 * w2_std_scale``, each
    rounded once to the storage type.  Router weights are drawn independently per layer.
    ``expert(l, e)`` materialises one expert's two matrices; ``layer(l)`` a whole layer.
    """

    def __init__(self, wl: MoEWorkload, n_layers: int, pool_seed: Optional[int] = None):
        assert wl.act == "gelu"
        self.wl, self.n_layers = wl, n_layers
        rng = np.random.default_rng(wl.seed if pool_seed is None else pool_seed)
        T, d, f, E = wl.T, wl.d_model, wl.d_ff, wl.E
        self.x = _normal(rng, (T, d), 1.0, wl.dtype)
        self.n1 = E * d * f
        self.pool = rng.standard_normal(2 * self.n1 + n_layers, dtype=np.float32)
        self.w1_scale = np.float32(d ** -0.5)
        self.w2_scale = np.float32(f ** -0.5 * wl.w2_std_scale)
        self.routers = [_normal(np.random.default_rng([wl.seed, l]), (d, E), d ** -0.5, "f32") for l in range(n_layers)]

    def expert(self, l: int, e: int):
        """(w1[e] as [d, f], w2[e] as [f, d]) of layer l, float32 arrays of storage-representable values."""
        d, f = self.wl.d_model, self.wl.d_ff
        n = d * f
        w1 = _store(self.pool[l + e * n:l + (e + 1) * n] * self.w1_scale, self.wl.dtype).reshape(d, f)
        w2 = _store(self.pool[self.n1 + l + e * n:self.n1 + l + (e + 1) * n] * self.w2_scale, self.wl.dtype).reshape(f, d)
        return w1, w2

    def layer(self, l: int) -> Dict[str, np.ndarray]:
        wl = self.wl
        d, f, E = wl.d_model, wl.d_ff, wl.E
        w1 = _store(self.pool[l:l + self.n1] * self.w1_scale, wl.dtype).reshape(E, d, f)
        w2 = _store(self.pool[self.n1 + l:self.n1 + l + self.n1] * self.w2_scale, wl.dtype).reshape(E, f, d)
        return {"w_router": self.routers[l], "b_router": np.zeros(E, dtype=np.float32), "w1": w1, "w2": w2,
                "b1": np.zeros((E, f), dtype=np.float32), "b2": np.zeros((E, d), dtype=np.float32)}


def make_ring_stack(wl: MoEWorkload, n_layers: int, pool_seed: Optional[int] = None):
    """Parameters for a stack of ``n_layers`` GELU MoE layers sharing one normal pool (see
    :class:`RingStackPool`).  Returns ``(x, layers)`` with ``layers[l]`` a dict like
    :func:`make_layer`'s (without ``x``)."""
    pool = RingStackPool(wl, n_layers, pool_seed)
    return pool.x, [pool.layer(l) for l in range(n_layers)]
