"""CPU oracle for the sparsely-gated MoE layer forward pass (TEST INFRASTRUCTURE).

This file is the checker, not the product: only ``tests/``, the smoke check and
the bench's ``cpu_baseline`` leg may import it.  It shares no code with the HIP
path and must never be called from the product package.

What it computes.  The paper names the layer but does not write its equations:
the experts are the "switching feed-forward network (FFN) layer" whose
parameters are sparsely activated (Section 3.2), the gates evaluated are GShard
(top-2) and top-1 gating (Section 5.2), and softmax is one of the operations
kept in fp32 while parameters are 16-bit (Section 5.2).  The definitions below
are therefore the standard ones of those cited gate families, written out
plainly in float64 with NumPy; every choice the paper leaves open is listed in
the repository's design notes and repeated at the function that takes it.

Everything is float64 and unblocked: one ``numpy.matmul`` per contraction, one
loop over experts, nothing fused or reordered, so the code can be read against
the definition by eye.

Pins (tests marked "not gpu"): brute-force top-k and slotting on tiny inputs
with constructed ties and overflow; probability / weight normalisation;
capacity closed forms; single expert == dense FFN and k == E == full softmax
mixture, both against torch's library softmax / gelu / silu / linear; identity
experts with top-1 return the gate-weighted input; infinite capacity ==
dropless; token permutation equivariance; ring schedule invariants from
Section 3.3.2.  No function here is "parity unpinned".
"""
from __future__ import annotations

from fractions import Fraction
from typing import Dict, List, Optional, Tuple

import numpy as np
from scipy.special import erf

DROPLESS = 2 ** 31 - 1


# --------------------------------------------------------------------------- gate
def gate_logits(x: np.ndarray, w_router: np.ndarray, b_router: Optional[np.ndarray]) -> np.ndarray:
    """z[t,e] = sum_i x[t,i] * W_g[i,e] + b_g[e]   (router of the top-k gates of Section 5.2)."""
    z = np.matmul(np.asarray(x, dtype=np.float64), np.asarray(w_router, dtype=np.float64))
    if b_router is not None:
        z = z + np.asarray(b_router, dtype=np.float64)[None, :]
    return z


def softmax_rows(z: np.ndarray) -> np.ndarray:
    """Row softmax with the row maximum subtracted (the fp32 softmax of Section 5.2, here in fp64)."""
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    return e / e.sum(axis=1, keepdims=True)


def topk_by_logit(z: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest logits per row, descending; equal logits -> lower expert first.

    Ranking uses the logits (softmax is monotone, so the set is the same as
    ranking probabilities, without merging logits that exp() would round
    together).  A stable sort of -z keeps the lower index first among ties.
    """
    order = np.argsort(-z, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def gate(x, w_router, b_router, k: int, renormalize: bool):
    """Top-k softmax gate.  Returns (probs[T,E] f64, topk_idx[T,k] i32, topk_w[T,k] f64).

    topk_w[t,j] = p[t, idx[t,j]]; with ``renormalize`` the k weights are divided
    by their sum (GShard top-2).  Top-1 keeps w = p (Switch), so identity
    experts return the gate-weighted input.
    """
    z = gate_logits(x, w_router, b_router)
    p = softmax_rows(z)
    idx = topk_by_logit(z, k)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renormalize:
        w = w / w.sum(axis=1, keepdims=True)
    return p, idx, w


# ----------------------------------------------------------------------- dispatch
def capacity(T: int, E: int, k: int, capacity_factor: float) -> int:
    """C = ceil(k*T*CF/E), at least 1, in exact rational arithmetic; CF <= 0 -> dropless.

    CF is taken as the float32 value the C ABI carries.
    """
    if capacity_factor <= 0:
        return DROPLESS
    cf = Fraction(float(np.float32(capacity_factor)))
    q = Fraction(k * T) * cf / E
    c = -((-q.numerator) // q.denominator)
    return int(min(max(c, 1), DROPLESS))


def dispatch_plan(topk_idx: np.ndarray, E: int, C: int):
    """Capacity-bounded, order-preserving slotting of the k*T assignments.

    Assignment id a = j*T + t (all first choices in token order, then all
    second choices...).  Expert e keeps its first min(count_e, C) assignments
    in increasing a; kept rows of expert e occupy rows
    [offsets[e], offsets[e+1]) of the dispatched buffer in that order.

    Returns (counts[E] pre-capacity, offsets[E+1], assign_to_row[k*T] (-1 =
    dropped), row_to_assign[R]).
    """
    T, k = topk_idx.shape
    experts = np.ascontiguousarray(topk_idx.T).reshape(-1).astype(np.int64)  # index a = j*T+t
    counts = np.bincount(experts, minlength=E).astype(np.int64)
    kept = np.minimum(counts, C)
    offsets = np.zeros(E + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(kept)
    assign_to_row = np.full(k * T, -1, dtype=np.int64)
    for e in range(E):
        a_e = np.nonzero(experts == e)[0]           # increasing a
        a_kept = a_e[:kept[e]]
        assign_to_row[a_kept] = offsets[e] + np.arange(a_kept.size)
    R = int(offsets[E])
    row_to_assign = np.empty(R, dtype=np.int64)
    kept_a = np.nonzero(assign_to_row >= 0)[0]
    row_to_assign[assign_to_row[kept_a]] = kept_a
    return (counts.astype(np.int32), offsets.astype(np.int32),
            assign_to_row.astype(np.int32), row_to_assign.astype(np.int32))


def dispatch(x: np.ndarray, topk_idx: np.ndarray, E: int, C: int):
    """Plan + gather: xd[r,:] = x[row_to_assign[r] mod T, :]."""
    T = topk_idx.shape[0]
    counts, offsets, a2r, r2a = dispatch_plan(topk_idx, E, C)
    xd = np.asarray(x)[r2a.astype(np.int64) % T]
    return counts, offsets, a2r, r2a, xd


# ---------------------------------------------------------------------- expert FFN
def gelu(u: np.ndarray) -> np.ndarray:
    """Exact GELU u*Phi(u) = u/2 * (1 + erf(u/sqrt 2))."""
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


def silu(u: np.ndarray) -> np.ndarray:
    """u * sigmoid(u)."""
    return u / (1.0 + np.exp(-u))


def expert_rows_ffn(rows: np.ndarray, e: int, weights: Dict[str, np.ndarray], act: str) -> np.ndarray:
    """One expert's FFN on its rows (the sparsely activated FFN of Section 3.2), float64.

    GELU:   y = gelu(x W1_e + b1_e) W2_e + b2_e
    SwiGLU: y = (silu(x Wg_e) * (x Wu_e)) Wd_e
    """
    xr = np.asarray(rows, dtype=np.float64)
    if act == "gelu":
        u = np.matmul(xr, weights["w1"][e].astype(np.float64))
        if weights.get("b1") is not None:
            u = u + weights["b1"][e].astype(np.float64)[None, :]
        y = np.matmul(gelu(u), weights["w2"][e].astype(np.float64))
        if weights.get("b2") is not None:
            y = y + weights["b2"][e].astype(np.float64)[None, :]
        return y
    if act == "swiglu":
        g = np.matmul(xr, weights["w_gate_proj"][e].astype(np.float64))
        u = np.matmul(xr, weights["w_up"][e].astype(np.float64))
        return np.matmul(silu(g) * u, weights["w_down"][e].astype(np.float64))
    raise ValueError(act)


def expert_ffn(xd: np.ndarray, offsets: np.ndarray, weights: Dict[str, np.ndarray], act: str) -> np.ndarray:
    """yd[r,:] = FFN_e(xd[r,:]) for r in [offsets[e], offsets[e+1])."""
    E = len(offsets) - 1
    d_out = (weights["w2"] if act == "gelu" else weights["w_down"]).shape[2]
    yd = np.zeros((xd.shape[0], d_out), dtype=np.float64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            yd[lo:hi] = expert_rows_ffn(xd[lo:hi], e, weights, act)
    return yd


# ------------------------------------------------------------------------ combine
def combine(yd: np.ndarray, assign_to_row: np.ndarray, topk_w: np.ndarray,
            residual: Optional[np.ndarray]) -> np.ndarray:
    """out[t] = residual[t] + sum over kept choices j of topk_w[t,j] * yd[assign_to_row[j*T+t]].

    Dropped choices contribute nothing and the surviving weights are not
    rescaled; a token with every choice dropped yields the residual (or 0).
    """
    T, k = topk_w.shape
    d = yd.shape[1]
    out = np.zeros((T, d), dtype=np.float64)
    if residual is not None:
        out += np.asarray(residual, dtype=np.float64)
    for j in range(k):
        rows = assign_to_row[j * T:(j + 1) * T].astype(np.int64)
        keep = rows >= 0
        out[keep] += topk_w[keep, j][:, None] * yd[rows[keep]]
    return out


# ------------------------------------------------------------------ whole layer
def layer_forward(x, weights: Dict[str, np.ndarray], *, E: int, k: int, capacity_factor: float,
                  renormalize: bool, act: str, residual=None) -> Dict[str, np.ndarray]:
    """gate -> dispatch -> expert FFN -> combine; returns every intermediate."""
    T = x.shape[0]
    p, idx, w = gate(x, weights["w_router"], weights.get("b_router"), k, renormalize)
    C = capacity(T, E, k, capacity_factor)
    counts, offsets, a2r, r2a, xd = dispatch(x, idx, E, C)
    yd = expert_ffn(xd, offsets, weights, act)
    out = combine(yd, a2r, w, residual)
    return dict(probs=p, topk_idx=idx, topk_w=w, capacity=C, expert_counts=counts,
                expert_offsets=offsets, assign_to_row=a2r, row_to_assign=r2a, xd=xd, yd=yd, out=out)


def sampled_tokens_forward(x, weights, plan: Dict[str, np.ndarray], tokens: np.ndarray, *,
                           act: str, residual=None) -> np.ndarray:
    """out[t] for the listed tokens only, one token at a time from the definition.

    ``plan`` carries the oracle's own routing (topk_idx, topk_w, assign_to_row).
    Used where the full-size FFN is too slow for the CPU: each sampled token's
    kept choices go through their expert's FFN individually.
    """
    T, k = plan["topk_idx"].shape
    outs = []
    for t in np.asarray(tokens, dtype=np.int64):
        acc = np.zeros(x.shape[1], dtype=np.float64)
        if residual is not None:
            acc += np.asarray(residual[t], dtype=np.float64)
        for j in range(k):
            if plan["assign_to_row"][j * T + t] >= 0:
                e = int(plan["topk_idx"][t, j])
                acc += plan["topk_w"][t, j] * expert_rows_ffn(x[t:t + 1], e, weights, act)[0]
        outs.append(acc)
    return np.stack(outs) if outs else np.zeros((0, x.shape[1]))


# ------------------------------------------------------- ring memory offloading
def ring_schedule(n_layers: int, n_sections: int, n_steps: int) -> List[Tuple[str, int, int]]:
    """Event list of ring memory offloading (Section 3.3.2, steps 2-4 of the timeline figure).

    The GPU holds K = n_sections expert-parameter slots for a model of
    N = n_layers layers whose expert parameters all sit in CPU memory.  First
    the K slots are loaded with layers 0..K-1.  Then for each layer i in order:
    compute it from its slot, release the slot and start the asynchronous load
    of layer K+i into that same slot.  Repeated inference steps continue the
    same sequence with the layer index taken modulo N (the paper shows one
    pass; wrapping is this build's reading): the g-th layer evaluation overall
    (g = step*N + i) uses slot g mod K and is followed by the load of layer
    (g+K) mod N into that slot.  When K >= N every layer stays resident and
    nothing is reloaded.

    Returns tuples ("load", layer, slot) and ("compute", layer, slot).
    """
    N, K = n_layers, min(n_sections, n_layers)
    ev: List[Tuple[str, int, int]] = [("load", l, l % K) for l in range(K)]
    for g in range(n_steps * N):
        ev.append(("compute", g % N, g % K))
        if K < N:
            ev.append(("load", (g + K) % N, g % K))
    return ev


def stack_forward(x, layers: List[Dict[str, np.ndarray]], *, E, k, capacity_factor, renormalize, act):
    """x_{l+1} = x_l + MoE_l(x_l) over a list of layers (free-running, float64)."""
    h = np.asarray(x, dtype=np.float64)
    for w in layers:
        h = layer_forward(h, w, E=E, k=k, capacity_factor=capacity_factor,
                          renormalize=renormalize, act=act, residual=h)["out"]
    return h
