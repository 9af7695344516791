"""CPU oracle for the backward pass of the sparsely-gated MoE layer (TEST INFRASTRUCTURE).

This file is the checker, not the product: only ``tests/`` may import it.  It was
written and pinned before any backward kernel, so that they can be built against it.

What it computes.  The paper is mainly a training system (Section 3.2) but, as for the
forward pass, never writes the layer's equations; the backward pass is the chain rule
applied to the forward definition that ``moe_oracle.layer_forward`` writes out, with the
routing (which experts, which rows are kept) held fixed, as it is piecewise constant in
the inputs.  For an upstream gradient G = d loss / d out [T, d_model]:

  combine      d_res = G;  kept (t,j) with row r:  d_y[r] = w[t,j] G[t],  d_w[t,j] = <G[t], y[r]>;
               dropped choices: d_w = 0
  GELU FFN     d_h = d_y W2_e^T;  dW2_e = h_e^T d_y_e;  db2_e = sum_r d_y[r]
               d_u = d_h * gelu'(u),  gelu'(u) = Phi(u) + u phi(u)
               d_xd = d_u W1_e^T;  dW1_e = xd_e^T d_u_e;  db1_e = sum_r d_u[r]
  SwiGLU FFN   h = silu(g) * u with g = xd Wg_e, u = xd Wu_e;  d_h = d_y Wd_e^T;  dWd_e = h_e^T d_y_e
               d_g = d_h * u * silu'(g),  d_u = d_h * silu(g),  silu'(v) = s(v) (1 + v (1 - s(v)))
               d_xd = d_g Wg_e^T + d_u Wu_e^T;  dWg_e = xd_e^T d_g_e;  dWu_e = xd_e^T d_u_e
  dispatch     d_x[t] += sum over kept j of d_xd[r(t,j)]
  gate         renormalised: w_j = p_j / S, S = sum over the k selected (dropped ones included):
               d_p_i = d_w_i / S - (sum_j d_w_j w_j) / S;   otherwise d_p_i = d_w_i
               softmax: d_z = p * (d_p - sum_e d_p_e p_e), d_p being zero off the selected experts
               d_x += d_z W_g^T;  dW_g = x^T d_z;  db_g = sum_t d_z
  auxiliary    the paper names auxiliary losses as the known remedy for expert imbalance (Section 1, the
  loss         computation challenge) and gives no formula; the reading taken is the load-balancing loss of the
               work it cites there (GShard / Switch Transformer):
                 L_aux = coef * E * sum_e f_e * Pbar_e,
               f_e = fraction of the tokens whose FIRST choice is expert e (before capacity), Pbar_e = mean over
               the tokens of p[t, e].  f is piecewise constant, so d L_aux / d p[t, e] = coef * E * f_e / T,
               which joins d_p before the softmax Jacobian (on every expert, not only the selected ones).

Everything is float64 and unblocked: one ``numpy.matmul`` per product, one loop over
experts.  Expert matrices are input-major ([E, in, out]) as in the forward oracle.

Pins (tests/test_backward_oracle_pins.py): central differences of the forward oracle
along random directions in every input and parameter (the step is small enough that
the routing does not change, which the test checks); torch's autograd in float64 on a
dense re-expression of the layer with the routing fixed; the special case E = 1 (a
dense FFN: gate gradients vanish); the weight-gradient product by brute force and
against the layer's own dW2; the auxiliary loss by its closed forms (uniform probabilities or uniform routing
give coef, everything on one expert gives coef * E * its mean probability), a from-scratch loop, and the same
central differences and autograd with the loss added to the objective.  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
from scipy.special import erf

from . import moe_oracle as F


def gelu_grad(u: np.ndarray) -> np.ndarray:
    """d/du [u Phi(u)] = Phi(u) + u phi(u)."""
    return 0.5 * (1.0 + erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def silu_grad(v: np.ndarray) -> np.ndarray:
    s = 1.0 / (1.0 + np.exp(-v))
    return s * (1.0 + v * (1.0 - s))


def aux_loss(probs: np.ndarray, topk_idx: np.ndarray, coef: float) -> float:
    """coef * E * sum_e f_e * Pbar_e (see the header): 1 * coef when either the routing or the probabilities are uniform."""
    probs = np.asarray(probs, dtype=np.float64)
    T, E = probs.shape
    f = np.bincount(np.asarray(topk_idx)[:, 0].astype(np.int64), minlength=E) / T
    return float(coef * E * np.sum(f * probs.mean(axis=0)))


def expert_ffn_backward(xd, offsets, weights: Dict[str, np.ndarray], d_y, act: str) -> Dict[str, np.ndarray]:
    """Gradients of the per-expert FFN for the gradient d_y of its output rows: "xd" and one entry per
    parameter present in ``weights`` (input-major, like the parameters)."""
    xd = np.asarray(xd, dtype=np.float64)
    d_y = np.asarray(d_y, dtype=np.float64)
    E = len(offsets) - 1
    R, d = xd.shape
    grads: Dict[str, np.ndarray] = {}
    d_xd = np.zeros((R, d))
    names = ("w1", "b1", "w2", "b2") if act == "gelu" else ("w_gate_proj", "w_up", "w_down")
    for n in names:
        if weights.get(n) is not None:
            grads[n] = np.zeros(np.shape(weights[n]), dtype=np.float64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi <= lo:
            continue
        xe, dye = xd[lo:hi], d_y[lo:hi]
        if act == "gelu":
            w1, w2 = weights["w1"][e].astype(np.float64), weights["w2"][e].astype(np.float64)
            u = np.matmul(xe, w1)
            if weights.get("b1") is not None:
                u = u + weights["b1"][e].astype(np.float64)[None, :]
            h = F.gelu(u)
            d_h = np.matmul(dye, w2.T)
            grads["w2"][e] = np.matmul(h.T, dye)
            if "b2" in grads:
                grads["b2"][e] = dye.sum(axis=0)
            d_u = d_h * gelu_grad(u)
            grads["w1"][e] = np.matmul(xe.T, d_u)
            if "b1" in grads:
                grads["b1"][e] = d_u.sum(axis=0)
            d_xd[lo:hi] = np.matmul(d_u, w1.T)
        elif act == "swiglu":
            wg, wu, wd = (weights[n][e].astype(np.float64) for n in ("w_gate_proj", "w_up", "w_down"))
            g, u = np.matmul(xe, wg), np.matmul(xe, wu)
            h = F.silu(g) * u
            d_h = np.matmul(dye, wd.T)
            grads["w_down"][e] = np.matmul(h.T, dye)
            d_g = d_h * u * silu_grad(g)
            d_u = d_h * F.silu(g)
            grads["w_gate_proj"][e] = np.matmul(xe.T, d_g)
            grads["w_up"][e] = np.matmul(xe.T, d_u)
            d_xd[lo:hi] = np.matmul(d_g, wg.T) + np.matmul(d_u, wu.T)
        else:
            raise ValueError(act)
    grads["xd"] = d_xd
    return grads


def layer_backward(x, weights: Dict[str, np.ndarray], d_out, *, E: int, k: int, capacity_factor: float,
                   renormalize: bool, act: str, residual: Optional[np.ndarray] = None,
                   aux_coef: float = 0.0) -> Dict[str, np.ndarray]:
    """Gradients of sum(out * d_out) + aux_loss(probs, topk_idx, aux_coef) with respect to x, the residual and
    every parameter."""
    x = np.asarray(x, dtype=np.float64)
    G = np.asarray(d_out, dtype=np.float64)
    T, d = x.shape
    fw = F.layer_forward(x, weights, E=E, k=k, capacity_factor=capacity_factor, renormalize=renormalize, act=act,
                         residual=residual)
    p, idx, w = fw["probs"], fw["topk_idx"], fw["topk_w"]
    a2r, offsets, xd, yd = fw["assign_to_row"], fw["expert_offsets"], fw["xd"], fw["yd"]
    R = xd.shape[0]
    grads: Dict[str, np.ndarray] = {"residual": G.copy()}

    # combine
    d_y = np.zeros((R, d))
    d_w = np.zeros((T, k))
    for j in range(k):
        rows = a2r[j * T:(j + 1) * T].astype(np.int64)
        keep = rows >= 0
        d_y[rows[keep]] = w[keep, j][:, None] * G[keep]
        d_w[keep, j] = np.sum(G[keep] * yd[rows[keep]], axis=1)

    # expert FFN
    ffn = expert_ffn_backward(xd, offsets, weights, d_y, act)
    d_xd = ffn.pop("xd")
    grads.update(ffn)

    # dispatch
    d_x = np.zeros((T, d))
    for j in range(k):
        rows = a2r[j * T:(j + 1) * T].astype(np.int64)
        keep = rows >= 0
        d_x[keep] += d_xd[rows[keep]]

    # gate
    d_p = np.zeros((T, E))
    rows_t = np.arange(T)
    if renormalize:
        S = np.take_along_axis(p, idx.astype(np.int64), axis=1).sum(axis=1)
        common = np.sum(d_w * w, axis=1)
        for j in range(k):
            d_p[rows_t, idx[:, j]] = (d_w[:, j] - common) / S
    else:
        for j in range(k):
            d_p[rows_t, idx[:, j]] = d_w[:, j]
    if aux_coef != 0.0:
        f = np.bincount(idx[:, 0].astype(np.int64), minlength=E) / T
        d_p = d_p + (aux_coef * E / T) * f[None, :]
    d_z = p * (d_p - np.sum(d_p * p, axis=1, keepdims=True))
    w_router = np.asarray(weights["w_router"], dtype=np.float64)
    d_x += np.matmul(d_z, w_router.T)
    grads["w_router"] = np.matmul(x.T, d_z)
    if weights.get("b_router") is not None:
        grads["b_router"] = d_z.sum(axis=0)
    grads["x"] = d_x
    grads["topk_w"] = d_w
    grads["logits"] = d_z
    return grads


def expert_wgrad(a: np.ndarray, b: np.ndarray, offsets: np.ndarray) -> np.ndarray:
    """c[e] = a[rows of e]^T b[rows of e]: the weight-gradient products of the expert FFN above
    (dW2_e = h_e^T d_y_e, dW1_e = xd_e^T d_u_e and their transposes), one matmul per expert."""
    E = len(offsets) - 1
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    c = np.zeros((E, a.shape[1], b.shape[1]), dtype=np.float64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            c[e] = np.matmul(a[lo:hi].T, b[lo:hi])
    return c
