"""Do the oracle's pins catch mistakes?  Each mutant below plants one plausible error in the oracle (a
dropped term, a wrong sign or index, a transposed operand, a wrong priority or rounding rule) and the
whole pin suite of test_oracle_pins.py is run against it: at least one pin has to fail.  CPU only;
the mistakes live in the oracle for the duration of one check and nowhere else.
"""
import contextlib
import inspect
import itertools

import numpy as np
import pytest

from oracle import moe_oracle as O

import test_oracle_pins as P


def _pin_calls():
    """Every pin as a zero-argument callable (parametrized pins expanded)."""
    calls = []
    for name, fn in sorted(vars(P).items()):
        if not name.startswith("test_") or not inspect.isfunction(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        axes = []
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            axes.append([dict(zip(names, v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,)))
                         for v in m.args[1]])
        for combo in itertools.product(*axes):
            kw = {}
            for part in combo:
                kw.update(part)
            calls.append((f"{name}{sorted(kw.items())}", (lambda f=fn, k=kw: f(**k))))
    return calls


def failing_pins():
    bad = []
    for name, call in _pin_calls():
        try:
            call()
        except Exception:  # an assertion, or a crash caused by the planted mistake: both count as caught
            bad.append(name)
    return bad


@contextlib.contextmanager
def planted(**replacements):
    saved = {k: getattr(O, k) for k in replacements}
    try:
        for k, v in replacements.items():
            setattr(O, k, v)
        yield
    finally:
        for k, v in saved.items():
            setattr(O, k, v)


# ------------------------------------------------------------------ the mutants
_orig = {k: getattr(O, k) for k in dir(O) if callable(getattr(O, k)) and not k.startswith("_")}


def m_topk_ties_higher_first(z, k):
    E = z.shape[1]
    order = np.argsort(-z[:, ::-1], axis=1, kind="stable")
    return (E - 1 - order[:, :k]).astype(np.int32)


def m_topk_smallest(z, k):
    return np.argsort(z, axis=1, kind="stable")[:, :k].astype(np.int32)


def m_topk_unordered(z, k):  # right set, ascending expert index instead of rank order
    return np.sort(_orig["topk_by_logit"](z, k), axis=1).astype(np.int32)


def m_logits_no_bias(x, w, b):
    return _orig["gate_logits"](x, w, None)


def m_logits_transposed(x, w, b):
    w = np.asarray(w)
    return _orig["gate_logits"](x, w.T if w.shape[0] == w.shape[1] else w, b)


def m_softmax_wrong_axis(z):
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return e / e.sum(axis=0, keepdims=True)


def m_softmax_no_normalise(z):
    return np.exp(z - z.max(axis=1, keepdims=True))


def _gate_variant(always_renorm=None, top1_is_one=False, rank_on_probs_of=None):
    def gate(x, w_router, b_router, k, renormalize):
        z = O.gate_logits(x, w_router, b_router)
        p = O.softmax_rows(z)
        idx = O.topk_by_logit(z, k)
        w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
        r = renormalize if always_renorm is None else always_renorm
        if r:
            w = w / w.sum(axis=1, keepdims=True)
        if top1_is_one and k == 1:
            w = np.ones_like(w)
        return p, idx, w
    return gate


def m_capacity_floor(T, E, k, cf):
    if cf <= 0:
        return O.DROPLESS
    return max(int(np.floor(k * T * float(np.float32(cf)) / E)), 1)


def m_capacity_no_k(T, E, k, cf):
    return _orig["capacity"](T, E, 1, cf)


def m_capacity_zero_allowed(T, E, k, cf):
    if cf <= 0:
        return O.DROPLESS
    return int(np.ceil(k * T * float(np.float32(cf)) / E - 1e-9)) if k * T * cf / E >= 1 else 0


def _plan_variant(token_major=False, keep_last=False, no_clamp_offsets=False, drop_marker=-1):
    def plan(topk_idx, E, C):
        T, k = topk_idx.shape
        if token_major:
            experts_tm = np.ascontiguousarray(topk_idx).reshape(-1).astype(np.int64)  # index t*k + j
        experts = np.ascontiguousarray(topk_idx.T).reshape(-1).astype(np.int64)
        counts = np.bincount(experts, minlength=E).astype(np.int64)
        kept = np.minimum(counts, C)
        offsets = np.zeros(E + 1, dtype=np.int64)
        offsets[1:] = np.cumsum(counts if no_clamp_offsets else kept)
        a2r = np.full(k * T, drop_marker, dtype=np.int64)
        for e in range(E):
            if token_major:
                tm = np.nonzero(experts_tm == e)[0]          # priority order t*k + j
                a_e = (tm % k) * T + tm // k                  # back to a = j*T + t
            else:
                a_e = np.nonzero(experts == e)[0]
            a_kept = a_e[-kept[e]:] if (keep_last and kept[e] > 0) else a_e[:kept[e]]
            a2r[a_kept] = offsets[e] + np.arange(a_kept.size)
        R = int(offsets[E])
        r2a = np.zeros(R, dtype=np.int64)
        kept_a = np.nonzero(a2r >= 0)[0]
        r2a[a2r[kept_a]] = kept_a
        return counts.astype(np.int32), offsets.astype(np.int32), a2r.astype(np.int32), r2a.astype(np.int32)
    return plan


def m_dispatch_wrong_row(x, topk_idx, E, C):
    counts, offsets, a2r, r2a = O.dispatch_plan(topk_idx, E, C)
    k = topk_idx.shape[1]
    xd = np.asarray(x)[r2a.astype(np.int64) // max(k, 1) % x.shape[0]]  # a // k instead of a mod T
    return counts, offsets, a2r, r2a, xd


def m_gelu_tanh(u):
    return 0.5 * u * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (u + 0.044715 * u ** 3)))


def m_gelu_no_half(u):
    return 2.0 * _orig["gelu"](u)


def m_silu_sign(u):
    return u / (1.0 + np.exp(u))


def _ffn_variant(next_expert=False, no_b1=False, no_b2=False, swap_gate_up=False, w2_transposed=False):
    def ffn(rows, e, weights, act):
        w = dict(weights)
        if next_expert:
            e = (e + 1) % len(w["w1" if act == "gelu" else "w_up"])
        if no_b1:
            w["b1"] = None
        if no_b2:
            w["b2"] = None
        if swap_gate_up and act == "swiglu":
            w["w_gate_proj"], w["w_up"] = w["w_up"], w["w_gate_proj"]
        name = "w2" if act == "gelu" else "w_down"
        if w2_transposed and w[name].shape[1] == w[name].shape[2]:
            w[name] = np.transpose(w[name], (0, 2, 1))
        return _orig["expert_rows_ffn"](rows, e, w, act)
    return ffn


def m_expert_ffn_off_by_one(xd, offsets, weights, act):
    E = len(offsets) - 1
    d_out = (weights["w2"] if act == "gelu" else weights["w_down"]).shape[2]
    yd = np.zeros((xd.shape[0], d_out))
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi - 1 > lo:
            yd[lo:hi - 1] = O.expert_rows_ffn(xd[lo:hi - 1], e, weights, act)
    return yd


def _combine_variant(unweighted=False, no_residual=False, dropped_wraps=False, first_choice_only=False):
    def combine(yd, a2r, topk_w, residual):
        T, k = topk_w.shape
        out = np.zeros((T, yd.shape[1]))
        if residual is not None and not no_residual:
            out += np.asarray(residual, dtype=np.float64)
        for j in range(1 if first_choice_only else k):
            rows = a2r[j * T:(j + 1) * T].astype(np.int64)
            keep = np.ones(T, bool) if dropped_wraps else rows >= 0
            if yd.shape[0] == 0:
                continue
            w = 1.0 if unweighted else topk_w[keep, j][:, None]
            out[keep] += w * yd[rows[keep]]
        return out
    return combine


def _ring_variant(slot_shift=0, refill_shift=0, refill_other_slot=False):
    def sched(n_layers, n_sections, n_steps):
        N, K = n_layers, min(n_sections, n_layers)
        ev = [("load", l, l % K) for l in range(K)]
        for g in range(n_steps * N):
            ev.append(("compute", g % N, (g + slot_shift) % K))
            if K < N:
                ev.append(("load", (g + K + refill_shift) % N, ((g + 1) if refill_other_slot else g) % K))
        return ev
    return sched


def m_stack_no_residual(x, layers, *, E, k, capacity_factor, renormalize, act):
    h = np.asarray(x, dtype=np.float64)
    for w in layers:
        h = O.layer_forward(h, w, E=E, k=k, capacity_factor=capacity_factor, renormalize=renormalize, act=act)["out"]
    return h


MUTANTS = {
    "top-k ties prefer the higher index": dict(topk_by_logit=m_topk_ties_higher_first),
    "top-k takes the smallest logits": dict(topk_by_logit=m_topk_smallest),
    "top-k returned in index order, not rank order": dict(topk_by_logit=m_topk_unordered),
    "router bias dropped": dict(gate_logits=m_logits_no_bias),
    "router matrix transposed": dict(gate_logits=m_logits_transposed),
    "softmax over the token axis": dict(softmax_rows=m_softmax_wrong_axis),
    "softmax not normalised": dict(softmax_rows=m_softmax_no_normalise),
    "gate always renormalises": dict(gate=_gate_variant(always_renorm=True)),
    "gate never renormalises": dict(gate=_gate_variant(always_renorm=False)),
    "top-1 weight forced to one": dict(gate=_gate_variant(top1_is_one=True)),
    "capacity rounded down": dict(capacity=m_capacity_floor),
    "capacity ignores k": dict(capacity=m_capacity_no_k),
    "capacity may be zero": dict(capacity=m_capacity_zero_allowed),
    "token-major drop priority": dict(dispatch_plan=_plan_variant(token_major=True)),
    "capacity keeps the last assignments": dict(dispatch_plan=_plan_variant(keep_last=True)),
    "offsets ignore the capacity": dict(dispatch_plan=_plan_variant(no_clamp_offsets=True)),
    "dropped assignments marked 0": dict(dispatch_plan=_plan_variant(drop_marker=0)),
    "dispatch gathers token a div k": dict(dispatch=m_dispatch_wrong_row),
    "tanh-form GELU": dict(gelu=m_gelu_tanh),
    "GELU without the one half": dict(gelu=m_gelu_no_half),
    "SiLU with the wrong sign in exp": dict(silu=m_silu_sign),
    "FFN uses the next expert's weights": dict(expert_rows_ffn=_ffn_variant(next_expert=True)),
    "first bias dropped": dict(expert_rows_ffn=_ffn_variant(no_b1=True)),
    "second bias dropped": dict(expert_rows_ffn=_ffn_variant(no_b2=True)),
    "SwiGLU gate and up swapped": dict(expert_rows_ffn=_ffn_variant(swap_gate_up=True)),
    "second matrix transposed": dict(expert_rows_ffn=_ffn_variant(w2_transposed=True)),
    "last row of every expert skipped": dict(expert_ffn=m_expert_ffn_off_by_one),
    "combine ignores the gate weights": dict(combine=_combine_variant(unweighted=True)),
    "combine ignores the residual": dict(combine=_combine_variant(no_residual=True)),
    "combine reads row -1 for dropped choices": dict(combine=_combine_variant(dropped_wraps=True)),
    "combine uses the first choice only": dict(combine=_combine_variant(first_choice_only=True)),
    "ring computes from the next slot": dict(ring_schedule=_ring_variant(slot_shift=1)),
    "ring refills with layer g+K+1": dict(ring_schedule=_ring_variant(refill_shift=1)),
    "ring refills the neighbouring slot": dict(ring_schedule=_ring_variant(refill_other_slot=True)),
    "layer stack without the residual": dict(stack_forward=m_stack_no_residual),
}


def test_pins_pass_on_the_real_oracle():
    assert failing_pins() == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch(name):
    with planted(**MUTANTS[name]):
        caught = failing_pins()
    assert caught, f"no pin notices: {name}"
