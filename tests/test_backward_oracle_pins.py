"""Pins of the backward oracle (CPU only): central differences of the forward oracle, torch's autograd in
float64 on a dense re-expression of the layer with the routing held fixed, special cases, and planted
mistakes that these pins must catch."""
import contextlib

import numpy as np
import pytest
import torch

from oracle import moe_backward_oracle as B
from oracle import moe_oracle as F

CASES = [
    dict(T=24, d=8, f=12, E=4, k=2, cf=1.0, renorm=True, act="gelu", bias=True, rbias=True, res=True),
    dict(T=24, d=8, f=12, E=4, k=2, cf=0.6, renorm=True, act="swiglu", bias=False, rbias=False, res=False),
    dict(T=17, d=6, f=10, E=5, k=1, cf=0.0, renorm=False, act="gelu", bias=True, rbias=True, res=False),
    dict(T=19, d=6, f=8, E=3, k=3, cf=0.0, renorm=True, act="gelu", bias=False, rbias=True, res=True),
    dict(T=30, d=8, f=8, E=6, k=2, cf=0.5, renorm=False, act="swiglu", bias=False, rbias=True, res=False),
]


def make(c, seed=0):
    r = np.random.default_rng(seed)
    W = {"w_router": r.standard_normal((c["d"], c["E"])) * 0.7}
    if c["rbias"]:
        W["b_router"] = r.standard_normal(c["E"]) * 0.3
    if c["act"] == "gelu":
        W["w1"] = r.standard_normal((c["E"], c["d"], c["f"])) * 0.5
        W["w2"] = r.standard_normal((c["E"], c["f"], c["d"])) * 0.5
        if c["bias"]:
            W["b1"] = r.standard_normal((c["E"], c["f"])) * 0.3
            W["b2"] = r.standard_normal((c["E"], c["d"])) * 0.3
    else:
        for n, shape in (("w_gate_proj", (c["E"], c["d"], c["f"])), ("w_up", (c["E"], c["d"], c["f"])),
                         ("w_down", (c["E"], c["f"], c["d"]))):
            W[n] = r.standard_normal(shape) * 0.5
    x = r.standard_normal((c["T"], c["d"]))
    res = r.standard_normal((c["T"], c["d"])) if c["res"] else None
    G = r.standard_normal((c["T"], c["d"]))
    return x, W, res, G


def kw(c):
    return dict(E=c["E"], k=c["k"], capacity_factor=c["cf"], renormalize=c["renorm"], act=c["act"])


AUX = 0.7          # coefficient of the auxiliary loss in the pins below (large, so that a mistake in it shows)


def objective(o, G):
    return float(np.sum(o["out"] * G)) + B.aux_loss(o["probs"], o["topk_idx"], AUX)


def pin_central_differences(c):
    x, W, res, G = make(c, 1)
    g = B.layer_backward(x, W, G, residual=res, aux_coef=AUX, **kw(c))
    base = F.layer_forward(x, W, residual=res, **kw(c))
    if c["cf"] > 0 and c["cf"] < 1:
        assert (base["assign_to_row"] < 0).any()            # drops are part of the case
    r = np.random.default_rng(2)
    eps = 1e-6
    names = ["x"] + sorted(W) + (["residual"] if res is not None else [])
    for n in names:
        for trial in range(3):
            ref = x if n == "x" else res if n == "residual" else W[n]
            delta = r.standard_normal(ref.shape)

            def f(sign):
                xx, WW, rr = x, dict(W), res
                if n == "x":
                    xx = x + sign * eps * delta
                elif n == "residual":
                    rr = res + sign * eps * delta
                else:
                    WW[n] = W[n] + sign * eps * delta
                o = F.layer_forward(xx, WW, residual=rr, **kw(c))
                assert np.array_equal(o["topk_idx"], base["topk_idx"])          # same routing: differentiable here
                assert np.array_equal(o["assign_to_row"], base["assign_to_row"])
                return objective(o, G)

            num = (f(+1) - f(-1)) / (2 * eps)
            ana = float(np.sum(g[n] * delta))
            assert abs(num - ana) <= 2e-6 * max(1.0, abs(ana)), (n, num, ana)


def pin_torch_autograd(c):
    x, W, res, G = make(c, 3)
    g = B.layer_backward(x, W, G, residual=res, aux_coef=AUX, **kw(c))
    fw = F.layer_forward(x, W, residual=res, **kw(c))
    idx, a2r = fw["topk_idx"].astype(np.int64), fw["assign_to_row"]
    T, k = idx.shape
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tW = {n: torch.tensor(v, dtype=torch.float64, requires_grad=True) for n, v in W.items()}
    tres = torch.tensor(res, dtype=torch.float64, requires_grad=True) if res is not None else None
    z = tx @ tW["w_router"]
    if "b_router" in tW:
        z = z + tW["b_router"]
    p = torch.softmax(z, dim=1)
    w = torch.gather(p, 1, torch.tensor(idx))
    if c["renorm"]:
        w = w / w.sum(dim=1, keepdim=True)
    outs = []
    for t in range(T):
        acc = tres[t] if tres is not None else torch.zeros(x.shape[1], dtype=torch.float64)
        for j in range(k):
            if a2r[j * T + t] < 0:
                continue
            e = int(idx[t, j])
            if c["act"] == "gelu":
                u = tx[t] @ tW["w1"][e]
                if "b1" in tW:
                    u = u + tW["b1"][e]
                y = torch.nn.functional.gelu(u) @ tW["w2"][e]
                if "b2" in tW:
                    y = y + tW["b2"][e]
            else:
                y = (torch.nn.functional.silu(tx[t] @ tW["w_gate_proj"][e]) * (tx[t] @ tW["w_up"][e])) @ tW["w_down"][e]
            acc = acc + w[t, j] * y
        outs.append(acc)
    out = torch.stack(outs)
    assert np.allclose(out.detach().numpy(), fw["out"], rtol=1e-12, atol=1e-12)
    # the auxiliary loss written out from its definition: first-choice fractions (constants) times mean probabilities
    T_, E_ = p.shape
    first = torch.tensor([[1.0 if idx[t, 0] == e else 0.0 for e in range(E_)] for t in range(T_)], dtype=torch.float64)
    aux = AUX * E_ * (first.mean(dim=0) * p.mean(dim=0)).sum()
    assert abs(aux.item() - B.aux_loss(fw["probs"], fw["topk_idx"], AUX)) < 1e-12
    ((out * torch.tensor(G)).sum() + aux).backward()
    assert np.allclose(tx.grad.numpy(), g["x"], rtol=1e-9, atol=1e-11)
    for n in W:
        got = tW[n].grad.numpy() if tW[n].grad is not None else np.zeros_like(W[n])
        assert np.allclose(got, g[n], rtol=1e-9, atol=1e-11), n
    if res is not None:
        assert np.allclose(tres.grad.numpy(), g["residual"])


def pin_single_expert_is_a_dense_ffn(_c=None):
    c = dict(T=11, d=6, f=9, E=1, k=1, cf=0.0, renorm=False, act="gelu", bias=True, rbias=True, res=False)
    x, W, res, G = make(c, 4)
    g = B.layer_backward(x, W, G, **kw(c))
    assert np.allclose(g["w_router"], 0, atol=1e-13) and np.allclose(g["b_router"], 0, atol=1e-13)   # p == 1 whatever z
    tx = torch.tensor(x, requires_grad=True)
    t = {n: torch.tensor(W[n][0], requires_grad=True) for n in ("w1", "b1", "w2", "b2")}
    y = torch.nn.functional.gelu(tx @ t["w1"] + t["b1"]) @ t["w2"] + t["b2"]
    (y * torch.tensor(G)).sum().backward()
    assert np.allclose(tx.grad.numpy(), g["x"], rtol=1e-10, atol=1e-12)
    for n in t:
        assert np.allclose(t[n].grad.numpy(), g[n][0], rtol=1e-10, atol=1e-12)


def test_expert_wgrad_bruteforce_and_against_layer_backward():
    r = np.random.default_rng(8)
    offsets = np.array([0, 3, 3, 4, 9])
    A, Bm = r.standard_normal((9, 5)), r.standard_normal((9, 4))
    got = B.expert_wgrad(A, Bm, offsets)
    for e in range(4):
        for i in range(5):
            for j in range(4):
                want = sum(A[t, i] * Bm[t, j] for t in range(offsets[e], offsets[e + 1]))
                assert abs(got[e, i, j] - want) < 1e-12
    assert not got[1].any()
    # the layer's own weight gradients are such products: dW2_e (input-major [f, d]) = h_e^T d_y_e
    c = CASES[0]
    x, W, res, G = make(c, 5)
    g = B.layer_backward(x, W, G, residual=res, **kw(c))
    fw = F.layer_forward(x, W, residual=res, **kw(c))
    T, k = fw["topk_w"].shape
    d_y = np.zeros_like(fw["yd"])
    for j in range(k):
        rows = fw["assign_to_row"][j * T:(j + 1) * T]
        keep = rows >= 0
        d_y[rows[keep]] = fw["topk_w"][keep, j][:, None] * G[keep]
    h = np.zeros((fw["xd"].shape[0], c["f"]))
    for e in range(c["E"]):
        lo, hi = fw["expert_offsets"][e], fw["expert_offsets"][e + 1]
        h[lo:hi] = F.gelu(fw["xd"][lo:hi] @ W["w1"][e] + W["b1"][e])
    assert np.allclose(B.expert_wgrad(h, d_y, fw["expert_offsets"]), g["w2"], rtol=1e-12, atol=1e-12)


def test_aux_loss_closed_forms():
    r = np.random.default_rng(11)
    T, E = 40, 5
    idx = r.integers(0, E, size=(T, 2))
    assert abs(B.aux_loss(np.full((T, E), 1.0 / E), idx, 0.3) - 0.3) < 1e-15                 # uniform probabilities
    p = r.random((T, E)); p /= p.sum(axis=1, keepdims=True)
    even = np.stack([np.arange(T) % E, (np.arange(T) + 1) % E], axis=1)
    assert abs(B.aux_loss(p, even, 0.3) - 0.3) < 1e-15                                       # uniform routing
    one = np.zeros((T, 2), dtype=np.int64); one[:, 1] = 1
    assert abs(B.aux_loss(p, one, 0.3) - 0.3 * E * p[:, 0].mean()) < 1e-15                   # everything on expert 0
    # second choices do not count
    idx2 = idx.copy(); idx2[:, 1] = (idx2[:, 1] + 1) % E
    assert B.aux_loss(p, idx, 1.0) == B.aux_loss(p, idx2, 1.0)
    # from scratch
    want = 0.0
    for e in range(E):
        want += sum(1 for t in range(T) if idx[t, 0] == e) / T * sum(p[t, e] for t in range(T)) / T
    assert abs(B.aux_loss(p, idx, 2.0) - 2.0 * E * want) < 1e-14
    assert B.aux_loss(p, idx, 0.0) == 0.0


def test_aux_gradient_is_additive():
    c = CASES[0]
    x, W, res, G = make(c, 6)
    g0 = B.layer_backward(x, W, G, residual=res, **kw(c))
    g1 = B.layer_backward(x, W, np.zeros_like(G), residual=res, aux_coef=AUX, **kw(c))
    g = B.layer_backward(x, W, G, residual=res, aux_coef=AUX, **kw(c))
    for n in ("x", "w_router", "b_router", "logits"):
        assert np.allclose(g[n], g0[n] + g1[n], rtol=1e-12, atol=1e-14)
    assert np.abs(g1["w_router"]).max() > 1e-4 and not g1["w1"].any()      # reaches the router only


PINS = [pin_central_differences, pin_torch_autograd]


@pytest.mark.parametrize("c", CASES, ids=lambda c: f"{c['act']}-k{c['k']}-E{c['E']}-cf{c['cf']}")
@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_backward_pin(pin, c):
    pin(c)


def test_single_expert():
    pin_single_expert_is_a_dense_ffn()


# ------------------------------------------------------------------------- planted mistakes
@contextlib.contextmanager
def planted(name, fn):
    saved = getattr(B, name)
    setattr(B, name, fn)
    try:
        yield
    finally:
        setattr(B, name, saved)


def _wrap(transform):
    orig = B.layer_backward

    def mutant(*a, **k):
        return transform(orig(*a, **k), a, k)
    return mutant


def _wrap_kw(change):
    orig = B.layer_backward

    def mutant(*a, **k):
        return orig(*a, **change(k))
    return mutant


def _renorm_term_dropped(g, a, k):
    # recompute the gate part without the -(sum d_w w)/S term
    if not k["renormalize"]:
        return g
    x, W = np.asarray(a[0], dtype=np.float64), a[1]
    fw = F.layer_forward(x, W, **{n: v for n, v in k.items() if n != "aux_coef"})
    p, idx = fw["probs"], fw["topk_idx"].astype(np.int64)
    S = np.take_along_axis(p, idx, axis=1).sum(axis=1)
    d_p = np.zeros_like(p)
    for j in range(idx.shape[1]):
        d_p[np.arange(len(p)), idx[:, j]] = g["topk_w"][:, j] / S
    d_p += k.get("aux_coef", 0.0) * p.shape[1] / len(p) * (np.bincount(idx[:, 0], minlength=p.shape[1]) / len(p))[None, :]
    d_z = p * (d_p - np.sum(d_p * p, axis=1, keepdims=True))
    g = dict(g)
    g["x"] = g["x"] - g["logits"] @ np.asarray(W["w_router"]).T + d_z @ np.asarray(W["w_router"]).T
    g["w_router"] = x.T @ d_z
    if "b_router" in g:
        g["b_router"] = d_z.sum(axis=0)
    return g


MUTANTS = {
    "gelu' without the u*phi(u) term": lambda: planted("gelu_grad", lambda u: 0.5 * (1.0 + B.erf(u / np.sqrt(2.0)))),
    "silu' = sigmoid": lambda: planted("silu_grad", lambda v: 1.0 / (1.0 + np.exp(-v))),
    "gate path into d_x missing": lambda: planted("layer_backward", _wrap(
        lambda g, a, k: {**g, "x": g["x"] - g["logits"] @ np.asarray(a[1]["w_router"], dtype=np.float64).T})),
    "dW_router transposed contraction (sum over experts)": lambda: planted("layer_backward", _wrap(
        lambda g, a, k: {**g, "w_router": np.asarray(a[0]).T @ (g["logits"] * 0 + g["logits"].sum(axis=1, keepdims=True))})),
    "renormalisation's common term dropped": lambda: planted("layer_backward", _wrap(_renorm_term_dropped)),
    "residual gradient scaled": lambda: planted("layer_backward", _wrap(lambda g, a, k: {**g, "residual": 2 * g["residual"]})),
    "auxiliary loss ignored by the backward pass": lambda: planted("layer_backward", _wrap_kw(lambda k: {**k, "aux_coef": 0.0})),
    "auxiliary gradient without the factor E": lambda: planted("layer_backward", _wrap_kw(lambda k: {**k, "aux_coef": k.get("aux_coef", 0.0) / k["E"]})),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name):
    caught = []
    with MUTANTS[name]():
        for pin in PINS:
            for c in CASES:
                try:
                    pin(c)
                except Exception:
                    caught.append((pin.__name__, c["act"]))
    assert caught, f"no pin notices: {name}"
