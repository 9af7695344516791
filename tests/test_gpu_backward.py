"""Backward pass pieces on the GPU against the backward oracle: the combine's backward and the expert FFN's
backward (input gradient, weight and bias gradients) on the forward pass's own routing."""
import numpy as np
import pytest
import torch

import paper_2205_10034_amd as M
from oracle import moe_backward_oracle as B
from oracle import moe_oracle as O
from workloads import WORKLOADS, make_layer

from gpu_util import alloc_ws, rel_fro, to_dev, to_np, upload_weights

pytestmark = pytest.mark.gpu


def forward_pieces(wl, L, W, x):
    """gate -> dispatch (with the gathered rows) -> expert FFN through the C ABI; returns the device buffers."""
    cfg = M.MoEConfig.from_workload(wl)
    A = wl.k * wl.T
    idx = torch.empty(wl.T, wl.k, dtype=torch.int32, device="cuda")
    w = torch.empty(wl.T, wl.k, dtype=torch.float32, device="cuda")
    M.moe_gate(cfg, x, W.tensors["w_router"], W.tensors.get("b_router"), idx, w)
    counts = torch.empty(wl.E, dtype=torch.int32, device="cuda")
    offsets = torch.empty(wl.E + 1, dtype=torch.int32, device="cuda")
    a2r = torch.empty(A, dtype=torch.int32, device="cuda")
    r2a = torch.empty(A, dtype=torch.int32, device="cuda")
    lay = M.moe_workspace_layout(cfg)
    xd = torch.zeros(max(lay["r_max"], 1), wl.d_model, dtype=torch.bfloat16, device="cuda")
    M.moe_dispatch(cfg, x, idx, counts, offsets, a2r, r2a, xd, alloc_ws(cfg, 1))
    yd = torch.zeros_like(xd)
    ws_ffn = alloc_ws(cfg, 2)
    M.moe_expert_ffn(cfg, W, xd, offsets, yd, ws_ffn)
    torch.cuda.synchronize()
    h = ws_ffn[:lay["r_max"] * wl.d_ff * 2].view(torch.bfloat16).reshape(lay["r_max"], wl.d_ff)
    return cfg, dict(idx=idx, w=w, offsets=offsets, a2r=a2r, xd=xd, yd=yd, h=h, r_max=lay["r_max"])


def expert_grad_buffers(wl, L, grad_dtype=torch.float32):
    """(w1_input_major, w2_input_major, d_w1, d_b1, d_w2, d_b2) in the layouts the C ABI documents; SwiGLU: the gate
    and up projections stacked.  grad_dtype: the element type of the weight gradients (the bias gradients are float32)."""
    nan32 = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    nanw = lambda *shape: torch.full(shape, float("nan"), dtype=grad_dtype, device="cuda")
    if wl.act == "swiglu":
        w1_im = to_dev(np.concatenate([L["w_gate_proj"], L["w_up"]], axis=2), wl.dtype)      # [E, d_model, 2 d_ff]
        return w1_im, to_dev(L["w_down"], wl.dtype), nanw(wl.E, 2 * wl.d_ff, wl.d_model), None, nanw(wl.E, wl.d_model, wl.d_ff), None
    return (to_dev(L["w1"], wl.dtype), to_dev(L["w2"], wl.dtype), nanw(wl.E, wl.d_ff, wl.d_model), nan32(wl.E, wl.d_ff),
            nanw(wl.E, wl.d_model, wl.d_ff), nan32(wl.E, wl.d_model))


def expert_grad_errors(wl, ref, d_w1, d_b1, d_w2, d_b2):
    """Relative Frobenius error of every expert-parameter gradient against the oracle's (input-major) ones."""
    g1, g2 = d_w1.float().cpu().numpy().transpose(0, 2, 1), d_w2.float().cpu().numpy().transpose(0, 2, 1)
    if wl.act == "swiglu":
        return {"w_gate_proj": rel_fro(g1[:, :, :wl.d_ff], ref["w_gate_proj"]), "w_up": rel_fro(g1[:, :, wl.d_ff:], ref["w_up"]),
                "w_down": rel_fro(g2, ref["w_down"])}
    return {"w1": rel_fro(g1, ref["w1"]), "w2": rel_fro(g2, ref["w2"]), "b1": rel_fro(d_b1.cpu().numpy(), ref["b1"]),
            "b2": rel_fro(d_b2.cpu().numpy(), ref["b2"])}


@pytest.mark.parametrize("name,kw", [("gpt", dict(T=700, E=4, d_model=256, d_ff=512)),
                                     ("gpt", dict(T=1500, E=8, d_model=512, d_ff=256, capacity_factor=0.6)),
                                     ("gpt", dict(T=96, E=16, d_model=256, d_ff=256, k=1, capacity_factor=0.0)),
                                     ("large", dict(T=700, E=4, d_model=256, d_ff=512)),
                                     ("large", dict(T=1500, E=8, d_model=512, d_ff=256, capacity_factor=0.6)),
                                     ("large", dict(T=96, E=16, d_model=256, d_ff=256, k=1, capacity_factor=0.0))],
                         ids=lambda v: str(v).replace(" ", ""))
def test_combine_and_expert_ffn_backward(name, kw):
    wl = WORKLOADS[name].scaled(**kw)
    print(f"backward case {wl}", flush=True)
    L = make_layer(wl, with_bias=True)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    cfg, fw = forward_pieces(wl, L, W, x)
    ref_fw = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor, renormalize=wl.renormalize,
                             act=wl.act)
    assert np.array_equal(fw["a2r"].cpu().numpy(), ref_fw["assign_to_row"])
    R = int(ref_fw["expert_offsets"][-1])
    rng = np.random.default_rng(3)
    G_np = to_np(to_dev(rng.standard_normal(L["x"].shape).astype(np.float32), wl.dtype))
    G = to_dev(G_np, wl.dtype)

    # ---- combine backward (fed the GPU's own yd and gate weights, like the oracle below)
    d_yd = torch.full_like(fw["yd"], float("nan"))
    d_w = torch.full((wl.T, wl.k), float("nan"), dtype=torch.float32, device="cuda")
    M.moe_combine_backward(cfg, G, fw["yd"], fw["a2r"], fw["w"], d_yd, d_w)
    torch.cuda.synchronize()
    yd_np, w_np = to_np(fw["yd"]), fw["w"].cpu().numpy()
    a2r = ref_fw["assign_to_row"]
    ref_dy = np.zeros((R, wl.d_model))
    ref_dw = np.zeros((wl.T, wl.k))
    for j in range(wl.k):
        rows = a2r[j * wl.T:(j + 1) * wl.T]
        keep = rows >= 0
        ref_dy[rows[keep]] = w_np[keep, j][:, None].astype(np.float64) * G_np[keep]
        ref_dw[keep, j] = np.sum(G_np[keep].astype(np.float64) * yd_np[rows[keep]], axis=1)
    assert rel_fro(to_np(d_yd[:R]), ref_dy) < 4e-3          # one bf16 rounding
    assert np.allclose(d_w.cpu().numpy(), ref_dw, rtol=1e-4, atol=1e-4)
    assert (d_w.cpu().numpy()[a2r.reshape(wl.k, wl.T).T < 0] == 0).all()

    # ---- expert FFN backward: the oracle gets the rows and the upstream gradient the GPU used
    w1_im, w2_im, d_w1, d_b1, d_w2, d_b2 = expert_grad_buffers(wl, L)         # (the generator's arrays are input-major)
    d_xd = torch.full_like(fw["xd"], float("nan"))
    nws = M.moe_expert_ffn_backward_workspace_bytes(cfg)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    for rep in range(2):
        M.moe_expert_ffn_backward(cfg, W, w1_im, w2_im, fw["xd"], fw["h"], d_yd, fw["offsets"], d_xd, d_w1, d_b1, d_w2,
                                  d_b2, ws)
        torch.cuda.synchronize()
        ref = B.expert_ffn_backward(to_np(fw["xd"][:R]), ref_fw["expert_offsets"], L, to_np(d_yd[:R]), wl.act)
        errs = {"xd": rel_fro(to_np(d_xd[:R]), ref["xd"]), **expert_grad_errors(wl, ref, d_w1, d_b1, d_w2, d_b2)}
        print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
        assert all(v < 1e-2 for v in errs.values()), errs
        # exact products of the stored bf16 operands (h is the GPU's rounding of the activation)
        if wl.act == "gelu":
            assert errs["b2"] < 1e-5 and errs["w2"] < 6e-3
        else:
            assert errs["w_down"] < 6e-3


@pytest.mark.parametrize("name,kw", [
    ("gpt", dict(T=700, E=4, d_model=256, d_ff=512)),
    ("gpt", dict(T=1500, E=8, d_model=512, d_ff=256, capacity_factor=0.6)),
    ("skew", dict(T=900, E=8, d_model=256, d_ff=512)),                     # top-1, router bias, not renormalised
    ("gpt", dict(T=300, E=64, d_model=256, d_ff=256, k=4, capacity_factor=0.0)),
    ("gpt", dict(T=300, E=96, d_model=256, d_ff=256, k=3, capacity_factor=0.0)),   # experts in two register chunks, the second partial
    ("gpt", dict(T=200, E=128, d_model=256, d_ff=256, k=2, capacity_factor=2.0)),
    ("gpt", dict()),                          # the benchmark's configuration at full size, in its launch configuration
    ("gpt", dict(T=4, E=8, d_model=256, d_ff=256, capacity_factor=0.0)),      # forward pass on the few-token kernels
    ("gpt", dict(T=1, E=8, d_model=256, d_ff=256, capacity_factor=0.0)),
    ("skew", dict(T=1, d_model=256, d_ff=512)),
    ("large", dict(T=700, E=4, d_model=256, d_ff=512)),                                         # SwiGLU experts
    ("large", dict(T=1500, E=8, d_model=512, d_ff=256, capacity_factor=0.6)),
    ("large", dict(T=900, E=8, d_model=256, d_ff=512, k=1, capacity_factor=0.0, renormalize=False)),
], ids=lambda v: str(v).replace(" ", ""))
@pytest.mark.parametrize("grad_dtype", [torch.float32, torch.bfloat16], ids=["f32grads", "bf16grads"])
def test_layer_backward(name, kw, grad_dtype):
    """moe_layer_forward with residual = x, then moe_layer_backward: every gradient against the fp64 oracle, with the
    weight gradients in float32 and rounded once to bfloat16."""
    wl = WORKLOADS[name].scaled(**kw)
    print(f"layer backward case {wl}", flush=True)
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    ws_f = alloc_ws(cfg)
    out = torch.empty_like(x)
    M.moe_layer_forward(cfg, W, x, x, out, ws_f)
    rng = np.random.default_rng(4)
    G_np = to_np(to_dev(rng.standard_normal(L["x"].shape).astype(np.float32), wl.dtype))
    G = to_dev(G_np, wl.dtype)
    ref = B.layer_backward(L["x"], L, G_np, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor, renormalize=wl.renormalize,
                           act=wl.act)
    lay = M.moe_workspace_layout(cfg)
    from gpu_util import ws_view
    torch.cuda.synchronize()
    got_idx = ws_view(ws_f, lay["topk_idx"], wl.T * wl.k, torch.int32).cpu().numpy().reshape(wl.T, wl.k)
    fw = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor, renormalize=wl.renormalize, act=wl.act)
    assert np.array_equal(got_idx, fw["topk_idx"])
    f32 = dict(dtype=torch.float32, device="cuda")
    d_x = torch.full_like(x, float("nan"))
    d_wr = torch.full((wl.d_model, wl.E), float("nan"), **f32)
    d_br = torch.full((wl.E,), float("nan"), **f32) if "b_router" in W.tensors else None
    w1_im, w2_im, d_w1, d_b1, d_w2, d_b2 = expert_grad_buffers(wl, L, grad_dtype)
    ws_b = torch.empty(M.moe_layer_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    for rep in range(2):
        M.moe_layer_backward(cfg, W, w1_im, w2_im, x, G, G, ws_f, d_x, d_wr, d_br, d_w1, d_b1, d_w2, d_b2, ws_b)
        torch.cuda.synchronize()
        errs = {
            "x": rel_fro(to_np(d_x), ref["x"] + G_np),
            "x (experts and gate only)": rel_fro(to_np(d_x).astype(np.float64) - G_np, ref["x"]),
            "w_router": rel_fro(d_wr.cpu().numpy(), ref["w_router"]),
            **expert_grad_errors(wl, ref, d_w1, d_b1, d_w2, d_b2),
        }
        if d_br is not None:
            errs["b_router"] = rel_fro(d_br.cpu().numpy(), ref["b_router"])
        print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
        assert errs["x"] < 1e-2
        assert all(v < 2e-2 for v in errs.values()), errs


@pytest.mark.parametrize("name,kw", [
    ("gpt", dict(T=700, E=4, d_model=256, d_ff=512)),
    ("skew", dict(T=900, E=8, d_model=256, d_ff=512)),                     # top-1 with a router bias: unbalanced routing
    ("gpt", dict(T=333, E=96, d_model=256, d_ff=256, k=3, capacity_factor=0.0)),
], ids=lambda v: str(v).replace(" ", ""))
def test_aux_loss_value_and_gradient(name, kw):
    """moe_gate_aux_loss against the oracle, and its gradient alone (d_out = 0) through moe_layer_backward."""
    wl = WORKLOADS[name].scaled(**kw)
    print(f"aux loss case {wl}", flush=True)
    coef = 3.0
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    fw = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor, renormalize=wl.renormalize, act=wl.act)
    # ---- the value
    idx = torch.empty(wl.T, wl.k, dtype=torch.int32, device="cuda")
    w = torch.empty(wl.T, wl.k, dtype=torch.float32, device="cuda")
    probs = torch.empty(wl.T, wl.E, dtype=torch.float32, device="cuda")
    M.moe_gate(cfg, x, W.tensors["w_router"], W.tensors.get("b_router"), idx, w, probs)
    frac = torch.full((wl.E,), float("nan"), dtype=torch.float32, device="cuda")
    pbar = torch.full((wl.E,), float("nan"), dtype=torch.float32, device="cuda")
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    M.moe_gate_aux_loss(cfg, probs, idx, coef, frac, pbar, loss)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), fw["topk_idx"])
    counts = np.bincount(fw["topk_idx"][:, 0], minlength=wl.E)
    assert np.array_equal(frac.cpu().numpy(), (counts.astype(np.float32) / np.float32(wl.T)))        # exact counts
    assert np.allclose(pbar.cpu().numpy(), fw["probs"].mean(axis=0), rtol=1e-5, atol=1e-7)
    want = B.aux_loss(fw["probs"], fw["topk_idx"], coef)
    assert abs(loss.item() - want) <= 1e-5 * abs(want), (loss.item(), want)
    # ---- the gradient: nothing flows back from the output, so every gradient is the auxiliary loss's
    ws_f = alloc_ws(cfg)
    out = torch.empty_like(x)
    M.moe_layer_forward(cfg, W, x, None, out, ws_f)
    G = torch.zeros_like(x)
    ref = B.layer_backward(L["x"], L, np.zeros(L["x"].shape), E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                           renormalize=wl.renormalize, act=wl.act, aux_coef=coef)
    f32 = dict(dtype=torch.float32, device="cuda")
    d_x = torch.full_like(x, float("nan"))
    d_wr = torch.full((wl.d_model, wl.E), float("nan"), **f32)
    d_br = torch.full((wl.E,), float("nan"), **f32)
    w1_im, w2_im, d_w1, d_b1, d_w2, d_b2 = expert_grad_buffers(wl, L)
    ws_b = torch.empty(M.moe_layer_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    for rep in range(2):
        M.moe_layer_backward(cfg, W, w1_im, w2_im, x, G, None, ws_f, d_x, d_wr, d_br, d_w1, d_b1, d_w2, d_b2, ws_b,
                             aux_loss_coef=coef)
        torch.cuda.synchronize()
        errs = {"x": rel_fro(to_np(d_x), ref["x"]), "w_router": rel_fro(d_wr.cpu().numpy(), ref["w_router"]),
                "b_router": rel_fro(d_br.cpu().numpy(), ref["b_router"])}
        print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
        assert np.abs(ref["w_router"]).max() > 0
        assert errs["x"] < 1e-2 and errs["w_router"] < 1e-4 and errs["b_router"] < 1e-4, errs    # bf16 d_x; fp32 sums
        assert not d_w1.any() and not d_w2.any()
    # without the coefficient the same call gives zeros: the term is the only source
    M.moe_layer_backward(cfg, W, w1_im, w2_im, x, G, None, ws_f, d_x, d_wr, d_br, d_w1, d_b1, d_w2, d_b2, ws_b)
    torch.cuda.synchronize()
    assert not d_x.float().any() and not d_wr.any()


def test_layer_backward_of_an_empty_batch_gives_zero_parameter_gradients():
    wl = WORKLOADS["gpt"].scaled(T=0, E=4, d_model=256, d_ff=256)
    L = make_layer(WORKLOADS["gpt"].scaled(T=8, E=4, d_model=256, d_ff=256), with_bias=True)     # parameters only
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = torch.empty(0, wl.d_model, dtype=torch.bfloat16, device="cuda")
    ws_f = alloc_ws(cfg)
    M.moe_layer_forward(cfg, W, x, None, torch.empty_like(x), ws_f)
    f32 = dict(dtype=torch.float32, device="cuda")
    d_wr = torch.full((wl.d_model, wl.E), float("nan"), **f32)
    d_br = torch.full((wl.E,), float("nan"), **f32)
    w1_im, w2_im, d_w1, d_b1, d_w2, d_b2 = expert_grad_buffers(wl, L)
    ws_b = torch.empty(max(M.moe_layer_backward_workspace_bytes(cfg), 256), dtype=torch.uint8, device="cuda")
    M.moe_layer_backward(cfg, W, w1_im, w2_im, x, x, None, ws_f, torch.empty_like(x), d_wr, d_br, d_w1, d_b1, d_w2, d_b2, ws_b,
                         aux_loss_coef=0.5)
    torch.cuda.synchronize()
    for name, g in (("w_router", d_wr), ("b_router", d_br), ("w1", d_w1), ("b1", d_b1), ("w2", d_w2), ("b2", d_b2)):
        assert not g.any(), name                              # (zeros, not the NaNs the buffers held)


def test_backward_refuses_what_it_cannot_do():
    wl = WORKLOADS["tiny"].scaled(T=64)                       # float32 layer: the backward pass is bf16 only
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    ws_f = alloc_ws(cfg)
    buf = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_layer_backward(cfg, W, buf, buf, x, x, None, ws_f, x, buf, buf, buf, buf, buf, buf, buf)
    assert "bf16" in str(e.value)
    # a workspace that is too small is refused before anything is launched
    wl = WORKLOADS["gpt"].scaled(T=64, E=4, d_model=256, d_ff=256)
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    ws_f = alloc_ws(cfg)
    M.moe_layer_forward(cfg, W, x, None, torch.empty_like(x), ws_f)
    w1_im, w2_im, d_w1, d_b1, d_w2, d_b2 = expert_grad_buffers(wl, L)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MoEError) as e:
        M.moe_layer_backward(cfg, W, w1_im, w2_im, x, x, None, ws_f, torch.empty_like(x), buf, buf, d_w1, d_b1, d_w2, d_b2, small)
    assert "workspace" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(d_w1).all()                            # untouched
