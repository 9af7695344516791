"""GPU parity: every stage and the whole layer, through the C ABI, against the fp64 oracle.

Bars: routing tables (top-k indices, counts, offsets, permutations) and the dispatched rows are
bit-exact; fp32 gate weights within 1e-5 relative; bf16 expert outputs / layer outputs within 1e-2
relative Frobenius error; fp32 outputs within 1e-5 relative Frobenius error.
"""
import numpy as np
import pytest
import torch

import paper_2205_10034_amd as M
from oracle import moe_oracle as O
from workloads import WORKLOADS, make_layer
from workloads import bf16_round as bf16_round_np

from gpu_util import alloc_ws, rel_fro, run_layer, tdtype, to_dev, to_np, upload_weights, ws_view
from oracle_sampling import oracle_out_for_tokens

pytestmark = pytest.mark.gpu

GATE_RTOL = 1e-5
BF16_TOL = 1e-2
F32_TOL = 1e-5


def small(name, **kw):
    return WORKLOADS[name].scaled(**kw)


# ----------------------------------------------------------------------------- gate
GATE_CASES = [
    small("tiny"),
    small("tiny", T=37, E=5, k=3, renormalize=True),
    small("gpt", T=1000),
    small("gpt", T=515, E=64, k=2, d_model=512),
    small("gpt", T=300, E=100, k=4, d_model=256),
    small("gpt", T=64, E=256, k=8, d_model=128),
    small("skew", T=2048),
    small("gpt", T=3, E=2, k=2, renormalize=False),
    # at most 16 tokens and 4, 8, 16, 32 or 64 experts: one workgroup per token
    small("ring", T=1, d_model=2048),
    small("ring", T=16, d_model=512, k=8),
    small("gpt", T=5, E=32, k=3, d_model=320),
    small("skew", T=9, d_model=768),                      # 8 experts, router bias, top-1
    small("tiny", T=16, E=4, k=4),                        # float32 activations, k = E
    small("gpt", T=5, E=33, k=3, d_model=320),            # other expert counts: the general kernels
    small("gpt", T=16, E=65, k=2, d_model=256),
    # 8192 tokens and more with at most 16 experts: two 16-token tiles per workgroup; ragged ends (a last workgroup
    # with one token in its second tile, with half a first tile and no second one), a router read element-wise
    small("gpt", T=8209, d_model=256),
    small("skew", T=8200, d_model=128),
    small("gpt", T=8197, E=5, k=3, d_model=192),
]


@pytest.mark.parametrize("wl", GATE_CASES, ids=lambda w: f"{w.name}-T{w.T}-E{w.E}-k{w.k}-{w.dtype}")
def test_gate(wl):
    print(f"gate case {wl}", flush=True)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    x = to_dev(L["x"], wl.dtype)
    wr, br = to_dev(L["w_router"], "f32"), to_dev(L["b_router"], "f32")
    idx = torch.full((wl.T, wl.k), -7, dtype=torch.int32, device="cuda")
    w = torch.zeros((wl.T, wl.k), dtype=torch.float32, device="cuda")
    probs = torch.zeros((wl.T, wl.E), dtype=torch.float32, device="cuda")
    M.moe_gate(cfg, x, wr, br if wl.router_bias != "none" else None, idx, w, probs)
    torch.cuda.synchronize()
    p_ref, idx_ref, w_ref = O.gate(L["x"], L["w_router"], L["b_router"], wl.k, wl.renormalize)
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    assert np.allclose(w.cpu().numpy(), w_ref, rtol=GATE_RTOL, atol=0)
    assert np.allclose(probs.cpu().numpy(), p_ref, rtol=GATE_RTOL, atol=1e-30)


def run_gate_packed(cfg, x_np, wr_np, br_np, with_probs=True):
    x, wr = to_dev(x_np, "bf16"), to_dev(wr_np, "f32")
    br = None if br_np is None else to_dev(br_np, "f32")
    packed = torch.empty(M.moe_router_pack_bytes(cfg.d_model, cfg.E), dtype=torch.uint8, device="cuda")
    M.moe_pack_router(wr, packed)
    idx = torch.full((cfg.T, cfg.k), -7, dtype=torch.int32, device="cuda")
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    probs = torch.zeros((cfg.T, cfg.E), dtype=torch.float32, device="cuda") if with_probs else None
    M.moe_gate_packed(cfg, x, wr, br, packed, idx, w, probs)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), w.cpu().numpy(), None if probs is None else probs.cpu().numpy()


PACKED_GATE_CASES = [wl for wl in GATE_CASES if wl.dtype == "bf16" and wl.E <= 64] + [
    small("gpt", T=333, E=8, k=2, d_model=4096),           # one row block, the large workload's router
    small("gpt", T=8200, E=8, k=2, d_model=512),           # 128 tokens per workgroup, ragged last workgroup
    small("skew", T=16384 + 40, d_model=768),              # 64 tokens per workgroup; 12 stages over 8 wavefronts
    small("gpt", T=8192 + 33, E=16, k=2, d_model=256),     # two row blocks, 64 tokens per workgroup
    small("gpt", T=200, E=21, k=3, d_model=192),           # 63 rows in two blocks; 3 stages: five wavefronts idle
    small("gpt", T=100, E=32, k=4, d_model=128),           # 96 rows = three full blocks
    small("gpt", T=77, E=42, k=2, d_model=320),            # four blocks, stages of 32
    small("gpt", T=90, E=53, k=5, d_model=128),            # five blocks
    small("ring", T=4096, d_model=2048),                   # the ring workload's router: six blocks, two rounds through LDS
    # longer token streams
    small("gpt", T=5000 + 7, E=8, k=2, d_model=1024),      # one row block, two stages, ragged last workgroup
    small("gpt", T=4100, E=16, k=2, d_model=1024),         # two row blocks
    small("gpt", T=8300, E=32, k=4, d_model=512),          # three row blocks, a single stage
    small("skew", T=3000, d_model=1536),                   # router bias, three stages (odd count)
]


@pytest.mark.parametrize("wl", PACKED_GATE_CASES, ids=lambda w: f"{w.name}-T{w.T}-E{w.E}-k{w.k}-d{w.d_model}")
def test_gate_packed_router(wl):
    """The gate on the pre-split router: same bar as moe_gate (indices bit-exact, weights and probabilities 1e-5)."""
    print(f"packed gate case {wl}", flush=True)
    L = make_layer(wl.scaled(d_ff=64))
    cfg = M.MoEConfig.from_workload(wl)
    idx, w, probs = run_gate_packed(cfg, L["x"], L["w_router"], L["b_router"] if wl.router_bias != "none" else None)
    p_ref, idx_ref, w_ref = O.gate(L["x"], L["w_router"], L["b_router"], wl.k, wl.renormalize)
    assert np.array_equal(idx, idx_ref)
    assert np.allclose(w, w_ref, rtol=GATE_RTOL, atol=0)
    assert np.allclose(probs, p_ref, rtol=GATE_RTOL, atol=1e-30)


@pytest.mark.parametrize("T", [700, 8217], ids=["one-tile", "two-tiles"])
@pytest.mark.parametrize("packed", [True, False])
@pytest.mark.parametrize("scale", [1.0, 1e3, 1e-3])
def test_gate_near_ties_at_any_scale(scale, packed, T):
    """Planted near-ties: pairs of router columns that differ in the last bits of a few weights, so that two
    experts' logits differ by far less than the fast path's accumulation error, at three input scales (the
    recompute margin scales with the partial sums).  Ranking must still equal the float64 oracle's."""
    rng = np.random.default_rng(11)
    d, E, k = 1024, 16, 2                                     # (T >= 8192: moe_gate takes two token tiles per workgroup)
    x = bf16_round_np(rng.standard_normal((T, d)).astype(np.float32) * np.float32(scale))
    wr = (rng.standard_normal((d, E)) / 32).astype(np.float32)
    for a, b in ((0, 5), (3, 9), (7, 12)):                   # b is a, a few weights nudged by one unit in the last place
        wr[:, b] = wr[:, a]
        rows = rng.integers(0, d, 6)
        wr[rows, b] = np.nextafter(wr[rows, b], np.float32(np.inf))
    wr[:, :3] += np.float32(0.02)                            # make the tied experts likely winners
    wr[:, 5] += np.float32(0.02)
    cfg = M.MoEConfig(T=T, d_model=d, d_ff=64, E=E, k=k, renormalize=True, dtype="bf16")
    if packed:
        idx, w, _ = run_gate_packed(cfg, x, wr, None, with_probs=False)
    else:
        idx_t = torch.empty((T, k), dtype=torch.int32, device="cuda")
        w_t = torch.empty((T, k), dtype=torch.float32, device="cuda")
        M.moe_gate(cfg, to_dev(x, "bf16"), to_dev(wr, "f32"), None, idx_t, w_t, None)
        torch.cuda.synchronize()
        idx, w = idx_t.cpu().numpy(), w_t.cpu().numpy()
    _, idx_ref, w_ref = O.gate(x, wr, None, k, True)
    z = O.gate_logits(x, wr, None)
    top = np.sort(z, axis=1)[:, ::-1]
    print(f"scale {scale}: smallest gap among the three leading logits {np.min(top[:, :2] - top[:, 1:3]):.3e} "
          f"(logit magnitude {np.abs(z).max():.3e})", flush=True)
    assert np.array_equal(idx, idx_ref)
    # the softmax is float32 (Section 5.2): a logit of magnitude |z| is rounded to 2^-24 |z| before the
    # exponential, which is a relative error of that size in its probability
    assert np.allclose(w, w_ref, rtol=GATE_RTOL + 2.0 ** -22 * np.abs(z).max(), atol=1e-30)


@pytest.mark.parametrize("packed", [False, True])
def test_gate_exact_ties_lower_index_first(packed):
    # integer-valued x and router: logits are exact on both sides; columns repeat, so ties are real
    rng = np.random.default_rng(0)
    T, d, E = 200, 64, 6
    x = rng.integers(-3, 4, size=(T, d)).astype(np.float32)
    base = rng.integers(-2, 3, size=(d, 3)).astype(np.float32)
    wr = np.concatenate([base, base], axis=1)                  # expert e and e+3 always tie
    cfg = M.MoEConfig(T=T, d_model=d, d_ff=64, E=E, k=4, renormalize=True, dtype="bf16")
    _, idx_ref, w_ref = O.gate(x, wr, None, 4, True)
    if packed:
        idx, w, _ = run_gate_packed(cfg, x, wr, None, with_probs=False)
        assert np.array_equal(idx, idx_ref) and np.allclose(w, w_ref, rtol=GATE_RTOL)
        return
    idx = torch.empty((T, 4), dtype=torch.int32, device="cuda")
    w = torch.empty((T, 4), dtype=torch.float32, device="cuda")
    M.moe_gate(cfg, to_dev(x, "bf16"), to_dev(wr, "f32"), None, idx, w, None)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), idx_ref)
    assert np.allclose(w.cpu().numpy(), w_ref, rtol=GATE_RTOL)


# ------------------------------------------------------------------------- dispatch
def run_dispatch(cfg, x_np, idx_np, with_rows=True):
    x = to_dev(x_np, cfg.dtype)
    idx = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int32)).cuda()
    A = cfg.k * cfg.T
    counts = torch.full((cfg.E,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((cfg.E + 1,), -1, dtype=torch.int32, device="cuda")
    a2r = torch.full((max(A, 1),), -5, dtype=torch.int32, device="cuda")
    r2a = torch.full((max(A, 1),), -5, dtype=torch.int32, device="cuda")
    rmax = M.moe_workspace_layout(cfg)["r_max"]
    xd = torch.zeros((max(rmax, 1), cfg.d_model), dtype=tdtype(cfg.dtype), device="cuda") if with_rows else None
    ws = alloc_ws(cfg, 1)
    M.moe_dispatch(cfg, x, idx, counts, offsets, a2r, r2a, xd, ws)
    torch.cuda.synchronize()
    return counts.cpu().numpy(), offsets.cpu().numpy(), a2r.cpu().numpy()[:A], r2a.cpu().numpy(), xd


DISPATCH_CASES = [
    dict(T=256, E=4, k=1, cf=1.25), dict(T=1000, E=16, k=2, cf=1.25), dict(T=5000, E=8, k=1, cf=0.0),
    dict(T=3000, E=64, k=2, cf=0.0), dict(T=1025, E=3, k=3, cf=0.5), dict(T=700, E=130, k=4, cf=1.0),
    dict(T=1, E=2, k=2, cf=1.0), dict(T=4097, E=8, k=2, cf=0.05),
]


@pytest.mark.parametrize("c", DISPATCH_CASES, ids=lambda c: "T{T}-E{E}-k{k}-cf{cf}".format(**c))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dispatch(c, dtype):
    print(f"dispatch case {c} {dtype}", flush=True)
    rng = np.random.default_rng(c["T"] + c["E"])
    T, E, k = c["T"], c["E"], c["k"]
    z = rng.standard_normal((T, E)) + 1.5 * rng.standard_normal(E)        # uneven loads
    idx = O.topk_by_logit(z, k)
    wl = small("gpt", T=T, E=E, k=k, d_model=128, dtype=dtype)
    x_np = make_layer(wl.scaled(E=1, d_ff=64))["x"]
    cfg = M.MoEConfig(T=T, d_model=128, d_ff=64, E=E, k=k, capacity_factor=c["cf"], dtype=dtype)
    C = O.capacity(T, E, k, c["cf"])
    assert M.moe_capacity(cfg) == C
    counts, offsets, a2r, r2a, xd = run_dispatch(cfg, x_np, idx)
    rc, ro, ra, rr, rxd = O.dispatch(x_np, idx, E, C)
    assert np.array_equal(counts, rc) and np.array_equal(offsets, ro)
    assert np.array_equal(a2r, ra)
    R = int(ro[-1])
    assert np.array_equal(r2a[:R], rr)
    assert np.array_equal(to_np(xd[:R]), rxd)                                # byte copies
    if c["cf"] > 0 and c["cf"] < 1:
        assert (ra < 0).any()


def test_dispatch_all_tokens_one_expert_and_empty_experts():
    T, E, k = 3000, 8, 1
    idx = np.full((T, 1), 5, dtype=np.int32)
    x_np = make_layer(small("gpt", T=T, E=1, d_model=64, d_ff=64))["x"]
    for cf in (0.0, 1.0):
        cfg = M.MoEConfig(T=T, d_model=64, d_ff=64, E=E, k=k, capacity_factor=cf)
        C = O.capacity(T, E, k, cf)
        counts, offsets, a2r, r2a, xd = run_dispatch(cfg, x_np, idx)
        rc, ro, ra, rr, rxd = O.dispatch(x_np, idx, E, C)
        assert np.array_equal(counts, rc) and np.array_equal(offsets, ro) and np.array_equal(a2r, ra)
        R = int(ro[-1])
        assert R == min(T, C) and np.array_equal(r2a[:R], rr) and np.array_equal(to_np(xd[:R]), rxd)


def test_empty_batch():
    cfg = M.MoEConfig(T=0, d_model=64, d_ff=64, E=4, k=2, capacity_factor=1.0)
    counts = torch.full((4,), -1, dtype=torch.int32, device="cuda")
    offsets = torch.full((5,), -1, dtype=torch.int32, device="cuda")
    ws = alloc_ws(cfg, 1)
    M.moe_dispatch(cfg, None, None, counts, offsets, None, None, None, ws)
    torch.cuda.synchronize()
    assert counts.cpu().tolist() == [0] * 4 and offsets.cpu().tolist() == [0] * 5


# ----------------------------------------------------------------- expert FFN + combine
FFN_CASES = [
    small("tiny", T=300, E=4, d_model=128, d_ff=256, act="gelu", dtype="f32"),
    small("tiny", T=300, E=3, d_model=64, d_ff=192, act="swiglu", dtype="f32"),
    small("gpt", T=1500, E=4, d_model=256, d_ff=512, act="gelu"),          # 256-wide tiles, ragged rows
    small("gpt", T=900, E=5, d_model=192, d_ff=320, act="gelu"),           # narrow-tile fallback
    small("gpt", T=1500, E=4, d_model=256, d_ff=384, act="swiglu"),
    small("gpt", T=700, E=3, d_model=192, d_ff=192, act="swiglu"),
    small("gpt", T=5, E=4, d_model=256, d_ff=512, act="gelu"),             # few rows: matrix-vector kernels on dispatched rows
    small("gpt", T=8, E=3, d_model=320, d_ff=256, act="swiglu"),
]


@pytest.mark.parametrize("wl", FFN_CASES, ids=lambda w: f"{w.act}-{w.dtype}-T{w.T}-E{w.E}-d{w.d_model}-f{w.d_ff}")
def test_expert_ffn_and_combine(wl):
    print(f"ffn case {wl}", flush=True)
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    ref = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                          renormalize=wl.renormalize, act=wl.act)
    W = upload_weights(L, wl.dtype)
    R = int(ref["expert_offsets"][-1])
    xd = to_dev(ref["xd"], wl.dtype)
    offsets = torch.from_numpy(ref["expert_offsets"]).cuda()
    yd = torch.zeros((max(R, 1), wl.d_model), dtype=tdtype(wl.dtype), device="cuda")
    ws = alloc_ws(cfg, 2)
    M.moe_expert_ffn(cfg, W, xd, offsets, yd, ws)
    torch.cuda.synchronize()
    tol = BF16_TOL if wl.dtype == "bf16" else F32_TOL
    err = rel_fro(to_np(yd[:R]), ref["yd"])
    print("yd rel fro", err, flush=True)
    assert err < tol
    # per-expert check too: a wrong expert index on a small expert must not hide in the norm
    for e in range(wl.E):
        lo, hi = ref["expert_offsets"][e], ref["expert_offsets"][e + 1]
        if hi > lo:
            assert rel_fro(to_np(yd[lo:hi]), ref["yd"][lo:hi]) < tol
    # combine on the oracle's routing and the GPU's yd
    a2r = torch.from_numpy(ref["assign_to_row"]).cuda()
    tw = torch.from_numpy(ref["topk_w"].astype(np.float32)).cuda()
    res_np = make_layer(wl.scaled(seed=wl.seed + 99))["x"]
    res = to_dev(res_np, wl.dtype)
    out = torch.empty((wl.T, wl.d_model), dtype=tdtype(wl.dtype), device="cuda")
    M.moe_combine(cfg, yd, a2r, tw, res, out)
    torch.cuda.synchronize()
    ref_out = O.combine(to_np(yd[:R]).astype(np.float64), ref["assign_to_row"], tw.cpu().numpy().astype(np.float64), res_np)
    assert rel_fro(to_np(out), ref_out) < (4e-3 if wl.dtype == "bf16" else 1e-6)   # one rounding of the sum
    M.moe_combine(cfg, yd, a2r, tw, None, out)
    torch.cuda.synchronize()
    ref_out = O.combine(to_np(yd[:R]).astype(np.float64), ref["assign_to_row"], tw.cpu().numpy().astype(np.float64), None)
    assert rel_fro(to_np(out), ref_out) < (4e-3 if wl.dtype == "bf16" else 1e-6)


def test_f32_ffn_input_major_layout():
    wl = small("tiny", T=200, E=3, d_model=64, d_ff=128)
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    ref = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor, renormalize=False, act="gelu")
    W = upload_weights(L, "f32", layout="input_major")
    r = run_layer(cfg, W, to_dev(L["x"], "f32"))
    assert np.array_equal(r["topk_idx"], ref["topk_idx"])
    assert rel_fro(r["out"], ref["out"]) < F32_TOL


# ------------------------------------------------------------------------- whole layer
def check_layer(wl, L, r, ref, tol):
    assert np.array_equal(r["topk_idx"], ref["topk_idx"])
    assert np.allclose(r["topk_w"], ref["topk_w"], rtol=GATE_RTOL, atol=0)
    assert np.array_equal(r["expert_counts"], ref["expert_counts"])
    assert np.array_equal(r["expert_offsets"], ref["expert_offsets"])
    assert np.array_equal(r["assign_to_row"], ref["assign_to_row"])
    assert np.array_equal(r["row_to_assign"], ref["row_to_assign"])
    if wl.dtype == "f32":            # bf16: the first GEMM gathers rows from x itself, xd is not materialised
        assert np.array_equal(r["xd"], ref["xd"])


LAYER_CASES = [
    ("tiny", {}),
    ("tiny", dict(T=777, capacity_factor=0.5, k=2, renormalize=True)),
    ("gpt", dict(T=1300, E=8)),
    ("gpt", dict(T=2048, E=16, capacity_factor=0.7)),
    ("skew", dict(T=3001)),
    ("large", dict(T=1536, d_model=512, d_ff=1024, E=4)),
    ("ring", dict(T=1024, d_model=256, d_ff=512, E=64)),
    ("gpt", dict(T=130, E=4, k=4)),
    ("ring", dict(d_ff=2048)),                      # 4096 tokens over 64 experts: ~128 rows per expert
    # one expert per token in bf16: the second GEMM finishes the combine (rows go straight to their tokens)
    ("gpt", dict(T=1300, E=8, k=1, capacity_factor=0.6)),          # about half the tokens dropped
    ("large", dict(T=1111, d_model=512, d_ff=1024, E=4, k=1)),     # SwiGLU
    ("ring", dict(T=1500, d_model=320, d_ff=512, E=32, k=1, capacity_factor=1.0)),   # narrow output tiles
    # steps of very few tokens (at most 8 assignments): the matrix-vector kernels
    ("ring", dict(T=1, d_model=256, d_ff=512, E=64)),
    ("ring", dict(T=4, d_model=512, d_ff=1024, E=64)),
    ("gpt", dict(T=3, E=8, d_model=320, d_ff=512, capacity_factor=0.0)),       # K no multiple of 512: ragged last K block
    ("gpt", dict(T=4, E=2, d_model=256, d_ff=512, capacity_factor=0.0)),       # several rows per expert
    ("gpt", dict(T=4, E=2, d_model=256, d_ff=512, capacity_factor=0.5)),       # ... with drops
    ("skew", dict(T=7, d_model=256, d_ff=512)),                                # top-1: combine in the second product
    ("gpt", dict(T=8, E=4, d_model=256, d_ff=256, k=1, capacity_factor=0.5)),  # top-1 with dropped tokens
    ("large", dict(T=2, d_model=512, d_ff=1024, E=4)),                         # SwiGLU
    ("large", dict(T=5, d_model=512, d_ff=1024, E=4, k=1)),
    # one token: the gate's kernel writes the dispatch tables too
    ("skew", dict(T=1, d_model=256, d_ff=512)),
    ("large", dict(T=1, d_model=512, d_ff=1024, E=4)),
    ("gpt", dict(T=1, E=16, k=8, d_model=256, d_ff=256, capacity_factor=0.05)),   # capacity 1: still nothing dropped
    ("ring", dict(T=8, d_model=256, d_ff=512, E=64)),                          # 9 to 16 assignments: the 4 x 16 shape
    ("gpt", dict(T=6, E=2, d_model=256, d_ff=512, capacity_factor=0.0)),       # up to 12 rows in one expert
    ("skew", dict(T=13, d_model=256, d_ff=512)),
    ("large", dict(T=7, d_model=512, d_ff=1024, E=4)),
]


def max_block_err(got, ref, rows):
    """Largest relative Frobenius error over blocks of `rows` consecutive rows (blocks whose reference is all
    zero - tokens with every choice dropped - must be zero in `got` too)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    n = (len(ref) // rows) * rows
    worst = 0.0
    for a, b in ((got[:n].reshape(-1, rows * ref.shape[1]), ref[:n].reshape(-1, rows * ref.shape[1])), (got[n:].reshape(1, -1), ref[n:].reshape(1, -1))):
        if b.size == 0:
            continue
        num, den = np.linalg.norm(a - b, axis=1), np.linalg.norm(b, axis=1)
        assert np.all(num[den == 0] == 0)
        worst = max(worst, float(np.max(num[den > 0] / den[den > 0], initial=0.0)))
    return worst


def top1_fused(wl):
    """One expert per token in bf16: no dispatched-order output exists, the second GEMM writes `out`."""
    return wl.k == 1 and wl.dtype == "bf16"


@pytest.mark.parametrize("name,kw", LAYER_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_layer_forward_small(name, kw):
    wl = small(name, **kw)
    print(f"layer case {wl}", flush=True)
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    ref = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                          renormalize=wl.renormalize, act=wl.act)
    W = upload_weights(L, wl.dtype)
    r = run_layer(cfg, W, to_dev(L["x"], wl.dtype))
    check_layer(wl, L, r, ref, None)
    tol = BF16_TOL if wl.dtype == "bf16" else F32_TOL
    e_yd = 0.0 if top1_fused(wl) else rel_fro(r["yd"], ref["yd"])
    e_out = rel_fro(r["out"], ref["out"])
    print(f"rel fro yd {e_yd:.3e} out {e_out:.3e}", flush=True)
    assert e_yd < tol and e_out < tol
    # with residual, in place on the residual buffer
    res = to_dev(L["x"], wl.dtype).clone()
    ws = alloc_ws(cfg)
    M.moe_layer_forward(cfg, W, res, res, res, ws)
    torch.cuda.synchronize()
    ref_res = ref["out"] + L["x"]
    assert rel_fro(to_np(res), ref_res) < tol


@pytest.mark.parametrize("name", ["gpt", "skew", "skew40"])
def test_layer_forward_full_size(name):
    """Full configuration in the launch shape the bench times; the oracle runs the whole layer."""
    wl = WORKLOADS[name]
    print(f"full-size layer {wl}", flush=True)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    ref = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                          renormalize=wl.renormalize, act=wl.act)
    W = upload_weights(L, wl.dtype, nullable_bias=True)
    r = run_layer(cfg, W, to_dev(L["x"], wl.dtype))
    check_layer(wl, L, r, ref, None)
    e_yd = 0.0 if top1_fused(wl) else rel_fro(r["yd"], ref["yd"])
    e_out = rel_fro(r["out"], ref["out"])
    print(f"{name}: loads {ref['expert_counts'].tolist()} rel fro yd {e_yd:.3e} out {e_out:.3e}", flush=True)
    assert e_yd < BF16_TOL and e_out < BF16_TOL
    # the same bar on every block of 64 consecutive tokens and, for the dispatched-order output, on every
    # block of 64 rows and every expert (a wrong tile cannot hide in the whole-matrix norm); three times the bar
    # on every single token (one row's rounding errors do not average out as a block's do)
    worst_blk, worst_tok = max_block_err(r["out"], ref["out"], 64), max_block_err(r["out"], ref["out"], 1)
    print(f"{name}: worst 64-token block {worst_blk:.3e}, worst token {worst_tok:.3e}", flush=True)
    assert worst_blk < BF16_TOL and worst_tok < 3 * BF16_TOL
    if not top1_fused(wl):
        assert max_block_err(r["yd"], ref["yd"], 64) < BF16_TOL
        off = ref["expert_offsets"]
        for e in range(wl.E):
            if off[e + 1] > off[e]:
                assert rel_fro(r["yd"][off[e]:off[e + 1]], ref["yd"][off[e]:off[e + 1]]) < BF16_TOL


def test_layer_forward_large_sampled():
    """32768 x 4096 x 14336 SwiGLU: routing compared in full, outputs on sampled tokens the oracle
    computes one by one (the full fp64 FFN is 23 TFLOP)."""
    wl = WORKLOADS["large"]
    print(f"full-size layer {wl}", flush=True)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    p, idx, w = O.gate(L["x"], L["w_router"], L["b_router"], wl.k, wl.renormalize)
    C = O.capacity(wl.T, wl.E, wl.k, wl.capacity_factor)
    counts, offsets, a2r, r2a = O.dispatch_plan(idx, wl.E, C)
    W = upload_weights(L, wl.dtype, nullable_bias=True)
    r = run_layer(cfg, W, to_dev(L["x"], wl.dtype))
    assert np.array_equal(r["topk_idx"], idx) and np.allclose(r["topk_w"], w, rtol=GATE_RTOL, atol=0)
    assert np.array_equal(r["expert_counts"], counts) and np.array_equal(r["expert_offsets"], offsets)
    assert np.array_equal(r["assign_to_row"], a2r) and np.array_equal(r["row_to_assign"], r2a)
    assert (a2r < 0).any()                                   # capacity factor 1.0 drops some
    # Sampled tokens, chosen by construction so that no tile position can be wrong unseen: the first and last
    # row of every expert; both sides of every 256-row boundary of the fullest and the emptiest expert and of
    # every 320-row boundary of the fullest (the tile capacities of the grouped GEMM); the last rows of every
    # expert's last 64-row unit; tokens of every pattern of dropped choices; and random ones.
    rng = np.random.default_rng(0)
    rows = []
    for e in range(wl.E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            rows += [lo, hi - 1, lo + (hi - lo - 1) // 64 * 64]
    fullest, emptiest = int(np.argmax(counts)), int(np.argmin(counts))
    for e, step in ((fullest, 256), (emptiest, 256), (fullest, 320)):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        for b in range(lo + step, hi, step):
            rows += [b - 1, b]
    toks = [int(r2a[r_]) % wl.T for r_ in rows]
    kept = (a2r.reshape(wl.k, wl.T) >= 0)
    for pattern in ((True, True), (True, False), (False, True), (False, False)):
        hit = np.nonzero((kept[0] == pattern[0]) & (kept[1] == pattern[1]))[0]
        print(f"large: {len(hit)} tokens with (first, second) choice kept = {pattern}", flush=True)
        toks += hit[:6].tolist() + hit[-2:].tolist()
    toks = np.unique(np.concatenate([np.array(toks, dtype=np.int64), rng.integers(0, wl.T, 40), [0, wl.T - 1]]))
    plan = dict(topk_idx=idx, topk_w=w, assign_to_row=a2r)
    ref = oracle_out_for_tokens(O, L["x"], L, plan, toks, act=wl.act)
    got = r["out"][toks]
    err = rel_fro(got, ref)
    print(f"large: loads {counts.tolist()} dropped {(a2r < 0).sum()} sampled tokens {len(toks)} rel fro {err:.3e}", flush=True)
    assert err < BF16_TOL
    for i, t in enumerate(toks):
        if np.any(ref[i]):
            assert rel_fro(got[i], ref[i]) < 3 * BF16_TOL, f"token {t}"
        else:
            assert not np.any(got[i]), f"token {t}: every choice dropped, output must be zero"
    # properties that hold at any size, over ALL tokens: a token whose choices were all dropped is exactly zero;
    # every other row is finite and non-zero
    all_dropped = ~kept.any(axis=0)
    assert not np.any(r["out"][all_dropped])
    assert np.isfinite(r["out"]).all() and np.all(np.any(r["out"][~all_dropped] != 0, axis=1))


def test_layer_forward_ring_layer_full_size_sampled():
    """One layer of the ring workload at full size (4096 x 2048 x 8192, 64 experts, ~128 rows per expert:
    the weight-streaming regime of the grouped GEMMs): routing compared in full, outputs on sampled tokens."""
    wl = WORKLOADS["ring"]
    print(f"full-size layer {wl}", flush=True)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    p, idx, w = O.gate(L["x"], L["w_router"], L["b_router"], wl.k, wl.renormalize)
    C = O.capacity(wl.T, wl.E, wl.k, wl.capacity_factor)
    counts, offsets, a2r, r2a = O.dispatch_plan(idx, wl.E, C)
    W = upload_weights(L, wl.dtype, nullable_bias=True)
    r = run_layer(cfg, W, to_dev(L["x"], wl.dtype))
    assert np.array_equal(r["topk_idx"], idx) and np.allclose(r["topk_w"], w, rtol=GATE_RTOL, atol=0)
    assert np.array_equal(r["expert_counts"], counts) and np.array_equal(r["expert_offsets"], offsets)
    assert np.array_equal(r["assign_to_row"], a2r) and np.array_equal(r["row_to_assign"], r2a)
    rng = np.random.default_rng(1)
    smallest, largest = int(np.argmin(counts)), int(np.argmax(counts))
    edge = [int(r2a[offsets[e]]) % wl.T for e in (smallest, largest) if counts[e]] + \
           [int(r2a[offsets[e + 1] - 1]) % wl.T for e in (smallest, largest) if counts[e]]
    toks = np.unique(np.concatenate([rng.integers(0, wl.T, 60), edge, [0, wl.T - 1]]))
    plan = dict(topk_idx=idx, topk_w=w, assign_to_row=a2r)
    ref = O.sampled_tokens_forward(L["x"], L, plan, toks, act=wl.act)
    err = rel_fro(r["out"][toks], ref)
    print(f"ring layer: rows per expert {int(counts.min())}..{int(counts.max())} sampled rel fro {err:.3e}", flush=True)
    assert err < BF16_TOL
    for i, t in enumerate(toks):
        assert rel_fro(r["out"][t], ref[i]) < 3 * BF16_TOL


@pytest.mark.parametrize("with_bias", [False, True])
def test_layer_forward_top1_writes_every_token(with_bias):
    """k = 1 in bf16: kept tokens are written by the second GEMM's epilogue and dropped ones by the fill
    kernel; with a separate residual buffer, without one, and with `out` full of NaNs beforehand."""
    wl = small("gpt", T=2500, E=8, k=1, capacity_factor=0.5)
    L = make_layer(wl, with_bias=with_bias)
    cfg = M.MoEConfig.from_workload(wl)
    ref = O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                          renormalize=wl.renormalize, act=wl.act)
    dropped = ref["assign_to_row"] < 0
    assert dropped.sum() > wl.T // 4 and (~dropped).sum() > wl.T // 4
    W = upload_weights(L, wl.dtype, nullable_bias=True)
    x = to_dev(L["x"], wl.dtype)
    ws = alloc_ws(cfg)
    out = torch.full_like(x, float("nan"))
    M.moe_layer_forward(cfg, W, x, None, out, ws)
    torch.cuda.synchronize()
    got = to_np(out)
    assert np.isfinite(got).all()
    assert (got[dropped] == 0).all()
    assert rel_fro(got, ref["out"]) < BF16_TOL
    rng = np.random.default_rng(11)
    res_np = to_np(to_dev(rng.standard_normal(L["x"].shape).astype(np.float32), wl.dtype))   # bf16-representable
    res = to_dev(res_np, wl.dtype)
    out.fill_(float("nan"))
    M.moe_layer_forward(cfg, W, x, res, out, ws)
    torch.cuda.synchronize()
    got = to_np(out)
    assert np.array_equal(got[dropped], res_np[dropped])
    assert rel_fro(got, ref["out"] + res_np) < BF16_TOL


@pytest.mark.parametrize("name,kw", [("gpt", dict(T=1500, E=8)), ("gpt", dict(T=40, E=16, k=2, capacity_factor=0.0)),
                                     ("skew", dict(T=2000)), ("large", dict(T=900, d_model=512, d_ff=1024, E=4)),
                                     ("ring", dict(T=64, d_model=512, d_ff=1024, E=64, capacity_factor=0.0)),
                                     # few tokens: the matrix-vector kernels read the scattered experts too
                                     ("skew", dict(T=3, d_model=256, d_ff=512)), ("gpt", dict(T=1, E=16, d_model=256, d_ff=512)),
                                     ("large", dict(T=6, d_model=512, d_ff=1024, E=4))],
                         ids=lambda v: str(v).replace(" ", ""))
def test_layer_with_experts_scattered_over_a_pool(name, kw):
    """Route, then experts, with every expert's parameters in its own slot of a pool (shuffled slots, one
    offset per expert): bit-identical to moe_layer_forward on the [E, ...] arrays."""
    wl = small(name, **kw)
    L = make_layer(wl, with_bias=True)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    want = run_layer(cfg, W, x)
    E, d, f = wl.E, wl.d_model, wl.d_ff
    names = ["w1", "w2", "b1", "b2"] if wl.act == "gelu" else ["w_gate_proj", "w_up", "w_down"]
    parts = [W.tensors[n] for n in names if n in W.tensors]
    sizes = [p[0].numel() for p in parts]
    stride = (sum(sizes) + 127) // 128 * 128
    n_slots = E + 3
    pool = torch.full((n_slots * stride,), float("nan"), dtype=torch.bfloat16, device="cuda")
    rng = np.random.default_rng(5)
    slot_of = rng.permutation(n_slots)[:E]
    counts = want["expert_counts"]
    for e in range(E):
        if counts[e] == 0:
            continue                                   # an expert without rows needs no slot at all
        o = int(slot_of[e]) * stride
        for p_, n in zip(parts, sizes):
            pool[o:o + n] = p_[e].reshape(-1)
            o += n
    offs = torch.tensor([int(slot_of[e]) * stride if counts[e] else 0 for e in range(E)], dtype=torch.int64, device="cuda")
    t = {"w_router": W.tensors["w_router"], "expert_elem_offset": offs}
    for n in ("b_router", "w_router_packed"):            # the same gate as the reference run
        if n in W.tensors:
            t[n] = W.tensors[n]
    base = pool.data_ptr()
    o = 0
    for n_, size in zip([n for n in names if n in W.tensors], sizes):
        t[n_] = base + 2 * o
        o += size
    Wp = M.Weights(t)
    ws = alloc_ws(cfg)
    out = torch.full_like(x, float("nan"))
    M.moe_layer_route(cfg, Wp, x, ws)
    torch.cuda.synchronize()
    lay = M.moe_workspace_layout(cfg)
    got_counts = ws_view(ws, lay["expert_counts"], E, torch.int32).cpu().numpy()
    assert np.array_equal(got_counts, counts)          # what a caller reads before it places the experts
    M.moe_layer_experts(cfg, Wp, x, None, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, want["out_tensor"])


def test_layer_experts_runs_again_on_the_same_routing():
    """moe_layer_route once, moe_layer_experts twice (and a third time after another layer's whole forward
    on a second workspace): the expert half leaves the routing tables and its own work counters as it found
    them, so every run gives the same bits as moe_layer_forward."""
    for name, kw in (("gpt", dict(T=2048, E=8)), ("skew", dict(T=3001)), ("large", dict(T=1536, d_model=512, d_ff=1024, E=4))):
        wl = small(name, **kw)
        L = make_layer(wl, with_bias=True)
        cfg = M.MoEConfig.from_workload(wl)
        W = upload_weights(L, wl.dtype)
        x = to_dev(L["x"], wl.dtype)
        want = run_layer(cfg, W, x)["out_tensor"]
        ws = alloc_ws(cfg)
        M.moe_layer_route(cfg, W, x, ws)
        for rep in range(3):
            out = torch.full_like(x, float("nan"))
            M.moe_layer_experts(cfg, W, x, None, out, ws)
            torch.cuda.synchronize()
            assert torch.equal(out, want), f"{name}: run {rep} of the expert half differs"


def test_both_matrix_instructions_give_the_same_bits():
    """The grouped GEMM multiplies with 16x16x32 or 32x32x16 MFMAs (chosen from the expected rows per expert);
    the layer's output does not depend on which: GELU with biases, SwiGLU, the fused top-1 combine, ragged experts."""
    for name, kw in (("gpt", dict(T=2048, E=8)), ("skew", dict(T=3001)), ("large", dict(T=1536, d_model=512, d_ff=1024, E=4))):
        wl = small(name, **kw)
        L = make_layer(wl, with_bias=True)
        cfg = M.MoEConfig.from_workload(wl)
        W = upload_weights(L, wl.dtype)
        x = to_dev(L["x"], wl.dtype)
        outs = {}
        try:
            M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, 256)
            for shape in (16, 32):
                M.moe_set_tuning(M.MOE_TUNE_GEMM_MFMA, shape)
                outs[shape] = run_layer(cfg, W, x)["out_tensor"].clone()
        finally:
            M.moe_set_tuning(M.MOE_TUNE_GEMM_MFMA, 0)
            M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, 0)
        assert torch.equal(outs[16], outs[32]), name


def test_determinism():
    wl = small("gpt", T=2048, E=8)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    a = run_layer(cfg, W, x)["out_tensor"]
    b = run_layer(cfg, W, x)["out_tensor"]
    assert torch.equal(a, b)


def test_layer_forward_does_not_need_a_cleared_workspace():
    """Nothing in the workspace has to be zero (or anything else) on entry: random bytes, and the leftovers of
    a call with a different routing, give the same bits as a cleared workspace."""
    wl = small("gpt", T=2048, E=8)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    want = run_layer(cfg, W, x)["out_tensor"]
    ws = alloc_ws(cfg)
    g = torch.Generator(device="cuda").manual_seed(5)
    ws.copy_(torch.randint(0, 256, ws.shape, dtype=torch.uint8, device="cuda", generator=g))
    out = torch.empty_like(x)
    M.moe_layer_forward(cfg, W, x, None, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    x2 = to_dev(make_layer(wl.scaled(seed=wl.seed + 7))["x"], wl.dtype)   # other tokens, other routing
    M.moe_layer_forward(cfg, W, x2, None, out, ws)
    M.moe_layer_forward(cfg, W, x, None, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, want)


@pytest.mark.parametrize("kw", [dict(T=2048, E=8), dict(T=1, E=8), dict(T=6, E=16)], ids=lambda v: str(v).replace(" ", ""))
def test_layer_forward_in_a_hip_graph(kw):
    """The call allocates nothing and never synchronises, so it can be captured; every replay (with eager
    work and synchronisations in between) gives the eager result bit for bit.  (T = 1 and 6: the few-token kernels.)"""
    wl = small("gpt", **kw)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype)
    x = to_dev(L["x"], wl.dtype)
    want = run_layer(cfg, W, x)["out_tensor"]
    ws = alloc_ws(cfg)
    out = torch.zeros_like(x)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        M.moe_layer_forward(cfg, W, x, None, out, ws, side)      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        M.moe_layer_forward(cfg, W, x, None, out, ws, torch.cuda.current_stream())
    for rep in range(4):
        out.fill_(float("nan"))
        ws.fill_(rep)                       # eager work between the replays; the workspace content must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep} differs from the eager result"
