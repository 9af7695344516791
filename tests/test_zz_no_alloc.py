"""moe_dispatch_static (the entry point that allocates nothing: static device scratch inside the library)
against moe_dispatch with a caller workspace, through the C ABI: every table and the copied rows bit for bit,
on calls that follow each other on one GPU with shrinking and growing inputs (the shared scratch keeps the
previous call's contents), plus the size limit and the oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2205_10034_amd as M
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu


def tables(cfg, idx, x, static):
    A = cfg.k * cfg.T
    counts = torch.full((cfg.E,), -7, dtype=torch.int32, device="cuda")
    offsets = torch.full((cfg.E + 1,), -7, dtype=torch.int32, device="cuda")
    a2r = torch.full((max(A, 1),), -7, dtype=torch.int32, device="cuda")
    r2a = torch.full((max(A, 1),), -7, dtype=torch.int32, device="cuda")
    xd = torch.zeros((max(A, 1), cfg.d_model), dtype=x.dtype, device="cuda")
    if static:
        M.moe_dispatch_static(cfg, x, idx, counts, offsets, a2r, r2a, xd)
    else:
        n = M.moe_workspace_bytes(cfg, M.binding.MOE_WS_DISPATCH)
        ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        M.moe_dispatch(cfg, x, idx, counts, offsets, a2r, r2a, xd, ws)
    torch.cuda.synchronize()
    R = int(offsets[-1].item())
    return counts.cpu().numpy(), offsets.cpu().numpy(), a2r.cpu().numpy()[:A], r2a.cpu().numpy()[:R], xd[:R].cpu()


# in this order on one GPU: large (scan kernel: more than 256 blocks), smaller, tiny (single block), empty,
# larger again
CASES = [dict(T=40000, E=16, k=2, cf=1.25), dict(T=5000, E=16, k=2, cf=0.5), dict(T=37, E=64, k=3, cf=0.0),
         dict(T=0, E=4, k=1, cf=1.0), dict(T=9000, E=130, k=4, cf=1.0)]


def test_static_scratch_dispatch_equals_workspace_dispatch_on_consecutive_calls():
    for c in CASES:
        print(f"static dispatch case {c}", flush=True)
        T, E, k = c["T"], c["E"], c["k"]
        rng = np.random.default_rng(T + E)
        idx_np = O.topk_by_logit(rng.standard_normal((T, E)) + 1.5 * rng.standard_normal(E), k).astype(np.int32)
        idx = torch.from_numpy(idx_np.reshape(T, k)).cuda()
        x = torch.from_numpy(rng.standard_normal((max(T, 1), 128)).astype(np.float32)).cuda().to(torch.bfloat16)[:T]
        cfg = M.MoEConfig(T=T, d_model=128, d_ff=64, E=E, k=k, capacity_factor=c["cf"], dtype="bf16")
        got = tables(cfg, idx, x, static=True)
        want = tables(cfg, idx, x, static=False)
        for g, w, name in zip(got, want, ("counts", "offsets", "assign_to_row", "row_to_assign", "xd")):
            assert (torch.equal(g, w) if name == "xd" else np.array_equal(g, w)), f"{c}: {name} differs"
        # and both equal the oracle's plan
        rc, ro, ra, rr = O.dispatch_plan(idx_np.reshape(T, k), E, O.capacity(T, E, k, c["cf"]))
        assert np.array_equal(got[0], rc) and np.array_equal(got[1], ro)
        assert np.array_equal(got[2], ra) and np.array_equal(got[3], rr)


def test_static_scratch_dispatch_rejects_sizes_beyond_its_buffer():
    # 2^20 assignments over 256 experts: (4096 + 1) * 256 * 4 bytes of block histograms > 1 MiB
    cfg = M.MoEConfig(T=1 << 20, d_model=64, d_ff=64, E=256, k=1, capacity_factor=0.0, dtype="bf16")
    assert M.moe_workspace_bytes(cfg, M.binding.MOE_WS_DISPATCH) > (1 << 20)
    fake = C.c_void_p(0x1000)
    c = cfg.c()
    st = M.lib().moe_dispatch_static(C.byref(c), fake, fake, fake, fake, fake, fake, None, None)
    assert st == 2 and b"static" in M.lib().moe_last_error()
