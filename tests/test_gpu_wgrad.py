"""Weight-gradient product of the expert FFN's backward pass on the GPU against the oracle: ragged row counts
around every boundary of the 32-row K-step (empty experts, 1 row, 31/32/33, several steps with a short or
a full tail), several tile grids, values with and without cancellation."""
import numpy as np
import pytest
import torch

import paper_2205_10034_amd as M
from oracle import moe_backward_oracle as B

from gpu_util import rel_fro, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rows,N1,N2", [
    ([0, 1, 31, 32, 33, 0, 64, 95, 96, 97], 256, 256),
    ([200, 0, 0, 517, 3], 512, 256),
    ([1000, 1100], 256, 768),
    ([129], 1024, 512),
    ([0, 0], 256, 256),
])
def test_wgrad_matches_oracle(rows, N1, N2):
    print(f"wgrad rows={rows} N1={N1} N2={N2}", flush=True)
    E, R = len(rows), int(sum(rows))
    rng = np.random.default_rng(len(rows) * 1000 + N1 + N2)
    offsets_np = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    a = to_dev(rng.standard_normal((max(R, 1), N1)).astype(np.float32), "bf16")
    b = to_dev((rng.standard_normal((max(R, 1), N2)) + 0.5).astype(np.float32), "bf16")
    ref = B.expert_wgrad(a.float().cpu().numpy()[:R], b.float().cpu().numpy()[:R], offsets_np)
    c = torch.full((E, N1, N2), float("nan"), dtype=torch.float32, device="cuda")
    offsets = torch.from_numpy(offsets_np).cuda()
    sums = torch.full((E, N1), float("nan"), dtype=torch.float32, device="cuda")
    a_np = a.float().cpu().numpy().astype(np.float64)
    for rep in range(2):
        c.fill_(float("nan"))
        sums.fill_(float("nan"))
        # the second call also asks for the column sums of a (the bias gradient that goes with the product)
        M.moe_expert_wgrad(a, b, offsets, c, max(rows + [1]), a_column_sums=sums if rep else None)
        torch.cuda.synchronize()
        got = c.cpu().numpy()
        assert np.isfinite(got).all()
        if rep:
            got_sums = sums.cpu().numpy()
            for e in range(E):
                want = a_np[offsets_np[e]:offsets_np[e + 1]].sum(axis=0)         # the definition: a plain column sum
                assert np.allclose(got_sums[e], want, rtol=1e-5, atol=1e-5 * np.sqrt(max(rows[e], 1))), f"column sums, expert {e}"
        else:
            assert torch.isnan(sums).all()                                      # not asked for: not touched
        for e in range(E):
            if rows[e] == 0:
                assert not got[e].any()
            else:
                err = rel_fro(got[e], ref[e])
                assert err < 1e-5, f"expert {e} ({rows[e]} rows): rel err {err}"
                # element-wise as well: fp32 accumulation of exact products
                assert np.allclose(got[e], ref[e], rtol=1e-4, atol=1e-4 * np.sqrt(rows[e]))


@pytest.mark.parametrize("rows,N1,N2", [([0, 1, 33, 0, 95, 256], 256, 512), ([1000, 1100], 256, 768)])
def test_wgrad_bf16_output_is_the_float32_result_rounded_once(rows, N1, N2):
    """c as bfloat16: bit for bit the float32 result of the same call rounded to nearest even (the sums are the same
    fp32 accumulators); experts without rows come out as zeros; the column sums stay float32."""
    E, R = len(rows), int(sum(rows))
    rng = np.random.default_rng(7 + N1 + N2)
    offsets = torch.from_numpy(np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)).cuda()
    a = to_dev(rng.standard_normal((R, N1)).astype(np.float32), "bf16")
    b = to_dev((rng.standard_normal((R, N2)) + 0.5).astype(np.float32), "bf16")
    c32 = torch.full((E, N1, N2), float("nan"), dtype=torch.float32, device="cuda")
    c16 = torch.full((E, N1, N2), float("nan"), dtype=torch.bfloat16, device="cuda")
    s32 = torch.full((E, N1), float("nan"), dtype=torch.float32, device="cuda")
    s16 = torch.full((E, N1), float("nan"), dtype=torch.float32, device="cuda")
    M.moe_expert_wgrad(a, b, offsets, c32, max(rows), a_column_sums=s32)
    M.moe_expert_wgrad(a, b, offsets, c16, max(rows), a_column_sums=s16)
    torch.cuda.synchronize()
    assert torch.equal(c16, c32.to(torch.bfloat16))
    assert torch.equal(s16, s32)


def test_wgrad_rejects_what_it_cannot_do():
    a = torch.zeros(8, 128, dtype=torch.bfloat16, device="cuda")
    offsets = torch.tensor([0, 8], dtype=torch.int32, device="cuda")
    c = torch.zeros(1, 128, 256, dtype=torch.float32, device="cuda")
    with pytest.raises(M.MoEError):
        M.moe_expert_wgrad(a, a, offsets, c, 8)
