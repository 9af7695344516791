"""Ring memory offloading on the GPU (Section 3.3.2): a stack of MoE layers whose expert weights live
in pinned host memory and stream through K HBM sections while the layers compute.

Checks: the ring-streamed stack is bit-identical to the same stack with every layer resident; each
layer matches the oracle when the oracle is fed the GPU's own input of that layer (teacher forcing:
a free-running fp64 chain would route differently after one bf16 layer); the bytes copied equal the
schedule's; wrap-around over two inference steps with N not a multiple of K.
"""
import numpy as np
import pytest
import torch

import paper_2205_10034_amd as M
from oracle import moe_oracle as O
from workloads import WORKLOADS, make_ring_stack

from gpu_util import alloc_ws, rel_fro, to_dev, to_np

pytestmark = pytest.mark.gpu


def pack_layer_host(L, wl):
    """One layer's expert blob in pinned host memory: [w1 (E,f,d) | w2 (E,d,f)] bf16, output-major."""
    w1 = torch.from_numpy(np.ascontiguousarray(L["w1"].transpose(0, 2, 1))).to(torch.bfloat16)
    w2 = torch.from_numpy(np.ascontiguousarray(L["w2"].transpose(0, 2, 1))).to(torch.bfloat16)
    blob = torch.empty(w1.numel() + w2.numel(), dtype=torch.bfloat16, pin_memory=True)
    blob[:w1.numel()] = w1.reshape(-1)
    blob[w1.numel():] = w2.reshape(-1)
    return blob, w1.numel() * 2


def weights_at(ptr, w2_off, routers, l):
    return M.Weights({"w1": ptr, "w2": ptr + w2_off, "w_router": routers[l]}, "output_major")


@pytest.mark.parametrize("N,K,steps", [(6, 2, 1), (5, 2, 2), (3, 4, 1)])
def test_ring_stack_matches_resident_and_oracle(N, K, steps):
    wl = WORKLOADS["ring"].scaled(T=512, d_model=256, d_ff=512, E=8)
    print(f"ring stack N={N} K={K} steps={steps} {wl}", flush=True)
    x_np, layers = make_ring_stack(wl, N)
    cfg = M.MoEConfig.from_workload(wl)
    blobs, w2_off = [], None
    for L in layers:
        b, w2_off = pack_layer_host(L, wl)
        blobs.append(b)
    layer_bytes = blobs[0].numel() * 2
    assert layer_bytes % 256 == 0
    routers = [to_dev(L["w_router"], "f32") for L in layers]
    ws = alloc_ws(cfg)
    compute = torch.cuda.current_stream()

    def run(get_ptr, after):
        x = to_dev(x_np, wl.dtype)
        ins = []
        for s in range(steps):
            for l in range(N):
                ins.append(x.clone())
                ptr = get_ptr(l)
                nxt = torch.empty_like(x)
                M.moe_layer_forward(cfg, weights_at(ptr, w2_off, routers, l), x, x, nxt, ws, compute)
                after(l)
                x = nxt
        torch.cuda.synchronize()
        return x, ins

    # all layers resident
    resident = [b.cuda() for b in blobs]
    out_res, ins_res = run(lambda l: resident[l].data_ptr(), lambda l: None)

    # streamed through the ring
    region = torch.empty(min(K, N) * layer_bytes, dtype=torch.uint8, device="cuda")
    copy_stream = torch.cuda.Stream()
    ring = M.Ring(region, region.numel(), K, blobs, layer_bytes, copy_stream=copy_stream)
    out_ring, ins_ring = run(lambda l: ring.acquire(l, compute), lambda l: ring.release(l, compute))
    st = ring.stats()
    ring.close()

    assert torch.equal(out_ring, out_res)                       # bit-identical to the resident run
    for a, b in zip(ins_ring, ins_res):
        assert torch.equal(a, b)
    Ke = min(K, N)
    want_copies = Ke + steps * N if Ke < N else Ke
    assert st["copies"] == want_copies and st["bytes_copied"] == want_copies * layer_bytes
    assert st["copy_ms"] > 0

    # teacher-forced oracle parity, layer by layer (first pass over the stack)
    for l in range(N):
        xin = to_np(ins_ring[l])
        xout = to_np(ins_ring[l + 1]) if l + 1 < len(ins_ring) else to_np(out_ring)
        ref = O.layer_forward(xin, layers[l], E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                              renormalize=wl.renormalize, act=wl.act, residual=xin)
        assert rel_fro(xout, ref["out"]) < 1e-2
        # the MoE branch alone: the sum x + branch is rounded to bf16 relative to |x| ~ 7 |branch|, so
        # the branch is only known to ~2^-9 * 7 = 1.4 % plus its own error; a wrong branch would be O(1)
        assert rel_fro(xout - xin, ref["out"] - xin) < 5e-2


def test_ring_rejects_out_of_order_on_gpu():
    blobs = [torch.zeros(1024, dtype=torch.uint8, pin_memory=True) for _ in range(3)]
    region = torch.empty(2 * 1024, dtype=torch.uint8, device="cuda")
    ring = M.Ring(region, region.numel(), 2, blobs, 1024)
    with pytest.raises(M.MoEError):
        ring.acquire(2)
    p0 = ring.acquire(0)
    ring.release(0)
    p1 = ring.acquire(1)
    assert p1 - p0 == 1024 and p0 == region.data_ptr()
    ring.release(1)
    assert ring.acquire(2) == p0                                # layer 2 refilled section 0
    ring.release(2)
    torch.cuda.synchronize()
    assert ring.stats()["copies"] == 2 + 3
    ring.close()


class _LazyExperts:
    """`weights["w1"]`-like view of one layer of a RingStackPool: `[e]` materialises that expert's matrix."""

    def __init__(self, pool, l, which, shape):
        self.pool, self.l, self.which, self.shape = pool, l, which, shape
        self._cache = {}

    def __getitem__(self, e):
        e = int(e)
        if e not in self._cache:
            self._cache = {e: self.pool.expert(self.l, e)}          # (keep one expert at a time)
        return self._cache[e][self.which]


@pytest.mark.timeout(1500)
def test_ring_stack_full_size_four_sections():
    """The ring workload as stated: 24 layers of d_model 2048, d_ff 8192, 64 experts (4 GiB of bf16 expert
    weights per layer), 4096 tokens per step, top-2, streamed from pinned host memory through K = 4 sections
    (16 GiB of HBM) by moe_ring_*.

    The GPU machine caps pinned host memory at about 64 GiB, below the stack's 96 GiB, so H = 8 distinct layer
    blobs are drawn (layers 0..7 of the seeded stack, 32 GiB pinned) and layer l streams blob l mod 8; every
    layer has its own router, so every layer routes differently.  Checked:
      (i)   the streamed stack is bit-identical, layer by layer, to the same stack reading every layer from a
            copy resident in HBM;
      (ii)  copies = K + N and bytes = (K + N) * 4 GiB for one step;
      (iii) every layer's routing equals the oracle's bit for bit on that layer's own (GPU) input, and its
            output matches the oracle on sampled tokens: the first and last row of the emptiest and of the
            fullest expert, plus random ones.
    """
    from workloads import RingStackPool
    from oracle_sampling import oracle_out_for_tokens
    wl = WORKLOADS["ring"]
    N, K, H = wl.n_layers, 4, 8
    E, d, f, T = wl.E, wl.d_model, wl.d_ff, wl.T
    print(f"full-size ring stack: N={N} K={K} distinct blobs {H} {wl}", flush=True)
    pool = RingStackPool(wl, N)
    n1 = pool.n1
    layer_bytes = 2 * n1 * 2
    assert layer_bytes == 1 << 32
    cfg = M.MoEConfig.from_workload(wl)
    # the H distinct blobs [w1 (E,f,d) | w2 (E,d,f)], output-major bf16: scaled and rounded on the device exactly
    # as the workload does on the host (one float32 multiply, round to nearest even), transposed by the library
    pool_dev = torch.from_numpy(pool.pool).cuda()
    dev_blobs, host_blobs = [], []
    for h in range(H):
        blob = torch.empty(2 * n1, dtype=torch.bfloat16, device="cuda")
        w1 = (pool_dev[h:h + n1] * float(pool.w1_scale)).to(torch.bfloat16).view(E, d, f)
        M.moe_transpose_expert_weights(w1, blob[:n1].view(E, f, d))
        w2 = (pool_dev[n1 + h:n1 + h + n1] * float(pool.w2_scale)).to(torch.bfloat16).view(E, f, d)
        M.moe_transpose_expert_weights(w2, blob[n1:].view(E, d, f))
        torch.cuda.synchronize()
        del w1, w2
        hb = torch.empty(2 * n1, dtype=torch.bfloat16, pin_memory=True)
        hb.copy_(blob)
        dev_blobs.append(blob)
        host_blobs.append(hb)
        print(f"  blob {h + 1}/{H} drawn", flush=True)
    del pool_dev
    # spot check of the device-side recipe against the host's: two experts of one blob, bit for bit
    for (h, e) in ((0, 0), (H - 1, E - 1)):
        w1_np, w2_np = pool.expert(h, e)
        got1 = dev_blobs[h][:n1].view(E, f, d)[e].float().cpu().numpy()
        got2 = dev_blobs[h][n1:].view(E, d, f)[e].float().cpu().numpy()
        assert np.array_equal(got1, w1_np.T) and np.array_equal(got2, w2_np.T)
    routers = [to_dev(r, "f32") for r in pool.routers]
    ws = alloc_ws(cfg)
    compute = torch.cuda.current_stream()
    w2_off = n1 * 2

    lay, A = M.moe_workspace_layout(cfg), wl.k * T
    tables = []   # (topk_idx, assign_to_row) of every layer of the last run, copied out of the workspace

    def run(get_ptr, after):
        x = to_dev(pool.x, wl.dtype)
        ins = []
        tables.clear()
        for l in range(N):
            ins.append(x)
            nxt = torch.empty_like(x)
            M.moe_layer_forward(cfg, weights_at(get_ptr(l), w2_off, routers, l), x, x, nxt, ws, compute)
            after(l)
            tables.append((ws[lay["topk_idx"]:lay["topk_idx"] + 4 * A].clone(), ws[lay["assign_to_row"]:lay["assign_to_row"] + 4 * A].clone()))
            x = nxt
        torch.cuda.synchronize()
        return ins + [x]

    acts_res = run(lambda l: dev_blobs[l % H].data_ptr(), lambda l: None)
    region = torch.empty(K * layer_bytes, dtype=torch.uint8, device="cuda")
    ring = M.Ring(region, region.numel(), K, [host_blobs[l % H] for l in range(N)], layer_bytes,
                  copy_stream=torch.cuda.Stream())
    acts_ring = run(lambda l: ring.acquire(l, compute), lambda l: ring.release(l, compute))
    st = ring.stats()
    ring.close()
    for l, (a, b) in enumerate(zip(acts_ring, acts_res)):
        assert torch.equal(a, b), f"activations entering layer {l} differ between the streamed and the resident stack"
    assert st["copies"] == K + N and st["bytes_copied"] == (K + N) * layer_bytes
    print(f"  streamed == resident; {st['copies']} copies, {st['bytes_copied'] / 2**30:.0f} GiB, "
          f"{st['bytes_copied'] / (st['copy_ms'] * 1e-3) / 1e9:.1f} GB/s", flush=True)
    del region, dev_blobs

    # teacher-forced oracle parity: each layer on the GPU's own input of that layer
    rng = np.random.default_rng(5)
    for l in range(N):
        xin, xout = to_np(acts_ring[l]), to_np(acts_ring[l + 1])
        p, idx, w = O.gate(xin, pool.routers[l], None, wl.k, wl.renormalize)
        counts, offsets, a2r, r2a = O.dispatch_plan(idx, E, O.capacity(T, E, wl.k, wl.capacity_factor))
        assert np.array_equal(tables[l][0].view(torch.int32).cpu().numpy().reshape(T, wl.k), idx), f"layer {l}: routing differs"
        assert np.array_equal(tables[l][1].view(torch.int32).cpu().numpy(), a2r), f"layer {l}: dispatch differs"
        lo_e, hi_e = int(np.argmin(np.where(counts > 0, counts, 1 << 30))), int(np.argmax(counts))
        rows = [offsets[lo_e], offsets[lo_e + 1] - 1, offsets[hi_e], offsets[hi_e + 1] - 1]
        toks = np.unique(np.concatenate([[int(r2a[r]) % T for r in rows], rng.integers(0, T, 1)]))
        h = l % H
        Lw = {"w_router": pool.routers[l], "w1": _LazyExperts(pool, h, 0, (E, d, f)), "w2": _LazyExperts(pool, h, 1, (E, f, d))}
        ref = oracle_out_for_tokens(O, xin, Lw, dict(topk_idx=idx, topk_w=w, assign_to_row=a2r), toks, act=wl.act, residual=xin)
        got = xout[toks]
        e_out = rel_fro(got, ref)
        e_branch = rel_fro(got - xin[toks], ref - xin[toks])
        print(f"  layer {l}: rows per expert {int(counts.min())}..{int(counts.max())}, {len(toks)} sampled tokens: "
              f"out {e_out:.2e}, MoE branch {e_branch:.2e}", flush=True)
        assert e_out < 1e-2
        # (the branch is about a seventh of the residual stream and the sum is rounded to bf16: 2^-9 * 7 = 1.4 %
        # of rounding on top of the branch's own error; a wrong expert or row would be O(1))
        assert e_branch < 5e-2
