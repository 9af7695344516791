"""Ring memory offloading benchmark (Section 3.3.2): a stack of MoE layers whose expert weights sit in
pinned host memory and stream through a ring of HBM sections while the layers compute.

Default = the ring workload: 24 layers, d_model 2048, d_ff 8192, 64 experts, top-2, bf16 (4 GiB of
expert weights per layer, ~103 GB in pinned host memory), 4096 tokens per step, 4 sections = 16 GiB of
HBM.  The step is bound by the host-to-device link; the figures of merit are the achieved H2D rate and
how close the step time gets to max(sum of copies, sum of compute).

    python -m paper_2205_10034_amd.ring_bench [--layers 24] [--sections 4] [--steps 2]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=24)
    ap.add_argument("--sections", type=int, default=4)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--tokens", type=int, default=4096)
    ap.add_argument("--distinct", type=int, default=8, help="distinct layer blobs held in pinned host memory")
    args = ap.parse_args()

    import torch
    import paper_2205_10034_amd as M
    from workloads import WORKLOADS

    wl = WORKLOADS["ring"].scaled(T=args.tokens)
    N, K = args.layers, args.sections
    E, d, f = wl.E, wl.d_model, wl.d_ff
    cfg = M.MoEConfig.from_workload(wl)
    n1 = E * f * d
    layer_bytes = 2 * n1 * 2
    print(f"ring bench: {N} layers x {layer_bytes / 2**30:.2f} GiB in pinned host memory, "
          f"{K} sections = {K * layer_bytes / 2**30:.1f} GiB of HBM", flush=True)

    # The seeded ring stack of workloads/ (one normal pool, layer l = the window at element l): the box caps pinned
    # host memory near 64 GiB, below the stack's 96 GiB, so `--distinct` blobs are drawn (layers 0 .. distinct-1
    # of the stack) and layer l streams blob l mod distinct; every layer has its own router.
    from workloads import RingStackPool
    t0 = time.time()
    pool = RingStackPool(wl, N)
    H = min(args.distinct, N)
    pool_dev = torch.from_numpy(pool.pool).cuda()
    distinct = []
    for h in range(H):
        dev = torch.empty(2 * n1, dtype=torch.bfloat16, device="cuda")
        w1 = (pool_dev[h:h + n1] * float(pool.w1_scale)).to(torch.bfloat16).view(E, d, f)
        M.moe_transpose_expert_weights(w1, dev[:n1].view(E, f, d))
        w2 = (pool_dev[n1 + h:n1 + h + n1] * float(pool.w2_scale)).to(torch.bfloat16).view(E, f, d)
        M.moe_transpose_expert_weights(w2, dev[n1:].view(E, d, f))
        torch.cuda.synchronize()
        del w1, w2
        blob = torch.empty(2 * n1, dtype=torch.bfloat16, pin_memory=True)
        blob.copy_(dev)
        distinct.append(blob)
        del dev
        print(f"  drew {h + 1}/{H} distinct layer blobs ({time.time() - t0:.0f} s)", flush=True)
    del pool_dev
    blobs = [distinct[l % H] for l in range(N)]
    routers = [torch.from_numpy(r).cuda() for r in pool.routers]
    torch.cuda.synchronize()

    x0 = torch.from_numpy(pool.x).cuda().to(torch.bfloat16)
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    region = torch.empty(min(K, N) * layer_bytes, dtype=torch.uint8, device="cuda")
    compute = torch.cuda.current_stream()
    copy_stream = torch.cuda.Stream()
    w2_off = n1 * 2

    def weights(ptr, l):
        return M.Weights({"w1": ptr, "w2": ptr + w2_off, "w_router": routers[l]}, "output_major")

    def stack(get_ptr, after):
        x = x0.clone()
        nxt = torch.empty_like(x)
        for l in range(N):
            M.moe_layer_forward(cfg, weights(get_ptr(l), l), x, x, nxt, ws, compute)
            after(l)
            x, nxt = nxt, x
        return x

    # compute alone: every layer reads section 0 (its contents do not matter for the timing)
    region[:layer_bytes].view(torch.bfloat16).copy_(blobs[0], non_blocking=False)
    for _ in range(2):
        stack(lambda l: region.data_ptr(), lambda l: None)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    stack(lambda l: region.data_ptr(), lambda l: None)
    e1.record()
    torch.cuda.synchronize()
    compute_ms = e0.elapsed_time(e1)

    ring = M.Ring(region, region.numel(), K, blobs, layer_bytes, copy_stream=copy_stream)
    stack(lambda l: ring.acquire(l, compute), lambda l: ring.release(l, compute))   # warm-up step
    torch.cuda.synchronize()
    s0 = ring.stats()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        stack(lambda l: ring.acquire(l, compute), lambda l: ring.release(l, compute))
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t1) / args.steps * 1e3
    s1 = ring.stats()
    ring.close()
    copied = s1["bytes_copied"] - s0["bytes_copied"]
    copy_ms = (s1["copy_ms"] - s0["copy_ms"]) / args.steps
    res = {
        "workload": f"ring stack: {N} layers, T={wl.T} d_model={d} d_ff={f} E={E} top-{wl.k}, {K} sections",
        "step_ms": step_ms, "tokens_per_s": wl.T / (step_ms * 1e-3),
        "bytes_copied_per_step": copied / args.steps, "sum_copy_ms_per_step": copy_ms,
        "h2d_gbs": copied / args.steps / (copy_ms * 1e-3) / 1e9 if copy_ms > 0 else None,
        "compute_only_ms_per_step": compute_ms,
        "overlap_efficiency": max(copy_ms, compute_ms) / step_ms,
        "hbm_weight_budget_gib": K * layer_bytes / 2 ** 30, "host_weight_gib": N * layer_bytes / 2 ** 30,
        "distinct_layer_blobs_in_pinned_memory": H, "data": "seeded ring stack of workloads/ (synthetic)",
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
