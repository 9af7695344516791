"""Expert-granular offloading benchmark: the ring workload's 24-layer stack (d_model 2048, d_ff 8192, 64
experts, top-2, bf16: 64 MiB per expert, 96 GiB in all) run with FEW tokens per step, where streaming whole
layers through the ring of sections moves 96 GiB per step whatever the batch.  Here every expert stays in
pinned host memory and enters a 16 GiB pool of HBM slots only when the step's routing activates it
(moe_layer_route -> moe_expert_pool_prepare -> moe_layer_experts per layer); which experts keep their
slots is decided by the frequency-based policy of the paper's sparse-parameter scheduling.

Host memory holds --host-layers distinct layers of parameters (default 4 = 16 GiB pinned); layer l reads
the blobs of layer l mod that number, but is cached under its own items, so hit rates and traffic are
those of 24 different layers.

    python -m paper_2205_10034_amd.pool_bench [--tokens 1,8,64] [--steps 20] [--skew 0,1]
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
    ap.add_argument("--host-layers", type=int, default=4)
    ap.add_argument("--pool-gib", type=float, default=16.0)
    ap.add_argument("--tokens", default="1,8,64")
    ap.add_argument("--skew", default="0,1", help="0: routers as initialised; 1: plus a log-Zipf(1.2) bias per expert")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--threshold", type=float, default=2.0)
    ap.add_argument("--beta", type=float, default=0.9)
    ap.add_argument("--decay-steps", type=int, default=256)
    ap.add_argument("--prefetch", action="store_true",
                    help="while a layer's experts run, route the next layer on this layer's input (second stream) and copy "
                         "the guessed experts that are not resident ahead of time")
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2205_10034_amd as M
    from workloads import WORKLOADS, zipf_masses

    base_wl = WORKLOADS["ring"]
    N, E, d, f = args.layers, base_wl.E, base_wl.d_model, base_wl.d_ff
    n1 = f * d
    blob_bytes = 2 * n1 * 2
    slot_bytes = blob_bytes
    slots = int(args.pool_gib * 2 ** 30) // slot_bytes
    print(f"pool bench: {N} layers x {E} experts x {blob_bytes / 2**20:.0f} MiB; pool {slots} slots = "
          f"{slots * slot_bytes / 2**30:.1f} GiB of HBM; {args.host_layers} distinct layers in pinned memory", flush=True)
    torch.manual_seed(0)
    t0 = time.time()
    host = []
    for hl in range(args.host_layers):
        for e in range(E):
            blob = torch.empty(2 * n1, dtype=torch.bfloat16, pin_memory=True)
            g = torch.randn(n1, device="cuda", dtype=torch.float32)
            blob[:n1].copy_((g * d ** -0.5).to(torch.bfloat16))
            g.normal_()
            blob[n1:].copy_((g * (f ** -0.5 * base_wl.w2_std_scale)).to(torch.bfloat16))
            host.append(blob)
        print(f"  filled {hl + 1}/{args.host_layers} host layers ({time.time() - t0:.0f} s)", flush=True)
    del g
    blobs = [host[(l % args.host_layers) * E + e] for l in range(N) for e in range(E)]
    routers = [(torch.randn(d, E, device="cuda") * d ** -0.5).contiguous() for _ in range(N)]
    zipf = torch.tensor(np.log(zipf_masses(E, 1.2)), dtype=torch.float32, device="cuda")
    perms = [torch.randperm(E, device="cuda") for _ in range(N)]       # each layer has its own popular experts
    dev_pool = torch.empty(slots * slot_bytes, dtype=torch.uint8, device="cuda")
    offs = torch.zeros(E, dtype=torch.int64, device="cuda")
    compute = torch.cuda.current_stream()

    for skew in [int(v) for v in args.skew.split(",")]:
        for T in [int(v) for v in args.tokens.split(",")]:
            wl = base_wl.scaled(T=T)
            cfg = M.MoEConfig.from_workload(wl)
            ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
            ws_guess = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
            lay = M.moe_workspace_layout(cfg)
            counts_dev = ws[lay["expert_counts"]:lay["expert_counts"] + 4 * E].view(torch.int32)
            guess_dev = ws_guess[lay["expert_counts"]:lay["expert_counts"] + 4 * E].view(torch.int32)
            side = torch.cuda.Stream()
            ahead = [0]
            pool = M.ExpertPool(dev_pool, slot_bytes, blobs, N, E, blob_bytes, args.threshold, args.beta, args.decay_steps)
            Ws = []
            for l in range(N):
                t = {"w_router": routers[l], "expert_elem_offset": offs, "w1": dev_pool.data_ptr(),
                     "w2": dev_pool.data_ptr() + 2 * n1}
                if skew:
                    t["b_router"] = zipf[perms[l]].contiguous()
                Ws.append(M.Weights(t))
            gen = torch.Generator(device="cuda").manual_seed(1)

            def step():
                x = torch.randn(T, d, device="cuda", generator=gen).to(torch.bfloat16)
                nxt = torch.empty_like(x)
                for l in range(N):
                    M.moe_layer_route(cfg, Ws[l], x, ws, compute)
                    pool.prepare(l, counts_dev, 2, offs, compute)
                    M.moe_layer_experts(cfg, Ws[l], x, x, nxt, ws, compute)
                    if args.prefetch and l + 1 < N:
                        # (x is complete: prepare() waited for the compute stream after this layer's routing)
                        M.moe_layer_route(cfg, Ws[l + 1], x, ws_guess, side)
                        ahead[0] += pool.prefetch(l + 1, guess_dev, side)
                    x, nxt = nxt, x
                return x

            for _ in range(args.warmup):
                step()
            torch.cuda.synchronize()
            s0 = pool.stats()
            ahead[0] = 0
            t1 = time.perf_counter()
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t1
            s1 = pool.stats()
            pool.close()
            # (a copy ahead of time is a miss of the policy; the request that follows it is a hit)
            req = (s1["hits"] - s0["hits"]) + (s1["misses"] - s0["misses"]) - ahead[0]
            copied = s1["bytes_copied"] - s0["bytes_copied"]
            res = {
                "workload": f"expert pool: {N} layers, T={T} d_model={d} d_ff={f} E={E} top-{wl.k}, "
                            f"{slots} slots, router {'log-Zipf(1.2) bias' if skew else 'unbiased'}{', next layer guessed and copied ahead' if args.prefetch else ''}",
                "step_ms": dt / args.steps * 1e3, "tokens_per_s": T * args.steps / dt,
                "experts_requested_per_step": req / args.steps,
                "hit_rate": (s1["hits"] - s0["hits"]) / max(req, 1),
                "gib_copied_per_step": copied / args.steps / 2 ** 30,
                **({"copied_ahead_per_step": ahead[0] / args.steps} if args.prefetch else {}),
                "h2d_gbs_over_whole_step": copied / dt / 1e9,
                "whole_layer_streaming_gib_per_step": N * E * blob_bytes / 2 ** 30,
            }
            print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
