"""Latency of one MoE layer at decode-sized batches with every expert resident in HBM: the ring workload's layer
(d_model 2048, d_ff 8192, 64 experts, top-2, bf16: 64 MiB per expert) run with 1 ... 256 tokens per step.
With so few tokens the layer's time is the time to stream the activated experts' weights once; up to 16
assignments per step the expert products run on the matrix-vector kernels instead of MFMA tiles
(``--general-kernels`` switches them off through moe_set_tuning, for comparison).

    python -m paper_2205_10034_amd.decode_bench [--tokens 1,2,4,8,16,32,64,128,256] [--steps 50] [--general-kernels]

One JSON line per batch size.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", default="1,2,4,8,16,32,64,128,256")
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--general-kernels", action="store_true")
    args = ap.parse_args()
    import torch
    import paper_2205_10034_amd as M
    if args.general_kernels:
        M.moe_set_tuning(M.MOE_TUNE_FEW_TOKEN_KERNELS, 0)
    from workloads import WORKLOADS

    base = WORKLOADS["ring"]
    E, d, f = base.E, base.d_model, base.d_ff
    torch.manual_seed(0)
    dt = torch.bfloat16
    w1 = (torch.randn(E, f, d, device="cuda") * d ** -0.5).to(dt)
    w2 = (torch.randn(E, d, f, device="cuda") * f ** -0.5).to(dt)
    W = M.Weights({"w1": w1, "w2": w2, "w_router": (torch.randn(d, E, device="cuda") * d ** -0.5).contiguous()})
    for T in [int(v) for v in args.tokens.split(",")]:
        wl = base.scaled(T=T)
        cfg = M.MoEConfig.from_workload(wl)
        ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        x = torch.randn(T, d, device="cuda").to(dt)
        out = torch.empty_like(x)
        for _ in range(args.warmup):
            M.moe_layer_forward(cfg, W, x, x, out, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            M.moe_layer_forward(cfg, W, x, x, out, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        lay = M.moe_workspace_layout(cfg)
        counts = ws[lay["expert_counts"]:lay["expert_counts"] + 4 * E].view(torch.int32)
        active = int((counts > 0).sum().item())
        wbytes = active * 2 * d * f * 2
        print(json.dumps({
            "workload": f"ring layer, resident: T={T} d_model={d} d_ff={f} E={E} top-{wl.k}",
            "layer_us": ms * 1e3, "tokens_per_s": T / (ms * 1e-3), "experts_activated": active,
            "weights_streamed_mib": wbytes / 2 ** 20, "weights_tb_per_s": wbytes / (ms * 1e-3) / 1e12,
            "matrix_vector_kernels": wl.k * T <= 16 and not args.general_kernels,
        }), flush=True)


if __name__ == "__main__":
    main()
