"""Forward + backward of one MoE layer (bf16, GELU or SwiGLU experts): time per step of each pass.

    python -m paper_2205_10034_amd.backward_bench [--workload gpt|large|...] [--steps 30]

Prints one JSON line.  The backward pass needs the transposed (input-major) copies of the expert matrices; they
are made once, outside the timed region, like the forward pass's output-major ones.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--bias", action="store_true", help="GELU experts with biases (and their gradients)")
    ap.add_argument("--bf16-grads", action="store_true", help="weight gradients rounded once to bfloat16 (half the bytes written)")
    args = ap.parse_args()
    import torch
    import paper_2205_10034_amd as M
    from workloads import WORKLOADS

    wl = WORKLOADS[args.workload]
    if wl.dtype != "bf16":
        sys.exit("backward_bench: bf16 only")
    sw = wl.act == "swiglu"
    torch.manual_seed(0)
    dt = torch.bfloat16
    T, d, f, E = wl.T, wl.d_model, wl.d_ff, wl.E
    x = torch.randn(T, d, device="cuda").to(dt)
    g = torch.randn(T, d, device="cuda").to(dt)
    def mat(n, k): return (torch.randn(E, n, k, device="cuda") * k ** -0.5).to(dt)
    router = (torch.randn(d, E, device="cuda") * d ** -0.5).contiguous()
    w2_im = torch.empty(E, f, d, dtype=dt, device="cuda")
    if sw:
        wg, wu, wd = mat(f, d), mat(f, d), mat(d, f)   # output-major
        w1_im = torch.cat([wg.transpose(1, 2), wu.transpose(1, 2)], dim=2).contiguous()     # [E, d, 2f]: gate | up
        M.moe_transpose_expert_weights(wd, w2_im)
        W = M.Weights({"w_gate_proj": wg, "w_up": wu, "w_down": wd, "w_router": router})
    else:
        w1, w2 = mat(f, d), mat(d, f)                  # output-major
        w1_im = torch.empty(E, d, f, dtype=dt, device="cuda")
        M.moe_transpose_expert_weights(w1, w1_im)
        M.moe_transpose_expert_weights(w2, w2_im)
        t = {"w1": w1, "w2": w2, "w_router": router}
        if args.bias:
            t["b1"] = (torch.randn(E, f, device="cuda") * 0.1).to(dt)
            t["b2"] = (torch.randn(E, d, device="cuda") * 0.1).to(dt)
        W = M.Weights(t)
    cfg = M.MoEConfig.from_workload(wl)
    ws_f = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(M.moe_layer_backward_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    out, d_x = torch.empty_like(x), torch.empty_like(x)
    f32 = dict(dtype=torch.float32, device="cuda")
    gw = dict(dtype=torch.bfloat16 if args.bf16_grads else torch.float32, device="cuda")
    d_wr, d_w1, d_w2 = torch.empty(d, E, **f32), torch.empty(E, (2 if sw else 1) * f, d, **gw), torch.empty(E, d, f, **gw)

    def fwd():
        M.moe_layer_forward(cfg, W, x, x, out, ws_f)

    with_b = args.bias and not sw
    d_b1 = torch.empty(E, f, **f32) if with_b else None
    d_b2 = torch.empty(E, d, **f32) if with_b else None

    def bwd():
        M.moe_layer_backward(cfg, W, w1_im, w2_im, x, g, g, ws_f, d_x, d_wr, None, d_w1, d_b1, d_w2, d_b2, ws_b)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()
    t_f = timed(fwd, args.steps)
    t_b = timed(bwd, args.steps)
    t_fb = timed(lambda: (fwd(), bwd()), args.steps)
    lay = M.moe_workspace_layout(cfg)
    R = int(ws_f[lay["expert_offsets"]:lay["expert_offsets"] + 4 * (E + 1)].view(torch.int32)[-1].item())
    gemm = 2.0 * R * d * f
    res = {
        "workload": f"{wl.name}: T={T} d_model={d} d_ff={f} E={E} top-{wl.k} CF={wl.capacity_factor} {wl.act}{' with biases' if with_b else ''}{', bf16 weight gradients' if args.bf16_grads else ''}, kept rows {R}",
        "forward_ms": t_f, "backward_ms": t_b, "forward_backward_ms": t_fb,
        "tokens_per_s_forward_backward": T / (t_fb * 1e-3),
        # products of 2 R d_model d_ff flops.  GELU: two forward; backward two input gradients, two weight gradients,
        # one recomputation.  SwiGLU: three forward; backward three input gradients (d_h, and d_xd over gate and
        # up), three weight gradients, two recomputations
        "backward_tflops": (8 if sw else 5) * gemm / (t_b * 1e-3) / 1e12,
        "forward_backward_tflops": (11 if sw else 7) * gemm / (t_fb * 1e-3) / 1e12,
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
