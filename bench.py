#!/usr/bin/env python3
"""MoE-layer forward throughput on one MI355X.

A step is one pass of the whole hot path (gate -> dispatch -> expert FFN ->
combine, ``moe_layer_forward``) over one batch of seeded synthetic tokens of
the GPT-style workload: 8192 tokens, d_model 1024, d_ff 4096, 16 experts,
top-2 renormalised, capacity factor 1.25, bf16 with fp32 accumulation and an
fp32 gate.  Inputs and (output-major) weights are resident in HBM before the
timed region; weight transposition and workspace allocation are outside it.

Prints one JSON line: tokens/s, plus ``roofline`` for the dominant kernel (the
grouped bf16 MFMA GEMM, timed with HIP events recorded on the launch stream)
and ``cpu_baseline`` (the fp64 NumPy oracle timed on this host's cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

FP32_VECTOR_PEAK_TFLOPS = 157.3   # published fp32 vector rate (256 CUs, 2.4 GHz)
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the dominant kernel (grouped GEMM 1) from rocprofv3 FETCH_SIZE + WRITE_SIZE, both
# scaled by 1.000 against the weight-transpose kernel of known size (profiles/layer_forward_gpt_hbm_traffic.txt);
# a separate counter run, so it is a constant here and only quoted for the workload it was measured on.
MEASURED_TRAFFIC_BYTES = {"gpt": (151107.6 + 132461.0) * 1024}


def cpu_baseline(wl, L, budget_s=20.0):
    """The oracle as it stands, whole layer, on the host cores; repeats until ~budget_s is used."""
    import numpy as np
    from oracle import moe_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    reps, t_total = 0, 0.0
    while True:
        t0 = time.perf_counter()
        O.layer_forward(L["x"], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                        renormalize=wl.renormalize, act=wl.act)
        t_total += time.perf_counter() - t0
        reps += 1
        if t_total >= budget_s / 2 or reps >= 5:
            break
    return {"value": wl.T * reps / t_total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"whole {wl.name} layer ({wl.T} tokens), fp64 NumPy oracle, {reps} pass(es), {t_total:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="gpt")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2205_10034_amd as M
    from workloads import WORKLOADS, make_layer
    from gpu_util import alloc_ws, to_dev, upload_weights, ws_view

    wl = WORKLOADS[args.workload]
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype, nullable_bias=True)
    x = to_dev(L["x"], wl.dtype)
    out = torch.empty_like(x)
    ws = alloc_ws(cfg)
    timer = M.StageTimer()
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        M.moe_layer_forward(cfg, W, x, None, out, ws, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        M.moe_layer_forward(cfg, W, x, None, out, ws, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-kernel durations: same steps again with HIP events recorded on the launch stream around every stage
    stage = np.zeros(len(M.STAGE_NAMES))
    for _ in range(args.steps):
        M.moe_layer_forward_timed(cfg, W, x, None, out, ws, timer, stream)
        stage += np.array(timer.read())
    stage /= args.steps
    stage_ms = dict(zip(M.STAGE_NAMES, [float(v) for v in stage]))
    # the same with cold caches: 1 GiB streamed through L2 and the 256 MB last-level cache before every step
    # (consecutive steps otherwise find part of x, h and yd still cached)
    flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cold = np.zeros(len(M.STAGE_NAMES))
    n_cold = min(20, args.steps)
    for _ in range(n_cold):
        flush.fill_(1)
        M.moe_layer_forward_timed(cfg, W, x, None, out, ws, timer, stream)
        cold += np.array(timer.read())
    cold /= max(n_cold, 1)
    del flush

    lay = M.moe_workspace_layout(cfg)
    R = int(ws_view(ws, lay["expert_offsets"], cfg.E + 1, torch.int32)[-1].item())
    mats = 3 if wl.act == "swiglu" else 2
    flops1 = 2.0 * R * wl.d_model * wl.d_ff * (mats - 1)
    flops2 = 2.0 * R * wl.d_model * wl.d_ff
    dom = "gemm1" if stage_ms["gemm1"] >= stage_ms["gemm2"] else "gemm2"
    dom_flops = flops1 if dom == "gemm1" else flops2
    achieved = dom_flops / (stage_ms[dom] * 1e-3) / 1e12
    s = 2 if wl.dtype == "bf16" else 4
    hbm = {
        "gate": (wl.T * wl.d_model * s + 8 * wl.k * wl.T) / (stage_ms["gate"] * 1e-3) / 1e9,
        # bf16: routing tables only (12 B per assignment); the rows are gathered by the first GEMM
        "dispatch": (((wl.T + R) * wl.d_model * s if wl.dtype != "bf16" else 0) + 12 * wl.k * wl.T)
                    / (stage_ms["dispatch"] * 1e-3) / 1e9,
        "combine": ((R + wl.T) * wl.d_model * s + 8 * wl.k * wl.T) / (stage_ms["combine"] * 1e-3) / 1e9,
    }
    if wl.k == 1 and wl.dtype == "bf16":
        del hbm["combine"]   # the second GEMM's epilogue does the combine; the stage only fills dropped tokens' rows
    if wl.dtype == "bf16":
        roofline = {"bound": "mfma", "kernel": f"grouped_gemm_kernel ({dom})", "achieved": achieved,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name) if dom == "gemm1" else None,
                    "flops_per_launch": dom_flops, "avg_launch_ms": stage_ms[dom],
                    "note": "peak assumes 2.4 GHz; the kernel was measured at 1.7-2.0 GHz shader clock "
                            "(profiles/grouped_gemm_phase_timing_gpt_large.txt)"}
    else:   # the all-fp32 correctness configuration: plain FMA kernels, a few hundred kB of data
        roofline = {"bound": "alu", "kernel": f"ffn_f32_kernel ({dom})", "achieved": achieved,
                    "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / FP32_VECTOR_PEAK_TFLOPS,
                    "traffic": None, "flops_per_launch": dom_flops, "avg_launch_ms": stage_ms[dom],
                    "note": "launch latency sets the time at this size; the fraction is reported, not tuned for"}
    res = {
        "metric": "MoE-layer fwd tokens/s", "value": wl.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={wl.T} d_model={wl.d_model} d_ff={wl.d_ff} E={wl.E} top-{wl.k} "
                               f"CF={wl.capacity_factor} {wl.act} (seed {wl.seed})",
                   "kept_rows": R},
        "roofline": roofline,
        "stage_ms": stage_ms,
        "stage_ms_cold_caches": dict(zip(M.STAGE_NAMES, [float(v) for v in cold])),
        "ffn_tflops": (flops1 + flops2) / ((stage_ms["gemm1"] + stage_ms["gemm2"]) * 1e-3) / 1e12,
        "hbm_gbs": hbm,
        "hbm_frac": {k: v / HBM_PEAK_GBS for k, v in hbm.items()},
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, L)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
