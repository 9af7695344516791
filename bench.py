#!/usr/bin/env python3
"""MoE-layer forward throughput on one MI355X.

A step is one pass of the whole hot path (gate -> dispatch -> expert FFN ->
combine, ``moe_layer_forward``) over one batch of seeded synthetic tokens.  The
default workload is the largest configuration that fits one GPU, the
large-expert layer: 32768 tokens, d_model 4096, d_ff 14336, SwiGLU experts,
8 experts, top-2 renormalised, capacity factor 1.0, bf16 with fp32
accumulation and an fp32 gate (``--workload gpt|skew|skew40|ring|tiny`` times
the others).  Inputs and (output-major) weights are resident in HBM before the
timed region; weight transposition and workspace allocation are outside it.

Protocol: an untimed pre-warm brings clocks and caches to their steady state
(``--prewarm-s`` seconds of steps), then ``--warmup`` untimed steps, then
exactly ``--steps`` steps between two device synchronisations.

Prints one JSON line: tokens/s, plus ``roofline`` for the dominant kernel (the
grouped bf16 MFMA GEMM, timed with HIP events recorded on the launch stream;
its HBM traffic is read from the rocprofv3 counter summary committed under
``profiles/`` for the same workload) and ``cpu_baseline`` (the fp64 NumPy
oracle timed on this host's cores over a bounded sample of the same workload).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP32_VECTOR_PEAK_TFLOPS = 157.3   # published fp32 vector rate (256 CUs, 2.4 GHz)
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# the oracle's cost grows with T * d_model * d_ff; the CPU leg takes as many leading tokens as keep it near this
CPU_SAMPLE_FLOPS = 8e12


def measured_traffic(workload, stage):
    """HBM bytes per launch of `stage`'s kernel from the committed counter summary of this workload:
    a line `traffic_bytes_per_launch <stage> <bytes>` in profiles/layer_forward_<workload>_hbm_traffic.txt
    (FETCH_SIZE + WRITE_SIZE of a rocprofv3 --pmc run, scaled as the file says).  None if there is none."""
    path = os.path.join(ROOT, "profiles", f"layer_forward_{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                m = re.match(r"\s*traffic_bytes_per_launch\s+(\w+)\s+([0-9.eE+]+)", line)
                if m and m.group(1) == stage:
                    return float(m.group(2))
    except OSError:
        pass
    return None


def cpu_baseline(wl, L):
    """The oracle as it stands (whole layer: gate, dispatch, FFN, combine) on the host cores, over the first
    tokens of the workload: as many as make about CPU_SAMPLE_FLOPS of expert products."""
    from oracle import moe_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    mats = 3 if wl.act == "swiglu" else 2
    per_token = 2.0 * wl.k * mats * wl.d_model * wl.d_ff
    Ts = int(min(wl.T, max(256, CPU_SAMPLE_FLOPS // per_token)))
    t0 = time.perf_counter()
    O.layer_forward(L["x"][:Ts], L, E=wl.E, k=wl.k, capacity_factor=wl.capacity_factor,
                    renormalize=wl.renormalize, act=wl.act)
    dt = time.perf_counter() - t0
    what = "whole layer" if Ts == wl.T else f"first {Ts} of {wl.T} tokens (same weights, whole-layer oracle on that batch)"
    return {"value": Ts / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{wl.name}: {what}, fp64 NumPy oracle, one pass, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--prewarm-s", type=float, default=2.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pack-router", action="store_true", help="do not give the layer a pre-split router (moe_pack_router)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="moe_set_tuning before the run: gemm_tile_rows=256|320, few_token_kernels=0|1, gate_tokens=32|64|128, gemm_mfma=16|32")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2205_10034_amd as M
    from paper_2205_10034_amd.torch_util import alloc_ws, to_dev, upload_weights, ws_view
    from workloads import WORKLOADS, make_layer

    tuned = {}
    for kv in args.tune:
        key, val = kv.split("=")
        M.moe_set_tuning(getattr(M, "MOE_TUNE_" + key.upper()), int(val))
        tuned[key] = int(val)
    wl = WORKLOADS[args.workload]
    big = wl.T * wl.d_model * wl.d_ff > 1e12
    steps = args.steps if args.steps is not None else (40 if big else 200)
    warmup = args.warmup if args.warmup is not None else (5 if big else 20)
    L = make_layer(wl)
    cfg = M.MoEConfig.from_workload(wl)
    W = upload_weights(L, wl.dtype, nullable_bias=True, pack_router=not args.no_pack_router)
    x = to_dev(L["x"], wl.dtype)
    out = torch.empty_like(x)
    ws = alloc_ws(cfg)
    timer = M.StageTimer()
    stream = torch.cuda.current_stream()

    # untimed pre-warm to the steady state (clocks under load, caches, first-touch of every page)
    t0 = time.perf_counter()
    n_pre = 0
    while time.perf_counter() - t0 < args.prewarm_s or n_pre < 3:
        M.moe_layer_forward(cfg, W, x, None, out, ws, stream)
        n_pre += 1
        if n_pre % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()

    for _ in range(warmup):
        M.moe_layer_forward(cfg, W, x, None, out, ws, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        M.moe_layer_forward(cfg, W, x, None, out, ws, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3

    # per-kernel durations: same steps again with HIP events recorded on the launch stream around every stage
    stage = np.zeros(len(M.STAGE_NAMES))
    for _ in range(steps):
        M.moe_layer_forward_timed(cfg, W, x, None, out, ws, timer, stream)
        stage += np.array(timer.read())
    stage /= steps
    stage_ms = dict(zip(M.STAGE_NAMES, [float(v) for v in stage]))
    # the same with cold caches: 1 GiB streamed through L2 and the 256 MB last-level cache before every step
    # (consecutive steps otherwise find part of x, h and yd still cached)
    flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cold = np.zeros(len(M.STAGE_NAMES))
    n_cold = min(10 if big else 20, steps)
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
    # algorithmic bytes of the HBM-bound stages (the dispatch stage of the bf16 path only builds routing tables
    # - the rows are gathered by the first GEMM - so it is latency-bound and has no bandwidth figure)
    hbm = {"gate": (wl.T * wl.d_model * s + 8 * wl.k * wl.T) / (stage_ms["gate"] * 1e-3) / 1e9}
    if wl.dtype != "bf16":
        hbm["dispatch"] = ((wl.T + R) * wl.d_model * s + 12 * wl.k * wl.T) / (stage_ms["dispatch"] * 1e-3) / 1e9
    if not (wl.k == 1 and wl.dtype == "bf16"):  # (k = 1: the second GEMM's epilogue does the combine)
        hbm["combine"] = ((R + wl.T) * wl.d_model * s + 8 * wl.k * wl.T) / (stage_ms["combine"] * 1e-3) / 1e9
    other = "gemm2" if dom == "gemm1" else "gemm1"
    other_flops = flops2 if dom == "gemm1" else flops1
    if wl.dtype == "bf16":
        # unique bytes of the two GEMMs (every weight matrix, the kept rows in and out, once): with few rows per expert
        # the dominant GEMM streams weights and the HBM roofline is the one that binds
        wbytes = wl.E * wl.d_model * wl.d_ff * s
        gemm_bytes = {"gemm1": R * wl.d_model * s + (mats - 1) * wbytes + R * wl.d_ff * s,
                      "gemm2": R * wl.d_ff * s + wbytes + R * wl.d_model * s}
        hbm_frac_dom = gemm_bytes[dom] / (stage_ms[dom] * 1e-3) / 1e9 / HBM_PEAK_GBS
        mfma_frac_dom = achieved / MFMA_BF16_PEAK_TFLOPS
        if hbm_frac_dom > mfma_frac_dom:
            roofline = {"bound": "hbm", "kernel": f"grouped_gemm_kernel ({dom})",
                        "achieved": hbm_frac_dom * HBM_PEAK_GBS, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac_dom,
                        "traffic": measured_traffic(wl.name, dom), "bytes_per_launch": gemm_bytes[dom],
                        "avg_launch_ms": stage_ms[dom], "mfma_frac": mfma_frac_dom,
                        "other_gemm": {"kernel": f"grouped_gemm_kernel ({other})", "bytes_per_launch": gemm_bytes[other],
                                       "avg_launch_ms": stage_ms[other],
                                       "frac": gemm_bytes[other] / (stage_ms[other] * 1e-3) / 1e9 / HBM_PEAK_GBS}}
        else:
            roofline = {"bound": "mfma", "kernel": f"grouped_gemm_kernel ({dom})", "achieved": achieved,
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": mfma_frac_dom,
                        "traffic": measured_traffic(wl.name, dom),
                        "flops_per_launch": dom_flops, "avg_launch_ms": stage_ms[dom],
                        "other_gemm": {"kernel": f"grouped_gemm_kernel ({other})", "flops_per_launch": other_flops,
                                       "avg_launch_ms": stage_ms[other],
                                       "frac": other_flops / (stage_ms[other] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}}
    else:   # the all-fp32 correctness configuration: plain FMA kernels, a few hundred kB of data
        roofline = {"bound": "alu", "kernel": f"ffn_f32_kernel ({dom})", "achieved": achieved,
                    "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / FP32_VECTOR_PEAK_TFLOPS,
                    "traffic": None, "flops_per_launch": dom_flops, "avg_launch_ms": stage_ms[dom],
                    "note": "launch latency sets the time at this size; the fraction is reported, not tuned for"}
    res = {
        "metric": "MoE-layer fwd tokens/s", "value": wl.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={wl.T} d_model={wl.d_model} d_ff={wl.d_ff} E={wl.E} top-{wl.k} "
                               f"CF={wl.capacity_factor} {wl.act} (seed {wl.seed})",
                   "kept_rows": R, "prewarm_steps": n_pre, **({"tuning": tuned} if tuned else {})},
        "roofline": roofline,
        "stage_ms": stage_ms,
        "stage_ms_cold_caches": dict(zip(M.STAGE_NAMES, [float(v) for v in cold])),
        "ffn_tflops": (flops1 + flops2) / ((stage_ms["gemm1"] + stage_ms["gemm2"]) * 1e-3) / 1e12,
        "hbm_gbs": hbm,
        "hbm_frac": {k: v / HBM_PEAK_GBS for k, v in hbm.items()},
    }
    if not args.no_cpu_baseline:
        del W, x, out, ws
        res["cpu_baseline"] = cpu_baseline(wl, L)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
