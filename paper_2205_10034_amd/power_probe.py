"""Board power while the layer runs, next to the vendor's dense product on one expert's shapes.

``python -m paper_2205_10034_amd.power_probe [--workload large]`` samples the GPU's power sensor (hwmon, read-only)
every 20 ms while it repeats (a) ``moe_layer_forward`` of the workload, (b) ``torch.matmul`` (the vendor's bf16
product) of one expert's first-GEMM shapes on random operands and (c) the same on all-zero operands and (d) loops of nothing but MFMAs of either shape on random and on zero operands held in
registers (from the phase-timing build of the library, if it is built), and prints the mean power, the board's power
cap and the rate of each.  It answers one question: whether the grouped GEMM's rate
is set by the power cap rather than by the matrix pipes' issue rate.  Diagnostics only.
"""
from __future__ import annotations

import argparse
import ctypes
import glob
import os
import sys
import threading
import time

import torch

import paper_2205_10034_amd as M
from paper_2205_10034_amd.build import PROF_LIB
from workloads import WORKLOADS


def _sensor():
    for h in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
        for f in ("power1_average", "power1_input"):
            p = os.path.join(h, f)
            if os.path.exists(p):
                cap = os.path.join(h, "power1_cap")
                return p, cap if os.path.exists(cap) else None
    return None, None


def _read(path):
    try:
        with open(path) as f:
            return int(f.read().strip()) / 1e6
    except (OSError, ValueError):
        return float("nan")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="large")
    ap.add_argument("--seconds", type=float, default=5.0)
    a = ap.parse_args()
    sensor, cap = _sensor()
    if sensor is None:
        print("no power sensor under /sys/class/drm/card*/device/hwmon", file=sys.stderr)
        return 2
    samples, stop = [], threading.Event()

    def sampler():
        while not stop.is_set():
            samples.append((time.time(), _read(sensor)))
            time.sleep(0.02)

    threading.Thread(target=sampler, daemon=True).start()
    time.sleep(0.5)
    print(f"power cap {_read(cap):.0f} W, idle {samples[-1][1]:.0f} W" if cap else f"idle {samples[-1][1]:.0f} W", flush=True)

    def measure(label, fn, flops):
        fn()
        torch.cuda.synchronize()
        t0, n = time.time(), 0
        while time.time() - t0 < a.seconds:
            fn()
            n += 1
            if n % 4 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        dt = (time.time() - t0) / n
        pw = [p for t, p in samples if t > t0 + 1.0 and p == p]
        print(f"{label}: {dt * 1e3:8.3f} ms per call, {flops / dt / 1e12:7.0f} TFLOP/s, power mean {sum(pw) / max(len(pw), 1):5.0f} W "
              f"max {max(pw or [0]):5.0f} W ({len(pw)} samples)", flush=True)

    wl = WORKLOADS[a.workload]
    d, f, E = wl.d_model, wl.d_ff, wl.E
    torch.manual_seed(0)
    bf = torch.bfloat16
    x = torch.randn(wl.T, d, device="cuda").to(bf)
    t = {"w_router": (torch.randn(d, E, device="cuda") * d ** -0.5).contiguous()}

    def mat(n, k):
        return (torch.randn(E, n, k, device="cuda") * k ** -0.5).to(bf)

    if wl.act == "swiglu":
        t["w_gate_proj"], t["w_up"], t["w_down"] = mat(f, d), mat(f, d), mat(d, f)
    else:
        t["w1"], t["w2"] = mat(f, d), mat(d, f)
    W = M.Weights(t, "output_major")
    cfg = M.MoEConfig.from_workload(wl)
    ws = torch.empty(M.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(x)
    M.moe_layer_forward(cfg, W, x, None, out, ws)
    lay = M.moe_workspace_layout(cfg)
    R = int(ws[lay["expert_offsets"] + 4 * E:lay["expert_offsets"] + 4 * E + 4].view(torch.int32).item())
    mats = 3 if wl.act == "swiglu" else 2
    measure(f"moe_layer_forward ({a.workload}, {R} kept rows)", lambda: M.moe_layer_forward(cfg, W, x, None, out, ws), 2.0 * R * d * f * mats)
    rows, n1 = max(256, R // E), (2 if wl.act == "swiglu" else 1) * f
    p, q = torch.randn(rows, d, device="cuda").to(bf), torch.randn(n1, d, device="cuda").to(bf)
    r = torch.empty(rows, n1, device="cuda", dtype=bf)
    measure(f"vendor product {rows} x {d} x {n1}, random operands", lambda: torch.matmul(p, q.t(), out=r), 2.0 * rows * d * n1)
    p.zero_()
    q.zero_()
    measure(f"vendor product {rows} x {d} x {n1}, zero operands  ", lambda: torch.matmul(p, q.t(), out=r), 2.0 * rows * d * n1)
    if os.path.exists(PROF_LIB):
        L = ctypes.CDLL(PROF_LIB)
        L.moe_mfma_operand_loop.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double)]
        for kind, name in ((0, "32x32x16"), (1, "16x16x32")):
            for zero in (0, 1):
                rate, t0, n, tf = 0.0, time.time(), 0, ctypes.c_double()
                while time.time() - t0 < a.seconds:
                    if L.moe_mfma_operand_loop(kind, zero, 20000, ctypes.byref(tf)) != 0:
                        print("moe_mfma_operand_loop failed", file=sys.stderr)
                        return 1
                    rate += tf.value
                    n += 1
                pw = [p for t, p in samples if t > t0 + 1.5 and p == p]
                print(f"MFMA-only loop, v_mfma_f32_{name}_bf16, {'zero  ' if zero else 'random'} operands: {rate / n:7.0f} TFLOP/s, "
                      f"power mean {sum(pw) / max(len(pw), 1):5.0f} W", flush=True)
    stop.set()
    return 0


if __name__ == "__main__":
    sys.exit(main())
