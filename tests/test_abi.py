"""Host-only checks of the C ABI: the library loads, exports every declared symbol, validates
arguments before touching the GPU, and its integer host logic matches the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2205_10034_amd as M
from oracle import moe_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moesys.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)) - {"moe_ring_backend"})


def test_library_exports_every_declared_symbol():
    L = M.lib()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), f"{n} declared in moesys.h but not exported"


def test_diagnostics_library_exports_what_the_measurement_tools_call():
    """The phase-timing build carries the whole library plus the entry points of gemm_profile, hw_peaks and
    power_probe (loaded here without calling anything: those need a GPU)."""
    import ctypes
    import os
    from paper_2205_10034_amd.build import PROF_LIB
    if not os.path.exists(PROF_LIB):
        pytest.skip("diagnostics library not built")
    P = ctypes.CDLL(PROF_LIB)
    for n in declared_symbols() + ["moe_hw_peaks", "moe_mfma_operand_loop", "moe_gemm_profile_set"]:
        assert hasattr(P, n), n


def test_status_strings_and_version():
    L = M.lib()
    assert L.moe_version() >= 100
    seen = {L.moe_status_string(i) for i in range(6)}
    assert len(seen) == 6 and L.moe_status_string(99) == b"unknown status"


@pytest.mark.parametrize("T,E,k,cf", [(256, 4, 1, 1.25), (8192, 16, 2, 1.25), (32768, 8, 2, 1.0), (10, 1, 1, 1.1),
                                      (7, 3, 2, 1.5), (100, 7, 2, 0.3), (1, 64, 1, 0.01), (16384, 8, 1, 0.0),
                                      (16384, 8, 1, -2.0), (12345, 17, 3, 0.777), (0, 4, 2, 1.0),
                                      (5, 4, 2, 1e30), (1000, 4, 1, 1e-30)])
def test_capacity_matches_oracle(T, E, k, cf):
    cfg = M.MoEConfig(T=T, d_model=64, d_ff=64, E=E, k=k, capacity_factor=cf)
    want = O.capacity(T, E, k, cf)
    got = M.moe_capacity(cfg)
    if want >= O.DROPLESS - 1 and cf > 0:
        assert got >= k * T          # clamped, but never binding
    else:
        assert got == want


@pytest.mark.parametrize("bad", [dict(d_model=100), dict(d_ff=0), dict(E=0), dict(E=257), dict(k=0), dict(k=5, E=4),
                                 dict(k=9, E=16), dict(T=-1), dict(capacity_factor=float("nan")),
                                 dict(capacity_factor=float("inf"))])
def test_invalid_configs_are_rejected(bad):
    kw = dict(T=16, d_model=64, d_ff=64, E=4, k=2)
    kw.update(bad)
    cfg = M.MoEConfig(**kw)
    c = cfg.c()
    assert M.lib().moe_config_check(C.byref(c)) == 1
    assert M.lib().moe_capacity(C.byref(c)) == -1
    assert M.lib().moe_workspace_bytes(C.byref(c), 0) == 0
    assert len(M.lib().moe_last_error()) > 0


def test_null_and_workspace_errors_launch_nothing():
    # these return before any HIP call, so they run without a GPU
    L = M.lib()
    cfg = M.MoEConfig(T=16, d_model=64, d_ff=64, E=4, k=2).c()
    assert L.moe_gate(C.byref(cfg), None, None, None, None, None, None, None) == 1
    assert L.moe_dispatch(C.byref(cfg), None, None, None, None, None, None, None, None, 0, None) == 1
    fake = C.c_void_p(0x1000)
    fake2 = C.c_void_p(0x2000)
    assert L.moe_dispatch(C.byref(cfg), fake, fake, fake, fake, fake, fake, fake, None, 0, None) == 3
    assert L.moe_dispatch(C.byref(cfg), fake, fake, fake, fake, fake, fake, fake, C.c_void_p(0x1010), 1 << 20, None) == 3
    assert L.moe_dispatch(C.byref(cfg), fake, fake, fake, fake, fake, fake, fake, fake, 8, None) == 3
    w = M.binding._Weights()
    assert L.moe_expert_ffn(C.byref(cfg), C.byref(w), fake, fake, fake, fake, 1 << 30, None) == 1   # no w1/w2
    w.w1, w.w2, w.layout = 0x1000, 0x1000, 0
    assert L.moe_expert_ffn(C.byref(cfg), C.byref(w), fake, fake, fake, fake, 1 << 30, None) == 2   # bf16 input-major
    w.layout = 1
    assert L.moe_expert_ffn(C.byref(cfg), C.byref(w), fake, fake, fake, None, 0, None) == 3
    assert L.moe_layer_forward(C.byref(cfg), C.byref(w), fake, None, fake2, fake, 1 << 30, None) == 1  # no router
    w.w_router = 0x1000
    assert L.moe_layer_forward(C.byref(cfg), C.byref(w), fake, None, fake2, fake, 16, None) == 3
    assert L.moe_layer_forward(C.byref(cfg), C.byref(w), fake, None, fake2, None, 0, None) == 3
    assert L.moe_layer_forward(C.byref(cfg), C.byref(w), fake, None, fake, fake, 1 << 30, None) == 1   # out aliases x
    assert L.moe_combine(C.byref(cfg), fake, None, None, None, None, None) == 1
    assert L.moe_transpose_expert_weights(fake, fake, 1, 4, 4, 1, None) == 1
    assert L.moe_timer_read(None, None) == 1


def test_tuning_switches_validate_and_round_trip():
    assert M.moe_get_tuning(M.MOE_TUNE_GEMM_TILE_ROWS) == 0
    assert M.moe_get_tuning(M.MOE_TUNE_FEW_TOKEN_KERNELS) == 1
    for v in (256, 320, 0):
        M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, v)
        assert M.moe_get_tuning(M.MOE_TUNE_GEMM_TILE_ROWS) == v
    assert M.lib().moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, 128) == 1
    assert M.moe_get_tuning(M.MOE_TUNE_GEMM_TILE_ROWS) == 0
    assert M.lib().moe_set_tuning(M.MOE_TUNE_FEW_TOKEN_KERNELS, 2) == 1
    for v in (16, 32, 0):
        M.moe_set_tuning(M.MOE_TUNE_GEMM_MFMA, v)
        assert M.moe_get_tuning(M.MOE_TUNE_GEMM_MFMA) == v
    assert M.lib().moe_set_tuning(M.MOE_TUNE_GEMM_MFMA, 8) == 1
    assert M.lib().moe_set_tuning(7, 0) == 1
    assert M.lib().moe_get_tuning(7, None) == 1


def test_workspace_layout_is_consistent():
    for kw in [dict(T=8192, d_model=1024, d_ff=4096, E=16, k=2, capacity_factor=1.25),
               dict(T=16384, d_model=768, d_ff=3072, E=8, k=1, capacity_factor=0.0),
               dict(T=256, d_model=128, d_ff=512, E=4, k=1, capacity_factor=1.25, dtype="f32"),
               dict(T=0, d_model=64, d_ff=64, E=4, k=1)]:
        cfg = M.MoEConfig(**kw)
        L = M.moe_workspace_layout(cfg)
        assert L["total"] == M.moe_workspace_bytes(cfg, 0)
        C_ = O.capacity(cfg.T, cfg.E, cfg.k, cfg.capacity_factor)
        assert L["r_max"] == min(cfg.k * cfg.T, cfg.E * C_)
        order = ["topk_idx", "topk_w", "expert_counts", "expert_offsets", "assign_to_row", "row_to_assign",
                 "xd", "h", "yd", "scratch", "tile_counters", "total"]
        offs = [L[n] for n in order]
        assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
        s = 2 if cfg.dtype == "bf16" else 4
        # segments the bf16 path never writes are empty: xd (rows are gathered from x), yd when k = 1
        if cfg.dtype == "bf16":
            assert L["h"] == L["xd"]
        else:
            assert L["h"] - L["xd"] >= L["r_max"] * cfg.d_model * s
        assert L["yd"] - L["h"] >= L["r_max"] * cfg.d_ff * s
        if cfg.dtype == "bf16" and cfg.k == 1:
            assert L["scratch"] == L["yd"]
        else:
            assert L["scratch"] - L["yd"] >= L["r_max"] * cfg.d_model * s
        assert L["total"] - L["tile_counters"] >= 16 * 4
        assert M.moe_workspace_bytes(cfg, 2) >= L["r_max"] * cfg.d_ff * s + 16 * 4


# ----------------------------------------------------------------- ring state machine on the host
class FakeBackend:
    """Records every backend call; events are small integers; nothing touches a GPU."""

    def __init__(self, fail_copy_at=None):
        self.log = []
        self.n_events = 0
        self.copies = 0
        self.fail_copy_at = fail_copy_at
        B = M.binding

        def copy(user, dst, src, nbytes, stream):
            self.copies += 1
            if self.fail_copy_at is not None and self.copies == self.fail_copy_at:
                return 1
            self.log.append(("copy", dst, src, nbytes, stream))
            return 0

        def ev_create(user, out):
            self.n_events += 1
            out[0] = 1000 + self.n_events
            return 0

        def ev_destroy(user, ev):
            self.n_events -= 1
            return 0

        def ev_record(user, ev, stream):
            self.log.append(("record", ev, stream))
            return 0

        def wait(user, stream, ev):
            self.log.append(("wait", stream, ev))
            return 0

        def ev_sync(user, ev):
            return 0

        def elapsed(user, a, b, out):
            out[0] = 2.0
            return 0

        self.cbs = (B.RING_COPY_FN(copy), B.RING_EVCREATE_FN(ev_create), B.RING_EV_FN(ev_destroy),
                    B.RING_EV2_FN(ev_record), B.RING_EV2_FN(wait), B.RING_EV_FN(ev_sync), B.RING_ELAPSED_FN(elapsed))
        self.struct = B.RingBackend(None, *self.cbs)


COPY_STREAM, COMPUTE_STREAM = 0x7000, 0x8000
DEV_BASE, LAYER_BYTES = 0x100000, 4096


def host_ptr(layer):
    return 0x9000000 + layer * 0x10000


@pytest.mark.parametrize("N,K,steps", [(6, 2, 2), (5, 2, 3), (24, 4, 1), (3, 3, 2), (2, 4, 2), (7, 3, 2)])
def test_ring_follows_the_oracle_schedule(N, K, steps):
    be = FakeBackend()
    ring = M.Ring(DEV_BASE, K * LAYER_BYTES, K, [host_ptr(l) for l in range(N)], LAYER_BYTES,
                  copy_stream=COPY_STREAM, backend=be.struct)
    got = []
    for g in range(steps * N):
        layer = g % N
        n_before = len(be.log)
        p = ring.acquire(layer, COMPUTE_STREAM)
        # acquire = exactly one wait of the compute stream on an event
        assert [e[0] for e in be.log[n_before:]] == ["wait"] and be.log[n_before][1] == COMPUTE_STREAM
        got.append(("compute", layer, (p - DEV_BASE) // LAYER_BYTES))
        ring.release(layer, COMPUTE_STREAM)
    # rebuild the load/compute sequence from the backend log
    ev = []
    ci = 0
    for e in be.log:
        if e[0] == "copy":
            assert e[3] == LAYER_BYTES and e[4] == COPY_STREAM and (e[1] - DEV_BASE) % LAYER_BYTES == 0
            ev.append(("load", (e[2] - host_ptr(0)) // 0x10000, (e[1] - DEV_BASE) // LAYER_BYTES))
        elif e[0] == "wait" and e[1] == COMPUTE_STREAM:
            ev.append(got[ci])
            ci += 1
    assert ev == O.ring_schedule(N, K, steps)
    st = ring.stats()
    loads = sum(1 for e in ev if e[0] == "load")
    assert st["copies"] == loads and st["bytes_copied"] == loads * LAYER_BYTES and st["copy_ms"] == 2.0 * loads
    # a refill is ordered after the compute that released the section: record(compute) -> wait(copy) -> copy
    if min(K, N) < N:
        for i, e in enumerate(be.log):
            if e[0] == "copy" and i > 4 * min(K, N):
                kinds = [x[0] for x in be.log[max(0, i - 3):i]]
                assert kinds[-3:] == ["record", "wait", "record"], kinds
                assert be.log[i - 3][2] == COMPUTE_STREAM and be.log[i - 2][1] == COPY_STREAM
                assert be.log[i - 2][2] == be.log[i - 3][1]          # waits on the event just recorded
    ring.close()
    assert be.n_events == 0                                          # every event destroyed


def test_ring_rejects_out_of_order_use_and_bad_arguments():
    be = FakeBackend()
    ring = M.Ring(DEV_BASE, 2 * LAYER_BYTES, 2, [host_ptr(l) for l in range(4)], LAYER_BYTES, COPY_STREAM, be.struct)
    with pytest.raises(M.MoEError) as e:
        ring.acquire(1, COMPUTE_STREAM)
    assert e.value.status == 5
    ring.acquire(0, COMPUTE_STREAM)
    with pytest.raises(M.MoEError):
        ring.acquire(0, COMPUTE_STREAM)          # not released yet
    with pytest.raises(M.MoEError):
        ring.release(1, COMPUTE_STREAM)
    ring.release(0, COMPUTE_STREAM)
    with pytest.raises(M.MoEError):
        ring.release(0, COMPUTE_STREAM)
    ring.close()
    for kw in [dict(budget=LAYER_BYTES), dict(base=0), dict(base=DEV_BASE + 8), dict(layer_bytes=100), dict(K=0)]:
        with pytest.raises(M.MoEError) as e:
            M.Ring(kw.get("base", DEV_BASE), kw.get("budget", 2 * LAYER_BYTES), kw.get("K", 2),
                   [host_ptr(l) for l in range(4)], kw.get("layer_bytes", LAYER_BYTES), COPY_STREAM, FakeBackend().struct)
        assert e.value.status == 1


def test_ring_reports_a_failed_copy():
    be = FakeBackend(fail_copy_at=3)             # two preloads succeed, the first refill fails
    ring = M.Ring(DEV_BASE, 2 * LAYER_BYTES, 2, [host_ptr(l) for l in range(4)], LAYER_BYTES, COPY_STREAM, be.struct)
    ring.acquire(0, COMPUTE_STREAM)
    with pytest.raises(M.MoEError) as e:
        ring.release(0, COMPUTE_STREAM)
    assert e.value.status == 4
    ring.close()
    be2 = FakeBackend(fail_copy_at=1)
    with pytest.raises(M.MoEError):
        M.Ring(DEV_BASE, 2 * LAYER_BYTES, 2, [host_ptr(l) for l in range(4)], LAYER_BYTES, COPY_STREAM, be2.struct)
    assert be2.n_events == 0
    # the statistics stay readable after a failed copy (its event pair never joined the pending copies)
    be3 = FakeBackend(fail_copy_at=3)
    ring = M.Ring(DEV_BASE, 2 * LAYER_BYTES, 2, [host_ptr(l) for l in range(4)], LAYER_BYTES, COPY_STREAM, be3.struct)
    ring.acquire(0, COMPUTE_STREAM)
    with pytest.raises(M.MoEError):
        ring.release(0, COMPUTE_STREAM)
    st = ring.stats()
    assert st["copies"] == 2 and st["copy_ms"] == 4.0
    ring.close()
    assert be3.n_events == 0


def test_ring_recycles_its_copy_events_without_a_stats_call():
    """An inference loop that never reads the statistics: the number of live events stays bounded (a few rings'
    worth of copies), and the totals are still complete when they are finally read."""
    N, K = 6, 2
    be = FakeBackend()
    ring = M.Ring(DEV_BASE, K * LAYER_BYTES, K, [host_ptr(l) for l in range(N)], LAYER_BYTES, COPY_STREAM, be.struct)
    peak = 0
    for g in range(50 * N):
        ring.acquire(g % N, COMPUTE_STREAM)
        ring.release(g % N, COMPUTE_STREAM)
        peak = max(peak, be.n_events)
    assert peak <= 2 * K + 2 * (4 * K + 16) + 2, peak      # section events + event pairs of the pending copies
    st = ring.stats()
    assert st["copies"] == K + 50 * N and st["copy_ms"] == 2.0 * st["copies"]
    ring.close()
    assert be.n_events == 0


def test_binding_refuses_tensors_smaller_than_the_configuration_says():
    """bfloat16 tensors under a float32 configuration (or a short buffer) must fail on the host, before any launch:
    behind the C ABI they would be read and written past their end on the device."""
    import torch
    cfg = M.MoEConfig(T=64, d_model=128, d_ff=256, E=4, k=1, capacity_factor=0.0, act="gelu", dtype="f32")
    x = torch.zeros(64, 128, dtype=torch.bfloat16)       # half the bytes the configuration needs
    ok = torch.zeros(64, 128, dtype=torch.float32)
    wr = torch.zeros(128, 4)
    idx = torch.zeros(64, 1, dtype=torch.int32)
    w = torch.zeros(64, 1)
    with pytest.raises(ValueError, match="x holds"):
        M.moe_gate(cfg, x, wr, None, idx, w)
    with pytest.raises(ValueError, match="topk_idx holds"):
        M.moe_gate(cfg, ok, wr, None, idx[:32], w)
    with pytest.raises(ValueError, match="w_router holds"):
        M.moe_gate(cfg, ok, wr[:, :2].contiguous(), None, idx, w)
    W = M.Weights.__new__(M.Weights)                      # (no device pointers needed for the size check)
    W.tensors = {"w_router": wr, "w1": torch.zeros(4, 256, 128, dtype=torch.bfloat16), "w2": torch.zeros(4, 128, 256)}
    with pytest.raises(ValueError, match="w1 holds"):
        W.need(cfg)
    with pytest.raises(ValueError, match="out holds"):
        M.moe_combine(cfg, None, idx, w, None, x)
