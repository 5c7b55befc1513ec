"""The machine probes of the library on the GPU: sustained matrix-instruction and memory rates (the measured figures
that stand next to the published peaks in a roofline), compute-unit masks and dispatch latency."""
import ctypes as C

import pytest

from paper_2111_14255_amd import api, binding as B

pytestmark = pytest.mark.gpu


def test_peak_probes_are_sane_and_reject_bad_arguments():
    ctx = api.Context(0)
    try:
        for dt in ("f16", "bf16"):
            print("peak mfma", dt, flush=True)
            tf = ctx.peak_mfma(dt, 20000)
            print("  %.0f TFLOP/s" % tf, flush=True)
            assert 300.0 < tf < 2500.0 * 1.05       # a register-only loop cannot beat the published dense peak
        for mode in ("copy", "read"):
            print("peak stream", mode, flush=True)
            gb = ctx.peak_stream(mode, 1 << 30, reps=4)
            print("  %.0f GB/s" % gb, flush=True)
            assert 1500.0 < gb < 8000.0 * 1.05       # 1 GiB per launch is four times the last-level cache
        with pytest.raises(B.MtError):
            ctx.peak_mfma("f32", 10)
        with pytest.raises(B.MtError):
            ctx.peak_mfma("f16", 0)
        with pytest.raises(B.MtError):
            ctx.peak_stream("copy", 1000, reps=1)
        with pytest.raises(B.MtError):
            ctx.peak_stream("read", (1 << 20) + 8, reps=1)
        with pytest.raises(B.MtError):
            ctx.peak_stream("read", 1 << 20, reps=1, groups_per_unit=0)
    finally:
        ctx.close()


def test_cu_mask_probe_and_dispatch_latency():
    ctx = api.Context(0)
    try:
        cus = ctx.device_info().cu_count
        n = 512
        ids = (C.c_uint32 * (2 * n))()
        print("cu mask probe, share 32", flush=True)
        B.check(ctx.lib.mt_probe_cu_mask(ctx.h, 32, 0, n, ids))
        units = {(ids[2 * i] & 0xff00, ids[2 * i + 1] & 0xf) for i in range(n)}
        assert 1 <= len(units) <= 32                  # never more distinct units than the share
        B.check(ctx.lib.mt_probe_cu_mask(ctx.h, 0, 0, n, ids))
        assert len({(ids[2 * i] & 0xff00, ids[2 * i + 1] & 0xf) for i in range(n)}) > 32
        with pytest.raises(B.MtError):
            B.check(ctx.lib.mt_probe_cu_mask(ctx.h, cus + 1, 0, n, ids))
        us = (C.c_float * 2)()
        print("dispatch latency probe", flush=True)
        B.check(ctx.lib.mt_probe_dispatch_latency(ctx.h, 2, 0, 16, us))
        assert all(1.0 < v < 200.0 for v in us)
    finally:
        ctx.close()


def test_barrier_cost_probe_every_kind():
    ctx = api.Context(0)
    try:
        for n in (1, 3):
            base = None
            for kind in range(5):
                print("barrier probe, %d streams, kind %d" % (n, kind), flush=True)
                v = C.c_float()
                B.check(ctx.lib.mt_probe_barrier_cost(ctx.h, n, kind, 20, C.byref(v)))
                assert 1.0 < v.value < 5000.0
                if kind == 0:
                    base = v.value
            assert base is not None
        for bad in ((0, 0, 10), (2, 5, 10), (2, 1, 0), (17, 1, 10)):
            with pytest.raises(B.MtError):
                B.check(ctx.lib.mt_probe_barrier_cost(ctx.h, bad[0], bad[1], bad[2], C.byref(C.c_float())))
    finally:
        ctx.close()


def test_stream_conflict_probe_and_tenant_streams_side_by_side():
    """The pair probe returns a symmetric table whose entries are one or about two launch times, and the streams the
    runtime hands to tenant indices 0 .. 3 run side by side: four single-operator chains on four streams take far less
    than four times one chain."""
    ctx = api.Context(0)
    try:
        n = 6
        single = (C.c_float * n)()
        pair = (C.c_float * (n * n))()
        print("stream conflict probe", flush=True)
        B.check(ctx.lib.mt_probe_stream_conflicts(ctx.h, n, 16, single, pair))
        lo = min(single)
        assert 1.0 < lo < 200.0
        for i in range(n):
            assert pair[i * n + i] == single[i]
            for j in range(n):
                assert pair[i * n + j] == pair[j * n + i]
                assert 0.5 * lo < pair[i * n + j] < 8.0 * lo
        for bad in ((1, 16), (33, 16), (4, 0), (4, 257)):
            with pytest.raises(B.MtError):
                B.check(ctx.lib.mt_probe_stream_conflicts(ctx.h, bad[0], bad[1], single, pair))
        # kind 0 of the barrier probe: rounds of one short kernel per tenant stream, no barrier
        one, four = C.c_float(), C.c_float()
        B.check(ctx.lib.mt_probe_barrier_cost(ctx.h, 1, 0, 64, C.byref(one)))
        B.check(ctx.lib.mt_probe_barrier_cost(ctx.h, 4, 0, 64, C.byref(four)))
        print("round of 1 stream %.1f us, of 4 streams %.1f us" % (one.value, four.value), flush=True)
        assert four.value < 3.5 * one.value                 # four streams one after the other would take four times one
    finally:
        ctx.close()
