"""Benchmark of the staged multi-tenant forward pass on one MI355X.

One step = one pass of the whole hot path: every operator of every tenant of the workload, issued according
to a schedule (sequential, all-concurrent, or the searched pointer matrix), inputs resident in HBM.
Prints one JSON line; `value` is aggregate images per second under the searched schedule.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0, "f32": 157.3}
PEAK_HBM_GBS = 8000.0


def speedup(sequential_ms, ours_ms):
    """Speed-up as the paper's tables print it: sequential latency divided by ours (Tables I-II)."""
    return sequential_ms / ours_ms


def time_schedule(ctx, torch, sched, inputs, outputs, warmup, steps):
    bound = ctx.bind(inputs, outputs)              # pointer marshalling stays outside the timed loop
    for _ in range(warmup):
        ctx.run_makespan(sched, bound)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mk, issue = [], []
    for _ in range(steps):
        m, h = ctx.run_makespan(sched, bound)
        mk.append(m)
        issue.append(h)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    mk.sort()
    mean = sum(mk) / len(mk)
    return {"wall_ms_per_step": wall_ms, "makespan_ms_mean": mean, "makespan_ms_min": mk[0],
            "makespan_ms_stdev": (sum((v - mean) ** 2 for v in mk) / max(1, len(mk) - 1)) ** 0.5,
            "makespan_ms_median": mk[len(mk) // 2], "makespan_ms_p90": mk[(len(mk) * 9) // 10 if len(mk) > 1 else 0],
            "host_issue_ms_mean": sum(issue) / len(issue)}


def kernel_rooflines(ctx, inputs, outputs, dtype, repeats):
    """Per kernel family: launches, total time, algorithmic flops and bytes, from back-to-back timed launches."""
    from paper_2111_14255_amd import binding as B
    fam = {}
    for t in range(ctx.num_tenants()):
        ms = ctx.profile_ops(t, inputs[t], outputs[t], repeats)
        for i, d in enumerate(ms):
            info = ctx.op_info(t, i)
            name = B.load().mt_kernel_name(info.kernel_id).decode()
            f = fam.setdefault(name, {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
            f["launches"] += 1
            f["ms"] += d
            f["flops"] += info.flops
            f["bytes"] += info.bytes
    return fam


def measured_traffic(workload, kernel):
    """HBM bytes per launch of the dominant kernel, from the rocprofv3 counter runs summarised under profiles/
    (FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for a copy of known size)."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.json" % workload)
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    return rec.get(kernel, {}).get("hbm_bytes_per_launch")


def cpu_baseline(specs, raws, xs, budget_s=10.0):
    """The CPU oracle, as it stands, timed on this host: whole forward passes of tenants of the workload, one after
    another in tenant order (wrapping around), until `budget_s` seconds of CPU work are spent (at least one pass)."""
    from oracle import forward as OF, ops as oops
    params = [OF.prepare_params(m, raw) for m, raw in zip(specs, raws)]
    passes, images, macs, t0 = 0, 0, 0.0, time.perf_counter()
    while True:
        k = passes % len(specs)
        OF.forward(specs[k], params[k], xs[k])
        passes += 1
        images += specs[k].batch
        macs += specs[k].macs()
        dt = time.perf_counter() - t0
        if dt >= budget_s or passes >= 50 * len(specs):
            break
    return {"value": images / dt, "unit": "img/s", "cores": oops.num_threads(), "kind": "oracle",
            "sample": "%d tenant forward passes (tenants 0..%d of %d in turn, %d images, %.1f GMAC) in %.2f s" %
                      (passes, min(passes, len(specs)) - 1, len(specs), images, macs / 1e9, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg5", help="workload: cfg5 (the headline: the largest single-GPU one), cfg1 .. cfg4")
    ap.add_argument("--search-rounds", type=int, default=2)
    ap.add_argument("--search-candidates", type=int, default=6)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the three schedules of the headline mode and the roofline")
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the per-kernel timing pass (back-to-back launches of every operator) preceded by a "
                         "64 MiB elementwise copy that calibrates byte counters; this is the command profiled under rocprofv3")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); with more, independent tenants would be "
              "bin-packed across GPUs by their profiled latency, each GPU running its own schedule", file=sys.stderr)
        sys.exit(2)

    from paper_2111_14255_amd import api, binding as B     # first: sets the runtime's environment before HIP initialises
    import torch
    from synth import configs, weights

    cfg = configs.CONFIGS[args.config]
    specs = cfg.models()
    raws = [weights.make_params(m, cfg.seed, t) for t, m in enumerate(specs)]
    xs = [weights.make_input(m, cfg.seed, t, cfg.input_dist) for t, m in enumerate(specs)]
    # The CPU baseline comes first, before the first HIP call of the process: once the GPU runtime runs (with host
    # waits that poll the device signal) it keeps a polling thread of its own, which would share a core with one of
    # the oracle's threads and hold all of them back at every operator.
    cpu = None if (args.no_cpu_baseline or args.roofline_only) else cpu_baseline(specs, raws, xs)
    ctx = api.Context(0)
    for m, raw in zip(specs, raws):
        model = api.Model(m, raw)
        ctx.register(model)
        model.close()
    inputs = [ctx.make_input(t, x) for t, x in enumerate(xs)]
    outputs = [ctx.make_output(t) for t in range(len(specs))]
    images = sum(m.batch for m in specs)
    lens = ctx.lens()

    if args.roofline_only:
        cal = torch.ones(32 * 1024 * 1024, dtype=torch.float16, device="cuda")   # 64 MiB read + 64 MiB written
        cal2 = cal * 1
        torch.cuda.synchronize()
        fam = kernel_rooflines(ctx, inputs, outputs, cfg.dtype, repeats=10)
        print(json.dumps({"workload": cfg.name, "calibration_copy_bytes": int(cal.numel() * 2), "families": fam}))
        del cal2
        ctx.close()
        return

    # ---- the headline mode, fixed before anything is timed --------------------------------
    # One issuing host thread per tenant stream, stage barriers taken on the host, neighbouring operator pairs of a
    # stage that have a fused kernel issued as one launch (identical output bits).  The three schedules of the metric
    # (sequential, all-concurrent, searched) run in this same mode; `value` is the searched one.
    FE = B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_POOL
    MODE = FE | B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER
    # The searched schedule may also co-issue: where it puts two tenants of equal architecture on one stream, operator i
    # of both runs as one launch (identical output bits).  That is a form of running tenants side by side, so the two
    # baselines, which define "one after another" and "one stream each", run without it.
    SMODE = MODE | B.MT_SCHED_COISSUE
    HEAD = "searched"
    results = {}
    t0 = time.perf_counter()
    rho, cost, records, shares, prio, conc = ctx.search(
        inputs, outputs, cfg.n_stages, rounds=args.search_rounds, candidates=args.search_candidates, runs=5, warmup=1,
        seed=cfg.seed, cu_share_rounds=1, wave_priority_rounds=1, search_concurrency=True, playoff_top=3, playoff_runs=21,
        flags=SMODE)
    search_s = time.perf_counter() - t0
    trio = (("sequential", ctx.sequential(flags=MODE)),
            ("all_concurrent", ctx.all_concurrent(flags=MODE)),
            ("searched", ctx.schedule(rho, cfg.n_stages, concurrency=conc, cu_share=shares, flags=SMODE, wave_priority=prio)))
    for name, s in trio:
        results[name] = time_schedule(ctx, torch, s, inputs, outputs, args.warmup, args.steps)
    results[HEAD].update({"pointers": rho, "stage_concurrency": conc, "cu_share": shares, "wave_priority": prio,
                          "search_seconds": search_s, "search_evaluations": len(records),
                          "one_stage_matrix": all(v == n for row, n in zip(rho, lens) for v in row)})
    # when each tenant finishes inside the searched schedule (one more event per tenant; not part of the timed variants)
    st = ctx.schedule(rho, cfg.n_stages, concurrency=conc, cu_share=shares, wave_priority=prio, flags=SMODE | B.MT_SCHED_TIME_TENANTS)
    bound = ctx.bind(inputs, outputs)
    runs = [ctx.run(st, bound) for _ in range(args.warmup + 11)][args.warmup:]
    done = [r["tenant_done_ms"] for r in runs]
    results[HEAD]["tenant_done_ms_median"] = [sorted(d[t] for d in done)[len(done) // 2] for t in range(len(specs))]    # tenant order
    results[HEAD]["operators_inside_another_launch"] = runs[-1]["n_fused"]      # fused pairs of one tenant and co-issued operators
    st.close()

    if not args.no_extras:
        # context: the paper's single issuing thread on plain streams (pointer search only), and whole-schedule graph replay
        for flags, suffix in ((0, "+main_thread"), (B.MT_SCHED_GRAPH, "+graph")):
            t0 = time.perf_counter()
            rho2, cost2, rec2 = ctx.search(inputs, outputs, cfg.n_stages, rounds=args.search_rounds, candidates=args.search_candidates,
                                           runs=5, warmup=1, seed=cfg.seed, playoff_top=3, playoff_runs=11, flags=flags)
            s2 = time.perf_counter() - t0
            for name, s in (("sequential", ctx.sequential(flags=flags)), ("all_concurrent", ctx.all_concurrent(flags=flags)),
                            ("searched", ctx.schedule(rho2, cfg.n_stages, flags=flags))):
                results[name + suffix] = time_schedule(ctx, torch, s, inputs, outputs, args.warmup, args.steps)
            results["searched" + suffix].update({"pointers": rho2, "search_seconds": s2, "search_evaluations": len(rec2),
                                                 "one_stage_matrix": all(v == n for row, n in zip(rho2, lens) for v in row)})
    for k, r in results.items():
        suffix = k[k.index("+"):] if "+" in k else ""
        r["img_per_s"] = images / (r["wall_ms_per_step"] * 1e-3)
        r["speedup_vs_sequential"] = speedup(results["sequential" + suffix]["makespan_ms_mean"], r["makespan_ms_mean"])
        r["speedup_vs_all_concurrent"] = speedup(results["all_concurrent" + suffix]["makespan_ms_mean"], r["makespan_ms_mean"])
    head = results[HEAD]

    # ---- roofline of the dominant kernel ----------------------------------------------------
    fam = kernel_rooflines(ctx, inputs, outputs, cfg.dtype, repeats=10)
    dom = max(fam, key=lambda k: fam[k]["ms"])
    f = fam[dom]
    # The family is priced against the MFMA peak when its arithmetic intensity (algorithmic flops per algorithmic
    # byte over its launches) is above the ridge of the chip, against the HBM peak otherwise.
    ridge = PEAK_TFLOPS[cfg.dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    if f["bytes"] > 0 and f["flops"] / f["bytes"] >= ridge:
        achieved = f["flops"] / (f["ms"] * 1e-3) / 1e12
        roof = {"kernel": dom, "bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[cfg.dtype], "unit": "TFLOP/s",
                "frac": achieved / PEAK_TFLOPS[cfg.dtype]}
    else:
        achieved = f["bytes"] / (f["ms"] * 1e-3) / 1e9
        roof = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS}
    roof["arithmetic_intensity_flop_per_byte"] = f["flops"] / f["bytes"] if f["bytes"] else None
    roof["launches_per_step"] = f["launches"]
    roof["avg_launch_us"] = f["ms"] * 1e3 / f["launches"]
    roof["traffic"] = measured_traffic(cfg.name, dom)
    # every family against both peaks: MFMA utilisation for the conv / FC families, achieved HBM rate for the rest
    roof["families"] = {k: {"launches": v["launches"], "us": round(v["ms"] * 1e3, 2),
                            "TFLOP/s": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] > 0 else 0.0,
                            "GB/s": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else 0.0,
                            "frac_of_mfma_peak": round(v["flops"] / (v["ms"] * 1e-3) / 1e12 / PEAK_TFLOPS[cfg.dtype], 4) if v["ms"] > 0 else 0.0,
                            "frac_of_hbm_peak": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if v["ms"] > 0 else 0.0}
                        for k, v in fam.items()}
    total_flops = sum(v["flops"] for v in fam.values())
    total_bytes = sum(v["bytes"] for v in fam.values())
    # what this chip sustains on the simplest possible kernels, next to the published peaks the fractions above use
    measured = {"mfma_%s_TFLOP/s" % cfg.dtype: round(ctx.peak_mfma(cfg.dtype), 1) if cfg.dtype != "f32" else None,
                "hbm_copy_GB/s": round(ctx.peak_stream("copy"), 1),
                "hbm_read_GB/s": round(ctx.peak_stream("read"), 1)}
    roof["measured_peaks"] = measured
    m_peak = measured["mfma_%s_TFLOP/s" % cfg.dtype] if roof["bound"] == "mfma" else measured["hbm_read_GB/s"]
    roof["frac_of_measured_peak"] = achieved / m_peak if m_peak else None

    # the larger of the two whole-pass bounds over each schedule's makespan
    bound_ms = max(total_flops / (PEAK_TFLOPS[cfg.dtype] * 1e12), total_bytes / (PEAK_HBM_GBS * 1e9)) * 1e3
    for r in results.values():
        r["frac_of_roofline_bound"] = bound_ms / r["makespan_ms_mean"]

    out = {
        "metric": "aggregate images/s of the multi-tenant forward pass under the searched schedule (makespan in ms_per_step)",
        "value": head["img_per_s"],
        "unit": "img/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["wall_ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: %s, batch %d, %s storage, fp32 accumulate" % (cfg.name, "+".join(cfg.tenants), cfg.batch, cfg.dtype),
                   "images_per_step": images, "launches_per_step": sum(lens), "headline_schedule": HEAD,
                   "headline_mode": "one issuing thread per tenant stream, host-side stage barriers, fused operator pairs; searched schedule only: co-issue of equal tenants that share a stream",
                   "n_stages": cfg.n_stages},
        "speedup_vs_sequential": head["speedup_vs_sequential"],
        "speedup_vs_all_concurrent": head["speedup_vs_all_concurrent"],
        "schedules": results,
        "bounds": {"flops_bound_us": total_flops / (PEAK_TFLOPS[cfg.dtype] * 1e12) * 1e6,
                   "bytes_bound_us": total_bytes / (PEAK_HBM_GBS * 1e9) * 1e6,
                   "makespan_frac_of_bound": bound_ms / head["makespan_ms_mean"]},
        "roofline": roof,
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
