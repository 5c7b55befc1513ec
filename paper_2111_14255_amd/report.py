"""Reports on the scheduling layer, measured on the GPU: markdown on stdout.

  search   best-so-far latency against evaluations for coordinate descent and random search, and the wall time of
           the search (the analogues of the paper's search-curve figure and search-overhead table, Sec. IV)
  issue    breadth-first against depth-first issue of the same schedules, with the host issue time and the stall of
           every stream behind the main thread (Sec. III-D), and the same schedules replayed as a device graph
  mixes    sequential, all-concurrent and searched latency of the paper's tenant combinations (Tables I-II)
  fusion   every tenant alone and all tenants together, with and without the fused launches of neighbouring operators
           and with wave priorities (the runtime's additions to the paper's method)

    python -m paper_2111_14255_amd.report search --config cfg2
    python -m paper_2111_14255_amd.report issue --config cfg2
    python -m paper_2111_14255_amd.report mixes
    python -m paper_2111_14255_amd.report fusion --config cfg2
"""
import argparse
import sys
import time


def _setup(cfg):
    from synth import weights
    from . import api
    specs = cfg.models()
    ctx = api.Context(0)
    for t, m in enumerate(specs):
        model = api.Model(m, weights.make_params(m, cfg.seed, t))
        ctx.register(model)
        model.close()
    inputs = [ctx.make_input(t, weights.make_input(m, cfg.seed, t, cfg.input_dist)) for t, m in enumerate(specs)]
    outputs = [ctx.make_output(t) for t in range(len(specs))]
    return ctx, specs, inputs, outputs


def _time(ctx, sched, inputs, outputs, steps=40, warmup=5):
    for _ in range(warmup):
        ctx.run(sched, inputs, outputs)
    mk, issue = [], []
    for _ in range(steps):
        tm = ctx.run(sched, inputs, outputs)
        mk.append(tm["makespan_ms"])
        issue.append(tm["host_issue_ms"])
    mk.sort()
    issue.sort()
    return {"median": mk[len(mk) // 2], "min": mk[0], "p90": mk[(len(mk) * 9) // 10], "issue": issue[len(issue) // 2]}


def _best_so_far(records):
    out, best = [], float("inf")
    for _, c in records:
        best = min(best, c)
        out.append(best)
    return out


def report_search(args):
    from synth import configs
    from . import binding as B
    cfg = configs.ALL[args.config]
    ctx, specs, inputs, outputs = _setup(cfg)
    seq = _time(ctx, ctx.sequential(), inputs, outputs)
    allc = _time(ctx, ctx.all_concurrent(), inputs, outputs)
    print("# Search curves, workload %s (%s), %d stages" % (cfg.name, " + ".join(cfg.tenants), cfg.n_stages))
    print()
    print("Command: `python -m paper_2111_14255_amd.report search --config %s --rounds %d --candidates %d --runs %d --seeds %d`"
          % (cfg.name, args.rounds, args.candidates, args.runs, args.seeds))
    print()
    print("Cost of a candidate = median makespan of %d timed runs after 1 warm-up run, one stream per tenant, breadth-first "
          "issue, no baseline seeding (both searches start cold).  Sequential baseline %.4f ms, all-concurrent %.4f ms."
          % (args.runs, seq["median"], allc["median"]))
    print()
    budget = args.rounds * len(specs) * args.candidates
    marks = sorted(set([1, 2, 4, 8, 16, 32, 64, 128, 256, budget]))
    marks = [m for m in marks if m <= budget]
    print("| algorithm | seed | " + " | ".join("best@%d" % m for m in marks) + " | evaluated | search s | speed-up vs sequential |")
    print("|---|---|" + "---|" * (len(marks) + 3))
    summary = {}
    for algo, name in ((B.MT_SEARCH_COORDINATE, "coordinate descent"), (B.MT_SEARCH_RANDOM, "random")):
        finals, times = [], []
        for sd in range(args.seeds):
            t0 = time.perf_counter()
            # a uniformly drawn matrix is feasible with probability (1 / P!)^n: random search gets that many more
            # draws (capped), so that both searches run about the same number of schedules on the GPU
            factor = 1
            if algo == B.MT_SEARCH_RANDOM:
                for k in range(2, cfg.n_stages):
                    factor *= k
                factor = min(factor ** len(specs), 1024)
            rho, cost, rec = ctx.search(inputs, outputs, cfg.n_stages, rounds=args.rounds * factor, candidates=args.candidates,
                                        runs=args.runs, warmup=1, seed=cfg.seed + 1000 * sd, algo=algo, seed_baselines=False)
            dt = time.perf_counter() - t0
            curve = _best_so_far(rec)
            cells = ["%.4f" % curve[m - 1] if m <= len(curve) else "-" for m in marks]
            print("| %s | %d | %s | %d | %.2f | %.2f |" % (name, sd, " | ".join(cells), len(rec), dt, seq["median"] / cost))
            finals.append(cost)
            times.append(dt)
        summary[name] = (sum(finals) / len(finals), min(finals), max(finals), sum(times) / len(times))
    print()
    print("| algorithm | mean best ms | min | max | mean search s |")
    print("|---|---|---|---|---|")
    for name, (mean, lo, hi, t) in summary.items():
        print("| %s | %.4f | %.4f | %.4f | %.2f |" % (name, mean, lo, hi, t))
    print()
    print("Random search draws every pointer independently; a matrix with a decreasing row is infeasible and is discarded "
          "without being run (about 1 in (P!)^n survives), so it is given min((P!)^n, 1024) times the %d draws of the "
          "coordinate descent and `evaluated` counts the schedules it really ran." % budget)
    ctx.close()


def report_issue(args):
    from synth import configs
    from . import binding as B
    cfg = configs.ALL[args.config]
    ctx, specs, inputs, outputs = _setup(cfg)
    n = len(specs)
    P = cfg.n_stages - 1
    lens = ctx.lens()
    even = [[(lens[i] * (j + 1) + P) // (P + 1) for j in range(P)] for i in range(n)]
    rho, _, _ = ctx.search(inputs, outputs, cfg.n_stages, rounds=args.rounds, candidates=args.candidates, runs=args.runs,
                           warmup=1, seed=cfg.seed)
    print("# Issue order, workload %s (%s)" % (cfg.name, " + ".join(cfg.tenants)))
    print()
    print("Command: `python -m paper_2111_14255_amd.report issue --config %s --rounds %d --candidates %d --runs %d`"
          % (cfg.name, args.rounds, args.candidates, args.runs))
    print()
    print("Median of 40 runs, ms.  `host issue` is the time the issuing thread(s) spend launching one pass.  Under "
          "depth-first issue the main thread launches all of stream 0, then all of stream 1, ...: stream k cannot start "
          "before the main thread has issued every operator of the streams before it, which is the stall the paper's "
          "Fig. 5 measures; breadth-first issue hands every stream its first operator within one round.")
    print()
    print("| schedule | order | mode | makespan | min | p90 | host issue |")
    print("|---|---|---|---|---|---|---|")
    rows = [("all-concurrent (1 stage)", [[] for _ in specs], 1), ("even split", even, cfg.n_stages), ("searched", rho, cfg.n_stages)]
    for label, ptr, ns in rows:
        for order, oname in ((B.MT_ISSUE_BFS, "BFS"), (B.MT_ISSUE_DFS, "DFS")):
            for flags, mode in ((0, "streams"), (B.MT_SCHED_PARALLEL_ISSUE, "streams, one issuing thread per stream"),
                                (B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER, "the same, stage barriers on the host"),
                                (B.MT_SCHED_GRAPH, "graph replay")):
                r = _time(ctx, ctx.schedule(ptr, ns, order=order, flags=flags), inputs, outputs)
                print("| %s | %s | %s | %.4f | %.4f | %.4f | %.4f |" % (label, oname, mode, r["median"], r["min"], r["p90"], r["issue"]))
    print()
    print("Time from the start of a pass to the end of each tenant's first operator, all-concurrent schedule, one issuing "
          "thread, median of 40 runs, us (the paper's Fig. 5 reports 102.75 -> 51.23 us and 177.27 -> 51.23 us for its second "
          "and third stream on its GPU):")
    print()
    print("| order | " + " | ".join("%s (%d ops)" % (m.name, l) for m, l in zip(specs, lens)) + " |")
    print("|---|" + "---|" * n)
    for order, oname in ((B.MT_ISSUE_BFS, "BFS"), (B.MT_ISSUE_DFS, "DFS")):
        sched = ctx.schedule([[] for _ in specs], 1, order=order, flags=B.MT_SCHED_TIME_FIRST_OP)
        for _ in range(5):
            ctx.run(sched, inputs, outputs)
        cols = [[] for _ in specs]
        for _ in range(40):
            tm = ctx.run(sched, inputs, outputs)
            for i in range(n):
                cols[i].append(tm["first_op_done_ms"][i] * 1e3)
        print("| %s | " % oname + " | ".join("%.1f" % sorted(c)[len(c) // 2] for c in cols) + " |")
    ctx.close()


def report_mixes(args):
    from synth import configs
    from . import binding as B
    print("# The paper's tenant combinations (Tables I-II), batch 1, fp16 storage, MI355X")
    print()
    print("Command: `python -m paper_2111_14255_amd.report mixes --rounds %d --candidates %d --runs %d`" % (args.rounds, args.candidates, args.runs))
    print()
    print("Median makespan of 40 runs, ms; speed-up = sequential / schedule, as the paper's tables print it.  "
          "`searched` = coordinate descent over the pointer matrix (4 stages); `+shares` searches the number of streams in "
          "use per stage and the per-tenant CU shares as well, in the mode it is then run in: one issuing host thread per stream, stage barriers taken on the host.  The paper's own numbers (other GPUs, other kernels) are "
          "context only: its coordinate-descent speed-ups for these rows are 1.37, 1.49, 1.49, 1.31, 1.37, 1.63, 1.72 on Titan V.")
    print()
    print("| tenants | launches | sequential | all-concurrent | searched | searched+graph | searched+shares | streams | shares | best speed-up | search s |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    names = args.only.split(",") if args.only else list(configs.PAPER_MIXES)
    for name in names:
        cfg = configs.ALL[name]
        ctx, specs, inputs, outputs = _setup(cfg)
        seq = _time(ctx, ctx.sequential(), inputs, outputs)
        allc = _time(ctx, ctx.all_concurrent(), inputs, outputs)
        t0 = time.perf_counter()
        rho, _, _ = ctx.search(inputs, outputs, cfg.n_stages, rounds=args.rounds, candidates=args.candidates, runs=args.runs,
                               warmup=1, seed=cfg.seed)
        s1 = _time(ctx, ctx.schedule(rho, cfg.n_stages), inputs, outputs)
        rho_g, _, _ = ctx.search(inputs, outputs, cfg.n_stages, rounds=args.rounds, candidates=args.candidates, runs=args.runs,
                                 warmup=1, seed=cfg.seed, flags=B.MT_SCHED_GRAPH)
        s2 = _time(ctx, ctx.schedule(rho_g, cfg.n_stages, flags=B.MT_SCHED_GRAPH), inputs, outputs)
        rho_s, _, _, shares, conc = ctx.search(inputs, outputs, cfg.n_stages, rounds=args.rounds, candidates=args.candidates,
                                               runs=args.runs, warmup=1, seed=cfg.seed, cu_share_rounds=2,
                                               search_concurrency=True,
                                               flags=B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER)
        dt = time.perf_counter() - t0
        s3 = _time(ctx, ctx.schedule(rho_s, cfg.n_stages, concurrency=conc, cu_share=shares,
                                      flags=B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER),
                   inputs, outputs)
        best = min(s1["median"], s2["median"], s3["median"])
        print("| %s | %d | %.4f | %.4f | %.4f | %.4f | %.4f | %d | %s | %.2f | %.1f |" % (
            " + ".join(cfg.tenants), sum(ctx.lens()), seq["median"], allc["median"], s1["median"], s2["median"], s3["median"],
            conc[0], "/".join(str(v) for v in shares), seq["median"] / best, dt))
        sys.stdout.flush()
        ctx.close()


def report_fusion(args):
    from synth import configs, weights
    from . import api, binding as B
    cfg = configs.ALL[args.config]
    FE, FD, FP = B.MT_SCHED_FUSE_EXPAND, B.MT_SCHED_FUSE_DEPTHWISE, B.MT_SCHED_FUSE_POOL
    print("# Fused launches and wave priorities, workload %s (%s)" % (cfg.name, " + ".join(cfg.tenants)))
    print()
    print("Command: `python -m paper_2111_14255_amd.report fusion --config %s`" % args.config)
    print()
    print("Median makespan of 60 runs, ms.  Every output is bit-identical in all columns (tests/test_gpu_ops.py, "
          "tests/test_gpu_configs.py).  `1x1+dw`: MT_SCHED_FUSE_EXPAND, `dw+1x1`: MT_SCHED_FUSE_DEPTHWISE, `conv+pool`: "
          "MT_SCHED_FUSE_POOL; `fused` = operators that ran inside a neighbour's launch.")
    print()
    print("## Every tenant alone (sequential schedule of one tenant)")
    print()
    print("| tenant | operators | plain | 1x1+dw | fused | dw+1x1 | fused | conv+pool | fused | 1x1+dw and conv+pool |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    all_specs = cfg.models()
    for which, spec in enumerate(all_specs):
        ctx = api.Context(0)
        model = api.Model(spec, weights.make_params(spec, cfg.seed, which))
        ctx.register(model)
        model.close()
        inputs = [ctx.make_input(0, weights.make_input(spec, cfg.seed, which, cfg.input_dist))]
        outputs = [ctx.make_output(0)]
        row = []
        for fl in (0, FE, FD, FP, FE | FP):
            sched = ctx.sequential(flags=fl)
            r = _time(ctx, sched, inputs, outputs, steps=60, warmup=8)
            row.append((r["median"], ctx.run(sched, inputs, outputs)["n_fused"]))
        print("| %s | %d | %.4f | %.4f | %d | %.4f | %d | %.4f | %d | %.4f |" % (
            spec.name, ctx.lens()[0], row[0][0], row[1][0], row[1][1], row[2][0], row[2][1], row[3][0], row[3][1], row[4][0]))
        sys.stdout.flush()
        ctx.close()
    print()
    print("## All tenants concurrent (one stage, one issuing thread per stream, no CU masks)")
    print()
    ctx, specs, inputs, outputs = _setup(cfg)
    n = len(specs)
    PI = B.MT_SCHED_PARALLEL_ISSUE
    print("| launches | wave priority per tenant | makespan | min | p90 |")
    print("|---|---|---|---|---|")
    rows = [("plain", 0, [0] * n), ("fused", FE | FP, [0] * n), ("fused", FE | FP, [-1] * n)]
    rows += [("fused", FE | FP, [3 if j == i else 0 for j in range(n)]) for i in range(n)]
    for label, fl, pr in rows:
        sched = ctx.schedule([[] for _ in specs], 1, flags=fl | PI, wave_priority=pr)
        r = _time(ctx, sched, inputs, outputs, steps=60, warmup=8)
        print("| %s | %s | %.4f | %.4f | %.4f |" % (label, "/".join(str(v) for v in pr), r["median"], r["min"], r["p90"]))
        sys.stdout.flush()
    print()
    print("Priority -1 = 3 for the tenant's short kernels and 0 for the others; tenants in the order %s." % ", ".join(s.name for s in specs))
    ctx.close()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["search", "issue", "mixes", "fusion"])
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--candidates", type=int, default=8)
    ap.add_argument("--runs", type=int, default=7)
    ap.add_argument("--seeds", type=int, default=5)
    ap.add_argument("--only", default="", help="mixes: comma-separated subset of the mix names")
    args = ap.parse_args()
    {"search": report_search, "issue": report_issue, "mixes": report_mixes, "fusion": report_fusion}[args.what](args)


if __name__ == "__main__":
    main()
