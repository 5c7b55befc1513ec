"""Reports on the scheduling layer, measured on the GPU: markdown on stdout.

  search   best-so-far latency against evaluations for coordinate descent and random search, and the wall time of
           the search (the analogues of the paper's search-curve figure and search-overhead table, Sec. IV)
  issue    breadth-first against depth-first issue of the same schedules, with the host issue time and the stall of
           every stream behind the main thread (Sec. III-D), and the same schedules replayed as a device graph
  mixes    sequential, all-concurrent and searched latency of the paper's tenant combinations (Tables I-II)
  fusion   every tenant alone and all tenants together, with and without the fused launches of neighbouring operators
           and with wave priorities (the runtime's additions to the paper's method)

  barriers what a stage barrier costs (Sec. III-B "Stage"): the probe of mt_probe_barrier_cost for 1..8 streams and
           even-split staged schedules of a workload under the event, counter and host-side barriers
  layers   per-operator table of one tenant: GEMM shape, kernel, time alone on the GPU, fraction of its own roofline bound
  streams  which streams can run side by side (mt_probe_stream_conflicts: the dispatch pipes), and a workload in one
           stage on 1 .. n streams, with the tenants that share a stream issued one after the other or co-issued
  benchsum markdown table of bench.py outputs (all schedules and kernel families of each workload)
  rocprof  turns the CSV files of `rocprofv3 --kernel-trace --stats` / `--pmc ...` runs of `bench.py --roofline-only`
           into the per-family summary kept under profiles/

    python -m paper_2111_14255_amd.report search --config cfg2
    python -m paper_2111_14255_amd.report issue --config cfg2
    python -m paper_2111_14255_amd.report mixes
    python -m paper_2111_14255_amd.report fusion --config cfg2
    python -m paper_2111_14255_amd.report barriers --config cfg3
    python -m paper_2111_14255_amd.report layers --config cfg5 --tenant 0
    python -m paper_2111_14255_amd.report streams --config cfg5
    python -m paper_2111_14255_amd.report rocprof --config cfg5 --dir <directory with the rocprofv3 output>
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


def report_streams(args):
    import ctypes as C
    import hashlib
    from synth import configs
    from . import binding as B
    cfg = configs.ALL[args.config]
    ctx, specs, inputs, outputs = _setup(cfg)
    n = len(specs)
    print("# Streams that run side by side, stream counts and co-issue, workload %s (%s), MI355X" % (cfg.name, " + ".join(cfg.tenants)))
    print()
    print("Command: `python -m paper_2111_14255_amd.report streams --config %s`" % args.config)
    print()
    print("## Pairs of new streams (`mt_probe_stream_conflicts`)")
    print()
    print("Twelve new unmasked streams; every cell: us per round of 16 rounds in which the two streams launch one one-workgroup "
          "kernel each, every stream recording its own end and the host waiting (the diagonal: the stream alone).  A pair at "
          "twice the single figure is served one stream at a time: the two sit on the same dispatch pipe.  The library "
          "classifies its tenant streams this way when it creates them and gives tenant index i a stream of class i % 4.")
    print()
    m = 12
    single = (C.c_float * m)()
    pair = (C.c_float * (m * m))()
    B.check(ctx.lib.mt_probe_stream_conflicts(ctx.h, m, 16, single, pair))
    lo = min(single)
    cls = []
    for i in range(m):                      # classes by the first earlier stream this one conflicts with
        k = next((cls[j] for j in range(i) if pair[i * m + j] > 1.5 * lo), None)
        cls.append(max(cls) + 1 if k is None and cls else (0 if k is None else k))
    print("| stream | class | " + " | ".join(str(j) for j in range(m)) + " |")
    print("|---|---|" + "---|" * m)
    for i in range(m):
        print("| %d | %d | " % (i, cls[i]) + " | ".join("%.1f" % pair[i * m + j] for j in range(m)) + " |")
    print()
    print("Classes found: %d, sizes %s." % (max(cls) + 1, " / ".join(str(cls.count(k)) for k in range(max(cls) + 1))))
    print()
    print("## One stage on c streams, tenants of a stream one after the other or co-issued")
    print()
    print("Median makespan of 30 runs, ms; one issuing host thread per stream.  Co-issue (`MT_SCHED_COISSUE`): two tenants of "
          "equal architecture on one stream run operator i of both as one launch.  `inside` = operators that ran inside a "
          "mate's launch, of %d.  The last column: md5 of all tenants' output bits, which must not change along a row or a column." % sum(ctx.lens()))
    print()
    print("| streams | one after the other | co-issued | inside | ratio | output bits |")
    print("|---|---|---|---|---|---|")
    FL = B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER
    import torch
    for c in [v for v in (1, 2, 3, 4, 5, 6, 8) if v <= n]:
        row, digests, inside = [], set(), 0
        for flags in (FL, FL | B.MT_SCHED_COISSUE):
            sched = ctx.schedule([[] for _ in specs], 1, concurrency=[c], flags=flags)
            for o in outputs:
                o.zero_()
            r = _time(ctx, sched, inputs, outputs, steps=30)
            torch.cuda.synchronize()
            digests.add(hashlib.md5(b"".join(ctx.output_to_numpy(t, outputs[t]).tobytes() for t in range(n))).hexdigest()[:8])
            inside = ctx.run(sched, inputs, outputs)["n_fused"]
            row.append(r["median"])
            sched.close()
        print("| %d | %.3f | %.3f | %d | %.2f | %s |" % (c, row[0], row[1], inside, row[0] / row[1], " / ".join(sorted(digests))))
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


def _even(lens, n_stages):
    P = n_stages - 1
    return [[-(-n * (j + 1) // (P + 1)) for j in range(P)] for n in lens]


def report_barriers(args):
    import ctypes as C
    from synth import configs
    from . import binding as B
    cfg = configs.ALL[args.config]
    ctx, specs, inputs, outputs = _setup(cfg)
    print("# Cost of a stage barrier on MI355X (Sec. III-B \"Stage\")")
    print()
    print("Command: `python -m paper_2111_14255_amd.report barriers --config %s`" % cfg.name)
    print()
    print("## Probe: rounds of one short kernel per stream, a barrier between rounds (`mt_probe_barrier_cost`, 200 rounds, best of 3)")
    print()
    print("us per round; the barrier's cost is the difference to the first column.  events = every stream records an event and "
          "waits for the events of all others (n + n(n-1) runtime calls); memory ops = every stream writes a word of its own and "
          "waits for the words of all others; counter = a one-thread kernel per stream adds 1 to one word, every stream waits once "
          "for the total (2n calls); via main = events through the main stream (3n + 1 calls).  One issuing host thread: with "
          "three streams and more a round is bound by the runtime calls themselves.")
    print()
    print("| streams | no barrier | events | memory ops | counter | via main |")
    print("|---|---|---|---|---|---|")
    for n in (1, 2, 3, 4, 5, 8):
        row = []
        for kind in range(5):
            best = 1e30
            for _ in range(3):
                v = C.c_float()
                B.check(ctx.lib.mt_probe_barrier_cost(ctx.h, n, kind, 200, C.byref(v)))
                best = min(best, v.value)
            row.append(best)
        print("| %d | %.1f | %.1f | %.1f | %.1f | %.1f |" % (n, *row))
        sys.stdout.flush()
    lens = ctx.lens()
    print()
    print("## %s (%s, batch %d, %s): even split into 1 / 2 / 4 / 8 stages, median makespan of 21 runs, ms" % (
        cfg.name, " + ".join(cfg.tenants), cfg.batch, cfg.dtype))
    print()
    print("main thread = the paper's single issuing thread (Sec. III-D); threads = one issuing host thread per stream; host = the "
          "issuing thread of a stream waits on the host for the events of the stage before.  Outputs are bit-identical in every cell.")
    print()
    PI = B.MT_SCHED_PARALLEL_ISSUE
    forms = (("events, main thread", 0), ("counter, main thread", B.MT_SCHED_COUNTER_BARRIER), ("events, threads", PI),
             ("counter, threads", PI | B.MT_SCHED_COUNTER_BARRIER), ("host, threads", PI | B.MT_SCHED_HOST_BARRIER))
    print("| stages | " + " | ".join(f[0] for f in forms) + " |")
    print("|---|" + "---|" * len(forms))
    for ns in (1, 2, 4, 8):
        row = []
        for _, flags in forms:
            sc = ctx.schedule(_even(lens, ns), ns, flags=flags)
            row.append(_time(ctx, sc, inputs, outputs, steps=21, warmup=3)["median"])
            sc.close()
        print("| %d | " % ns + " | ".join("%.4f" % v for v in row) + " |")
        sys.stdout.flush()
    ctx.close()


def report_layers(args):
    from synth import configs
    from . import binding as B
    cfg = configs.ALL[args.config]
    ctx, specs, inputs, outputs = _setup(cfg)
    t = args.tenant
    m = specs[t]
    best = None
    for _ in range(3):
        ms = ctx.profile_ops(t, inputs[t], outputs[t], 20)
        best = ms if best is None else [min(a, b) for a, b in zip(best, ms)]
    print("# Per-operator pass of %s (tenant %d of %s, batch %d, %s) alone on MI355X" % (m.name, t, cfg.name, m.batch, m.dtype))
    print()
    print("Command: `python -m paper_2111_14255_amd.report layers --config %s --tenant %d`" % (cfg.name, t))
    print()
    print("Every operator 1 + 20 times back to back on one stream between two events (`mt_profile_ops`), best of 3 passes.  M x N x K = "
          "pixels x output channels x reduction length; bound = max(flops / 2.5 PFLOP/s, bytes / 8 TB/s) of the operator's algorithmic "
          "work; an empty dependent launch takes about 3.5 us on this machine, which a single short kernel cannot go below.")
    print()
    print("| op | kind | M | N | K | window | kernel | split | workgroups | us | bound us | frac | TFLOP/s | GB/s |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    tot = totb = 0.0
    fam = {}
    for i, (op, d) in enumerate(zip(m.ops, best)):
        info = ctx.op_info(t, i)
        M = m.batch * info.out_h * info.out_w
        K = op.r * op.s * (info.in_c // max(1, op.groups)) if op.kind in ("conv", "fc") else op.r * op.s
        us = d * 1e3
        bound = max(info.flops / 2.5e15, info.bytes / 8e12) * 1e6
        kn = B.load().mt_kernel_name(info.kernel_id).decode()
        print("| %d | %s | %d | %d | %d | %dx%d s%d | %s | %d | %d | %.2f | %.2f | %.3f | %.1f | %.0f |" % (
            i, op.kind, M, info.out_c, K, op.r, op.s, op.stride_h, kn, info.split_k, info.grid_blocks, us, bound, bound / us,
            info.flops / (d * 1e-3) / 1e12, info.bytes / (d * 1e-3) / 1e9))
        tot += us
        totb += bound
        f = fam.setdefault(kn, [0, 0.0, 0.0])
        f[0] += 1
        f[1] += us
        f[2] += bound
    print()
    print("Sum of the operator times %.1f us, sum of their bounds %.1f us (%.3f)." % (tot, totb, totb / tot))
    print()
    print("| family | launches | us | bound us | frac |")
    print("|---|---|---|---|---|")
    for k, v in sorted(fam.items(), key=lambda kv: -kv[1][1]):
        print("| %s | %d | %.1f | %.1f | %.3f |" % (k, v[0], v[1], v[2], v[2] / v[1]))
    ctx.close()


def _family_of(kernel_name):
    import re
    m = re.search(r"igemm_kernel<[^,]+, (\d+), (\d+)", kernel_name) or re.match(r"_ZN2mt12igemm_kernelI(?:DF16_|NS_4bf16E)Li(\d+)ELi(\d+)E", kernel_name)
    if m:
        return "igemm_%sx%s" % (m.group(1), m.group(2))
    for key, fam in (("stem_kernel", "stem_rows"), ("rowb_kernel", "igemm_resident_filters"), ("rowp_kernel", "igemm_resident_filters"), ("pconv_kernel", "igemm_patch_64x64"), ("pw_direct_kernel", "igemm_pointwise"), ("gemv_kernel", "gemv"), ("dwconv", "dwconv"), ("gap_kernel", "global_avgpool"),
                     ("pool", "pool"), ("conv_direct", "conv_direct"), ("lrn_kernel", "lrn"), ("add_kernel", "add")):
        if key in kernel_name:
            return fam
    return None


def report_rocprof(args):
    """Reads <dir>/live.json (stdout of `bench.py --roofline-only`), <dir>/trace/*kernel_stats.csv and the
    *counter_collection.csv files of the --pmc runs under <dir>/pmc_*/ ; prints the summary and, with --traffic-out,
    writes the per-family HBM bytes that bench.py reports as roofline.traffic."""
    import collections
    import csv
    import glob
    import json
    import os
    d = args.dir
    live = json.load(open(os.path.join(d, "live.json")))["families"]
    print("# Kernel time, HBM traffic and unit utilisation of the per-operator pass, workload %s (MI355X)" % args.config)
    print()
    print("Commands (run from /tmp on the MI355X box, repository root = $R; every --pmc set is a run of its own):")
    print()
    print("    python3 $R/bench.py --config %s --roofline-only > live.json" % args.config)
    print("    rocprofv3 --kernel-trace --stats -d trace -o roof --output-format csv -- python3 $R/bench.py --config %s --roofline-only" % args.config)
    for name in sorted(os.path.basename(x) for x in glob.glob(os.path.join(d, "pmc_*")) if os.path.isdir(x)):
        cs = set()
        for f in glob.glob(os.path.join(d, name, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                cs.add(r["Counter_Name"])
        print("    rocprofv3 --pmc %s -d %s -o p --output-format csv -- python3 $R/bench.py --config %s --roofline-only" % (" ".join(sorted(cs)), name, args.config))
    print("    python -m paper_2111_14255_amd.report rocprof --config %s --dir <the directory holding the above>" % args.config)
    print()
    print("`bench.py --roofline-only` launches every operator of every tenant 11 times back to back on one stream (1 warm-up + 10 timed), "
          "after a 64 MiB elementwise copy that calibrates the byte counters.")
    print()
    stats = []
    for f in glob.glob(os.path.join(d, "trace", "**", "*kernel_stats.csv"), recursive=True):
        stats = list(csv.DictReader(open(f)))
    fam = collections.defaultdict(lambda: [0, 0.0])
    print("## rocprofv3 --kernel-trace --stats (top kernels)")
    print()
    print("| kernel | calls | total us | avg us | % |")
    print("|---|---|---|---|---|")
    for r in stats[:12]:
        print("| %s | %s | %.1f | %.2f | %s |" % (r["Name"][:90], r["Calls"], float(r["TotalDurationNs"]) / 1e3, float(r["AverageNs"]) / 1e3, r["Percentage"]))
    for r in stats:
        k = _family_of(r["Name"])
        if k:
            fam[k][0] += int(r["Calls"])
            fam[k][1] += float(r["TotalDurationNs"]) / 1e3
    print()
    print("| family | launches per pass | rocprofv3 avg us (all 11 launches of every operator) | bench.py HIP events avg us (the 10 timed ones) |")
    print("|---|---|---|---|")
    for k, v in live.items():
        kk = "pool" if k in ("maxpool", "avgpool") else k
        if kk in fam and fam[kk][0]:
            print("| %s | %d | %.2f | %.2f |" % (k, v["launches"], fam[kk][1] / fam[kk][0], v["ms"] * 1e3 / v["launches"]))
    # counters: mean per dispatch and family
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    cal = collections.defaultdict(list)
    for f in glob.glob(os.path.join(d, "pmc_*", "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            k = _family_of(r["Kernel_Name"])
            if k:
                per[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
            if "elementwise" in r["Kernel_Name"] and int(r["Grid_Size"]) >= 32 * 1024 * 1024 // 8:
                cal[r["Counter_Name"]].append(float(r["Counter_Value"]))
    mean = lambda v: sum(v) / len(v) if v else 0.0
    traffic = {}
    if cal.get("FETCH_SIZE") and cal.get("WRITE_SIZE"):
        fs, ws = 65536.0 / max(cal["FETCH_SIZE"]), 65536.0 / max(cal["WRITE_SIZE"])
        print()
        print("## HBM traffic (FETCH_SIZE / WRITE_SIZE, KiB per dispatch, mean over the dispatches of a family)")
        print()
        print("Calibration: the 64 MiB copy (65536 KiB read, 65536 KiB written) reads FETCH_SIZE = %.1f and WRITE_SIZE = %.1f, so FETCH_SIZE "
              "is scaled by %.3f and WRITE_SIZE by %.3f." % (max(cal["FETCH_SIZE"]), max(cal["WRITE_SIZE"]), fs, ws))
        print()
        print("| family | dispatches | FETCH_SIZE | WRITE_SIZE | HBM bytes per launch (scaled) | algorithmic bytes per launch | ratio |")
        print("|---|---|---|---|---|---|---|")
        for k, v in live.items():
            kk = "pool" if k in ("maxpool", "avgpool") else k
            if "FETCH_SIZE" not in per[kk]:
                continue
            fm, wm = mean(per[kk]["FETCH_SIZE"]), mean(per[kk]["WRITE_SIZE"])
            hb = (fm * fs + wm * ws) * 1024
            alg = v["bytes"] / v["launches"]
            traffic[k] = {"hbm_bytes_per_launch": int(hb), "fetch_kib": round(fm, 1), "write_kib": round(wm, 1),
                          "fetch_scale": round(fs, 3), "write_scale": round(ws, 3)}
            print("| %s | %d | %.1f | %.1f | %d | %d | %.2f |" % (k, len(per[kk]["FETCH_SIZE"]), fm, wm, hb, alg, hb / alg))
    if any("SQ_VALU_MFMA_BUSY_CYCLES" in c for c in per.values()):
        print()
        print("## Unit utilisation from counters (sums over the dispatches of a family)")
        print()
        print("MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES): the share of the busy compute units' matrix-core "
              "cycles that executed a matrix instruction.  MFMA vs peak = the same cycles over (1024 SIMDs x GRBM_GUI_ACTIVE / 8 XCDs): "
              "against the whole chip for the whole launch.  LDS busy = SQ_LDS_IDX_ACTIVE / SQ_BUSY_CU_CYCLES, address unit busy = "
              "TA_TA_BUSY_sum / SQ_BUSY_CU_CYCLES, wait = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES (share of wave time spent waiting for "
              "any instruction's operands), L2 hit = TCC_HIT_sum / (TCC_HIT_sum + TCC_MISS_sum).  The time-derived figure beside them "
              "is algorithmic flops / duration / 2.5 PFLOP/s from bench.py's HIP events.  Counter runs slow the kernels down, so "
              "ratios of cycle counts are meaningful, absolute cycle counts are not.")
        print()
        print("| family | MFMA busy on busy units | MFMA vs chip peak (counters) | MFMA vs peak (time-derived) | LDS busy | address unit busy | wave wait share | L2 hit |")
        print("|---|---|---|---|---|---|---|---|")
        for k, v in live.items():
            kk = "pool" if k in ("maxpool", "avgpool") else k
            c = per[kk]
            if not c:
                continue
            sm = lambda n: sum(c.get(n, []))
            cu = sm("SQ_BUSY_CU_CYCLES")
            gui = sm("GRBM_GUI_ACTIVE")
            hit, miss = sm("TCC_HIT_sum"), sm("TCC_MISS_sum")
            td = v["flops"] / (v["ms"] * 1e-3) / 2.5e15 if v["ms"] > 0 else 0.0
            fmt = lambda a, b: "%.3f" % (a / b) if b else "-"
            print("| %s | %s | %s | %.4f | %s | %s | %s | %s |" % (
                k, fmt(sm("SQ_VALU_MFMA_BUSY_CYCLES"), 4 * cu), fmt(sm("SQ_VALU_MFMA_BUSY_CYCLES"), 1024 * gui / 8), td,
                fmt(sm("SQ_LDS_IDX_ACTIVE"), cu), fmt(sm("TA_TA_BUSY_sum"), cu), fmt(sm("SQ_WAIT_INST_ANY"), sm("SQ_WAVE_CYCLES")),
                fmt(hit, hit + miss)))
    if args.traffic_out and traffic:
        json.dump(traffic, open(args.traffic_out, "w"), indent=1)


def report_benchsum(args):
    """Markdown summary of bench.py JSON lines (one file per workload, given with --files a.json,b.json,...)."""
    import json
    print("# bench.py on one MI355X: the three schedules of every workload")
    print()
    print("Commands: `python bench.py` (cfg5, the headline) and `python bench.py --config cfg1|cfg2|cfg3|cfg4`; this table: "
          "`python -m paper_2111_14255_amd.report benchsum --files <their outputs>`.")
    print()
    print("Makespan = mean of the timed steps, ms; img/s from the host's clock around the timed steps.  Rows of one workload that "
          "share a suffix ran in the same mode: (none) = the headline mode (one issuing host thread per stream, host-side stage "
          "barriers, fused operator pairs; searched = pointers + streams in use + CU shares + wave priorities, leaders re-measured "
          "in a play-off), +main_thread = the paper's single issuing thread on plain streams (pointer search only), +graph = "
          "whole-schedule graph replay.  `one stage` = the searched pointer matrix puts every operator into stage 1.")
    print()
    for f in args.files.split(","):
        d = json.loads(open(f).read().strip().splitlines()[-1])
        cpu = d.get("cpu_baseline")
        print("## %s" % d["config"]["workload"])
        print()
        print("`value` %.0f img/s (%.4f ms per step), %.2fx sequential, %.2fx all-concurrent in the same mode; bounds of the pass: "
              "flops %.0f us, bytes %.0f us; makespan / bound %.3f%s." % (
                  d["value"], d["ms_per_step"], d["speedup_vs_sequential"], d["speedup_vs_all_concurrent"], d["bounds"]["flops_bound_us"],
                  d["bounds"]["bytes_bound_us"], d["bounds"]["makespan_frac_of_bound"],
                  "; CPU oracle %.2f img/s on %d threads (%s)" % (cpu["value"], cpu["cores"], cpu["sample"]) if cpu else ""))
        r = d["roofline"]
        print("Dominant kernel family %s: %s bound, %.1f %s = %.4f of the published peak (%.4f of the measured %s), %d launches per "
              "step of %.2f us, arithmetic intensity %.0f flop/B, measured HBM bytes per launch %s." % (
                  r["kernel"], r["bound"], r["achieved"], r["unit"], r["frac"], r["frac_of_measured_peak"] or 0.0,
                  json.dumps(r["measured_peaks"]), r["launches_per_step"], r["avg_launch_us"], r["arithmetic_intensity_flop_per_byte"] or 0.0,
                  r["traffic"]))
        print()
        print("| schedule | makespan ms | stdev | img/s | vs sequential | vs all-concurrent | host issue ms | searched result |")
        print("|---|---|---|---|---|---|---|---|")
        for k, v in d["schedules"].items():
            extra = ""
            if "pointers" in v:
                extra = "one stage" if v.get("one_stage_matrix") else "rho = %s" % json.dumps(v["pointers"])
                if "cu_share" in v:
                    extra += "; streams %d, shares %s, priorities %s" % (v["stage_concurrency"][0], json.dumps(v["cu_share"]), json.dumps(v["wave_priority"]))
                extra += "; search %.1f s" % v["search_seconds"]
            print("| %s | %.4f | %.4f | %.0f | %.2f | %.2f | %.3f | %s |" % (
                k, v["makespan_ms_mean"], v["makespan_ms_stdev"], v["img_per_s"], v["speedup_vs_sequential"], v["speedup_vs_all_concurrent"],
                v["host_issue_ms_mean"], extra))
        print()
        print("| kernel family | launches | us per step | TFLOP/s | GB/s | of MFMA peak | of HBM peak |")
        print("|---|---|---|---|---|---|---|")
        for k, v in sorted(r["families"].items(), key=lambda kv: -kv[1]["us"]):
            print("| %s | %d | %.1f | %.1f | %.0f | %.4f | %.4f |" % (k, v["launches"], v["us"], v["TFLOP/s"], v["GB/s"], v["frac_of_mfma_peak"], v["frac_of_hbm_peak"]))
        print()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["search", "issue", "mixes", "fusion", "barriers", "layers", "streams", "rocprof", "benchsum"])
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--candidates", type=int, default=8)
    ap.add_argument("--runs", type=int, default=7)
    ap.add_argument("--seeds", type=int, default=5)
    ap.add_argument("--only", default="", help="mixes: comma-separated subset of the mix names")
    ap.add_argument("--files", default="", help="benchsum: comma-separated bench.py outputs")
    ap.add_argument("--tenant", type=int, default=0, help="layers: which tenant of the workload")
    ap.add_argument("--dir", default="", help="rocprof: directory with live.json, trace/ and pmc_*/")
    ap.add_argument("--traffic-out", default="", help="rocprof: write the per-family HBM bytes here (profiles/traffic_<workload>.json)")
    args = ap.parse_args()
    {"search": report_search, "issue": report_issue, "mixes": report_mixes, "fusion": report_fusion, "barriers": report_barriers, "streams": report_streams,
     "layers": report_layers, "rocprof": report_rocprof, "benchsum": report_benchsum}[args.what](args)


if __name__ == "__main__":
    main()
