"""End-to-end parity of the benchmark workloads on the GPU: every tenant's logits against the CPU oracle,
and bit-identical outputs across schedules (sequential, all-concurrent, staged, DFS issue, graph replay)."""
import numpy as np
import pytest

from synth import configs
from paper_2111_14255_amd import binding as B
from gpu_harness import Mix, assert_close

pytestmark = pytest.mark.gpu


def even_split(lens, n_stages):
    P = n_stages - 1
    return [[-(-n * (j + 1) // (P + 1)) for j in range(P)] for n in lens]


def check_config(name, extra_schedules=()):
    cfg = configs.ALL[name]
    print("config", name, flush=True)
    mix = Mix(cfg.models(), cfg.seed, cfg.input_dist)
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        scheds = [ctx.sequential(), ctx.all_concurrent(),
                  ctx.schedule(even_split(lens, cfg.n_stages), cfg.n_stages, label="even-split"),
                  ctx.schedule(even_split(lens, cfg.n_stages), cfg.n_stages, order=B.MT_ISSUE_DFS, label="even-split-dfs"),
                  ctx.schedule(even_split(lens, 2), 2, flags=B.MT_SCHED_GRAPH, label="graph"),
                  ctx.schedule(even_split(lens, cfg.n_stages), cfg.n_stages, flags=B.MT_SCHED_PARALLEL_ISSUE, label="parallel-issue"),
                  ctx.all_concurrent(flags=B.MT_SCHED_PARALLEL_ISSUE)]
        scheds += [f(ctx, lens) for f in extra_schedules]
        ref = mix.oracle()
        first = None
        for s in scheds:
            print("  schedule", s.label, flush=True)
            reps = 3 if s.label in ("graph", "parallel-issue") else 1
            for _ in range(reps):                      # a graph is replayed several times, each replay checked
                got, tm = mix.run(s)
                assert tm["n_launches"] == sum(lens)
                for t, m in enumerate(mix.specs):
                    assert_close(got[t], ref[t], cfg.dtype, "%s tenant %d (%s) %s" % (name, t, m.name, s.label))
                if first is None:
                    first = got
                else:
                    for t in range(len(got)):
                        assert np.array_equal(first[t].view(np.uint32), got[t].view(np.uint32)), \
                            "outputs differ between schedules: %s tenant %d" % (s.label, t)
        return mix
    except Exception:
        mix.close()
        raise


def test_cfg1_tiny_fp32():
    # the 2-stage interleave: stage 1 = A ops 1-4 + all of B, stage 2 = A ops 5-8 + all of C
    mix = check_config("cfg1", [lambda ctx, lens: ctx.schedule([[4], [5], [0]], 2, label="interleave")])
    try:
        # the number of streams in use per stage as a searched coordinate
        ctx = mix.ctx
        outs = [ctx.make_output(t) for t in range(3)]
        rho, cost, rec, conc = ctx.search(mix.inputs, outs, 2, rounds=1, candidates=2, runs=3, warmup=1, seed=5, search_concurrency=True)
        assert len(conc) == 2 and conc[0] == conc[1] and 2 <= conc[0] <= 3
        base, _ = mix.run(ctx.sequential())
        got, _ = mix.run(ctx.schedule(rho, 2, concurrency=conc))
        for t in range(3):
            assert np.array_equal(got[t].view(np.uint32), base[t].view(np.uint32))
    finally:
        mix.close()


def test_cfg2_r18_vgg16_mbv2_fp16():
    mix = check_config("cfg2", [
        lambda ctx, lens: ctx.schedule([[0, 0], [lens[1], lens[1]], [0, lens[2]]], 3, label="one-tenant-per-stage"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 4), 4, concurrency=[2, 1, 3, 2], label="mixed-concurrency"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 3), 3, cu_share=[64, 128, 64], label="cu-shares"),
        lambda ctx, lens: ctx.all_concurrent(flags=B.MT_SCHED_FUSE_DEPTHWISE),
        lambda ctx, lens: ctx.all_concurrent(flags=B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_POOL | B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_PRIORITIZE_SHORT),
        lambda ctx, lens: ctx.schedule(even_split(lens, 4), 4, cu_share=[64, 64, 128], flags=B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_DEPTHWISE, label="fused-pairs"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 2), 2, flags=B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_POOL | B.MT_SCHED_STREAM_GRAPHS, label="graph"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 3), 3, cu_share=[64, 128, 64], flags=B.MT_SCHED_STREAM_GRAPHS, label="graph"),
        lambda ctx, lens: ctx.schedule([[] for _ in lens], 1, flags=B.MT_SCHED_STREAM_GRAPHS | B.MT_SCHED_FUSE_DEPTHWISE, label="graph"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 3), 3, cu_share=[[64, 128, 64], [0, 0, 0], [128, 64, 64]], label="per-stage-shares"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 3), 3, cu_share=[[96, 96, 64], [64, 64, 128], [0, 224, 32]],
                                       flags=B.MT_SCHED_PARALLEL_ISSUE, label="parallel-issue"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 5), 5, concurrency=[3, 2, 3, 1, 3],
                                       flags=B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER | B.MT_SCHED_FUSE_EXPAND, label="parallel-issue"),
        lambda ctx, lens: ctx.schedule([[0, 0], [lens[1], lens[1]], [0, lens[2]]], 3, cu_share=[64, 128, 64],
                                       flags=B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER, label="parallel-issue"),
        # the stage barrier taken with a counter word and one wait per stream instead of events
        lambda ctx, lens: ctx.schedule(even_split(lens, 4), 4, flags=B.MT_SCHED_COUNTER_BARRIER, label="counter-barrier"),
        lambda ctx, lens: ctx.schedule([[0, 0], [lens[1], lens[1]], [0, lens[2]]], 3, concurrency=[2, 1, 3],
                                       flags=B.MT_SCHED_COUNTER_BARRIER | B.MT_SCHED_FUSE_EXPAND, label="counter-barrier-empty-slices"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 5), 5, cu_share=[64, 128, 64],
                                       flags=B.MT_SCHED_COUNTER_BARRIER | B.MT_SCHED_PARALLEL_ISSUE, label="parallel-issue"),
    ])
    mix.close()


def test_cfg4_unbalanced_bf16():
    mix = check_config("cfg4")
    mix.close()


def test_cfg3_batch8_fp16():
    mix = check_config("cfg3", [lambda ctx, lens: ctx.all_concurrent(flags=B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_POOL)])     # fused pairs at batch 8
    mix.close()


def test_cfg5_eight_resnet50_batch16_bf16_cu_masks():
    # 8 tenants on 8 disjoint 32-CU shares, 8 stages
    mix = check_config("cfg5", [lambda ctx, lens: ctx.schedule(even_split(lens, 8), 8, cu_share=[32] * 8, label="cu-shares-8x32")])
    mix.close()


def test_paper_mix_r18_r34_fp16_with_share_search_and_first_op_timing():
    # a tenant combination of the paper's tables (adds ResNet-34), plus the flags no other test covers
    mix = check_config("mix_r18_r34", [
        lambda ctx, lens: ctx.schedule(even_split(lens, 3), 3, flags=B.MT_SCHED_TIME_FIRST_OP, label="first-op-timing"),
        lambda ctx, lens: ctx.schedule(even_split(lens, 2), 2, cu_share=[96, 160], flags=B.MT_SCHED_PARALLEL_ISSUE, label="shares-parallel"),
    ])
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        s = ctx.schedule([[], []], 1, order=B.MT_ISSUE_DFS, flags=B.MT_SCHED_TIME_FIRST_OP)
        _, tm = mix.run(s)
        first = tm["first_op_done_ms"]
        assert 0 < first[0] < first[1] < tm["makespan_ms"]       # DFS: the second stream starts after the first is issued
        # per-tenant completion times: one tenant after the other when sequential, all within the makespan always
        for sched in (ctx.sequential(flags=B.MT_SCHED_TIME_TENANTS),
                      ctx.all_concurrent(flags=B.MT_SCHED_TIME_TENANTS | B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_FUSE_POOL),
                      ctx.schedule(even_split(lens, 3), 3, cu_share=[128, 128], flags=B.MT_SCHED_TIME_TENANTS)):
            _, tm = mix.run(sched)
            done = tm["tenant_done_ms"]
            assert all(0 < d <= tm["makespan_ms"] * 1.001 + 1e-3 for d in done), (sched.label, done, tm["makespan_ms"])
            assert max(done) >= 0.8 * tm["makespan_ms"]
            if sched.label == "sequential":
                assert done[0] < done[1]
        _, tm = mix.run(ctx.all_concurrent())
        assert tm["tenant_done_ms"] == [0.0, 0.0]
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, flags=B.MT_SCHED_TIME_TENANTS | B.MT_SCHED_GRAPH)
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, flags=B.MT_SCHED_HOST_BARRIER)              # needs one issuing thread per stream
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, flags=B.MT_SCHED_COUNTER_BARRIER | B.MT_SCHED_GRAPH)
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, flags=B.MT_SCHED_COUNTER_BARRIER | B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER)
        ref = mix.oracle()
        outs = [ctx.make_output(t) for t in range(2)]
        rho, cost, rec, shares = ctx.search(mix.inputs, outs, 3, rounds=1, candidates=3, runs=3, warmup=1, seed=9,
                                            cu_share_rounds=1)
        assert len(shares) == 2 and all(v == 0 or (v % 32 == 0 and 32 <= v <= 224) for v in shares)
        assert cost <= min(c for _, c in rec) * 1.15      # a masked winner is re-measured, the unmasked one is in the records
        got, _ = mix.run(ctx.schedule(rho, 3, cu_share=shares))
        for t in range(2):
            assert_close(got[t], ref[t], "f16", "searched schedule tenant %d" % t)
        # wave priorities: searched as the last coordinate set, and never change a bit
        rho2, cost2, rec2, prio = ctx.search(mix.inputs, outs, 2, rounds=1, candidates=2, runs=3, warmup=1, seed=9,
                                             flags=B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_FUSE_POOL, wave_priority_rounds=1)
        assert len(prio) == 2 and all(-1 <= v <= 3 for v in prio)
        base, _ = mix.run(ctx.sequential())
        for pr, fl in ((prio, B.MT_SCHED_PARALLEL_ISSUE), ([3, 0], 0), ([-1, 2], B.MT_SCHED_GRAPH), ([1, -1], B.MT_SCHED_STREAM_GRAPHS)):
            sp = ctx.schedule(rho2, 2, flags=fl, wave_priority=pr)
            for rep in range(2):
                got, _ = mix.run(sp)
                if rep == 0:
                    sp.set_wave_priority([2, 3])          # captured graphs are dropped and captured again
            for t in range(2):
                assert np.array_equal(got[t].view(np.uint32), base[t].view(np.uint32)), (pr, fl, t)
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, wave_priority=[4, 0])
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, cu_share=[4, 0])             # a share that cannot cover the 8 XCDs
        with pytest.raises(B.MtError):
            ctx.schedule([[], []], 1, flags=B.MT_SCHED_TIME_FIRST_OP | B.MT_SCHED_GRAPH)
    finally:
        mix.close()


@pytest.mark.parametrize("name", ["ops_f32", "ops_f16", "alexnet_published"])
def test_operator_set_completion_workloads(name):
    # grouped convolution, local response normalisation and a stand-alone add inside whole tenants
    mix = check_config(name)
    mix.close()


@pytest.mark.parametrize("name", ["mix_vgg_r18", "mix_r34_r50", "mix_r50_r101", "mix_vgg_r18_r50", "mix_r18_r34_r50", "mix_5"])
def test_paper_tenant_mixes(name):
    # the other tenant combinations of the paper's scalability tables (Tables I-II), the five-tenant one included
    mix = check_config(name)
    mix.close()


def test_random_search_on_the_gpu_returns_a_valid_schedule_with_the_same_bits():
    # Sec. IV-D's random search with the profiled makespan as cost, then a play-off over its records
    cfg = configs.ALL["cfg1"]
    mix = Mix(cfg.models(), cfg.seed, cfg.input_dist)
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        outs = [ctx.make_output(t) for t in range(3)]
        base, _ = mix.run(ctx.sequential())
        for playoff in (0, 3):
            rho, cost, rec = ctx.search(mix.inputs, outs, 3, rounds=2, candidates=3, runs=3, warmup=1, seed=17,
                                        algo=B.MT_SEARCH_RANDOM, seed_baselines=True, playoff_top=playoff, playoff_runs=5)
            assert len(rho) == 3 and all(len(r) == 2 and 0 <= r[0] <= r[1] <= n for r, n in zip(rho, lens))
            assert 2 <= len(rec) <= 2 * 3 * 3 + 2 and all(c > 0 for _, c in rec)         # infeasible draws are skipped
            assert rec[0][0] == [[n, n] for n in lens]                                  # the one-stage matrix is recorded first
            if playoff == 0:
                assert cost == min(c for _, c in rec) and (rho, cost) in [(r, c) for r, c in rec]
            else:
                assert rho in [r for r, _ in rec] and cost > 0
            got, tm = mix.run(ctx.schedule(rho, 3))
            assert tm["n_launches"] == sum(lens)
            for t in range(3):
                assert np.array_equal(got[t].view(np.uint32), base[t].view(np.uint32))
                assert_close(got[t], mix.oracle()[t], cfg.dtype, "random search tenant %d" % t)
    finally:
        mix.close()


def test_stored_record_memory_can_be_replayed_on_the_gpu(tmp_path):
    # the record memory D of a search (Alg. 1) written to a file, read back, and its leaders profiled again
    from paper_2111_14255_amd import api
    cfg = configs.ALL["cfg1"]
    mix = Mix(cfg.models(), cfg.seed, cfg.input_dist)
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        outs = [ctx.make_output(t) for t in range(3)]
        rho, cost, rec = ctx.search(mix.inputs, outs, 3, rounds=2, candidates=3, runs=3, warmup=1, seed=5)
        path = str(tmp_path / "d.json")
        api.save_records(path, lens, 3, rec, note="cfg1")
        lens2, n_stages2, rec2 = api.load_records(path)
        assert lens2 == lens and n_stages2 == 3 and rec2 == rec
        rho2, cost2, measured = ctx.replay_records(rec2, 3, mix.inputs, outs, top_k=3, runs=5)
        distinct = {tuple(tuple(r) for r in m) for m, _ in rec2}
        assert 1 <= measured <= min(3, len(distinct)) + 1
        assert rho2 in [r for r, _ in rec2] or rho2 == [[n, n] for n in lens]
        assert 0 < cost2 < 20 * cost
        got, _ = mix.run(ctx.schedule(rho2, 3))
        for t in range(3):
            assert_close(got[t], mix.oracle()[t], cfg.dtype, "replayed schedule tenant %d" % t)
    finally:
        mix.close()


def test_tenant_registered_after_a_parallel_issue_run():
    # the issuing thread added for a later tenant must wait for the next run instead of waking for the finished one
    from synth import weights
    from paper_2111_14255_amd import api
    cfg = configs.ALL["cfg1"]
    specs = cfg.models()
    ctx = api.Context(0)
    try:
        raws = [weights.make_params(m, cfg.seed, t) for t, m in enumerate(specs)]
        xs = [weights.make_input(m, cfg.seed, t, cfg.input_dist) for t, m in enumerate(specs)]
        from oracle import forward as OF
        refs = [OF.forward(m, OF.prepare_params(m, raw), x) for m, raw, x in zip(specs, raws, xs)]
        inputs, outs = [], []
        for k in range(3):
            model = api.Model(specs[k], raws[k])
            ctx.register(model)
            model.close()
            inputs.append(ctx.make_input(k, xs[k]))
            outs.append(ctx.make_output(k))
            for flags in (B.MT_SCHED_PARALLEL_ISSUE, B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER):
                s = ctx.schedule(even_split(ctx.lens(), 2), 2, flags=flags)
                for _ in range(3):
                    for o in outs:
                        o.fill_(float("nan"))
                    tm = ctx.run(s, inputs, outs)
                    assert tm["n_launches"] == sum(ctx.lens())
                    for t in range(k + 1):
                        assert_close(ctx.output_to_numpy(t, outs[t]), refs[t], cfg.dtype, "tenant %d of %d" % (t, k + 1))
                s.close()
    finally:
        ctx.close()
