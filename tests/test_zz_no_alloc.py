"""mt_run_static_scratch (the pass for callers that cannot allocate) against mt_run, through the C ABI, on the GPU."""
import numpy as np
import pytest

from paper_2111_14255_amd import binding as B
from synth import GraphBuilder, zoo
from gpu_harness import Mix, assert_close

pytestmark = pytest.mark.gpu


def small_split_model(dtype="f16"):
    """Two 3x3 layers on a 7x7 map and a classifier: every convolution is split along its reduction."""
    g = GraphBuilder("small_split", dtype, 1, 7, 7, 256)
    t = g.conv(0, 256, 3, pad=1, bn=True)
    t = g.conv(t, 512, 3, pad=1, bn=True, res=-1)
    t = g.gap(t)
    g.fc(t, 100)
    return g.done()


def both_ways(mix, sched):
    """Outputs of mt_run and of mt_run_static_scratch under the same schedule (output buffers poisoned before each)."""
    ref, _ = mix.run(sched)
    outs = [mix.ctx.make_output(t) for t in range(len(mix.specs))]
    for o in outs:
        o.fill_(float("nan"))
    tm = mix.ctx.run_static_scratch(sched, mix.inputs, outs)
    got = [mix.ctx.output_to_numpy(t, o) for t, o in enumerate(outs)]
    return ref, got, tm


def uses_split(mix):
    return any(mix.ctx.op_info(t, i).split_k > 1 and B.load().mt_kernel_name(mix.ctx.op_info(t, i).kernel_id) != b"igemm_pointwise"
               for t in range(len(mix.specs)) for i in range(mix.ctx.lens()[t]))


def test_static_scratch_pass_equals_mt_run_twice_in_a_row():
    # first call: two tenants with many split layers; second call, right after it: a smaller tenant set, so that the
    # array still holds the first call's partial sums and counter values where the second one works
    big = Mix([zoo.resnet18("f16", 1), zoo.BUILDERS["mobilenetv2"]("f16", 1)], seed=911)
    small = Mix([small_split_model()], seed=912)
    try:
        assert uses_split(big) and uses_split(small)
        sb = big.ctx.schedule([[9, 15], [20, 40]], 3)
        ss = small.ctx.sequential()
        ref_b, got_b, tm_b = both_ways(big, sb)
        ref_s, got_s, tm_s = both_ways(small, ss)
        for r, g in zip(ref_b + ref_s, got_b + got_s):
            assert np.isfinite(g).all()
            np.testing.assert_array_equal(g, r)                   # same kernels, same reduction order: same bits
        assert tm_b["n_launches"] == sum(big.ctx.lens()) and tm_b["makespan_ms"] > 0 and tm_s["makespan_ms"] > 0
        # and the pass is the forward pass: oracle parity of the small one
        for t, m in enumerate(small.specs):
            assert_close(got_s[t], small.oracle()[t], m.dtype, m.name)
        # once more in the other order, all-concurrent, with a fused-pair schedule on the big set
        ref_s2, got_s2, _ = both_ways(small, ss)
        sb2 = big.ctx.all_concurrent(flags=B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_POOL)
        ref_b2, got_b2, _ = both_ways(big, sb2)
        for r, g in zip(ref_s2 + ref_b2, got_s2 + got_b2):
            np.testing.assert_array_equal(g, r)
        for a, b in zip(ref_b, ref_b2):
            np.testing.assert_array_equal(a, b)
    finally:
        big.close()
        small.close()


def test_static_scratch_limits_and_flags():
    mix = Mix([zoo.BUILDERS["vgg16"]("f16", 1), zoo.resnet18("f16", 1)], seed=913)      # needs more than the array holds
    try:
        outs = [mix.ctx.make_output(t) for t in range(2)]
        s = mix.ctx.sequential()
        with pytest.raises(B.MtError) as ei:
            mix.ctx.run_static_scratch(s, mix.inputs, outs)
        assert ei.value.code == B.MT_ERR_OUT_OF_MEMORY and str(B.MT_STATIC_SCRATCH_BYTES) in str(ei.value)
        for flags in (B.MT_SCHED_GRAPH, B.MT_SCHED_PARALLEL_ISSUE, B.MT_SCHED_STREAM_GRAPHS):
            sg = mix.ctx.all_concurrent(flags=flags)
            with pytest.raises(B.MtError) as ei:
                mix.ctx.run_static_scratch(sg, mix.inputs, outs)
            assert ei.value.code == B.MT_ERR_INVALID_ARG
        mix.ctx.run(s, mix.inputs, outs)                          # the ordinary pass still works after the refusals
        assert np.isfinite(mix.ctx.output_to_numpy(0, outs[0])).all()
    finally:
        mix.close()
