"""Co-issue on the GPU: up to four tenants that share a stream run operator i of all of them as one launch.  Outputs must have the
bits of the one-launch-per-operator schedule and match the oracle; tenants that cannot be paired must still run in order."""
import numpy as np
import pytest

from paper_2111_14255_amd import binding as B
from synth import GraphBuilder, zoo
from gpu_harness import Mix, assert_close

pytestmark = pytest.mark.gpu

CO = B.MT_SCHED_COISSUE
PAR = B.MT_SCHED_PARALLEL_ISSUE | B.MT_SCHED_HOST_BARRIER


def compare(mix, plain, scheds, dtype):
    ref, tm0 = mix.run(plain)
    assert tm0["n_fused"] == 0
    for t, m in enumerate(mix.specs):
        assert_close(ref[t], mix.oracle()[t], dtype, "plain tenant %d (%s)" % (t, m.name))
    fused = []
    for s in scheds:
        print("  schedule", s.label, flush=True)
        for _ in range(2):
            got, tm = mix.run(s)
            assert tm["n_launches"] == sum(mix.ctx.lens())
            for t in range(len(got)):
                assert np.array_equal(ref[t].view(np.uint32), got[t].view(np.uint32)), "%s tenant %d" % (s.label, t)
        fused.append(tm["n_fused"])
    return fused


def test_equal_tenants_are_paired_and_keep_their_bits():
    # four ResNet-50 with their own weights and inputs: every operator has a two-operator form
    print("case 4 x resnet50 batch 2 bf16", flush=True)
    mix = Mix([zoo.resnet50("bf16", 2) for _ in range(4)], seed=921)
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        two = [[lens[t] // 2] for t in range(4)]
        fused = compare(mix, ctx.schedule([[] for _ in lens], 1, concurrency=[2], label="two streams"),
                        [ctx.schedule([[] for _ in lens], 1, concurrency=[2], flags=CO, label="co-issue, two streams"),
                         ctx.schedule([[] for _ in lens], 1, concurrency=[2], flags=CO | PAR, label="co-issue, issuing threads"),
                         ctx.schedule([[] for _ in lens], 1, concurrency=[1], flags=CO, label="co-issue, one stream"),
                         ctx.schedule(two, 2, concurrency=[2, 2], flags=CO | PAR, label="co-issue, two stages"),
                         ctx.schedule([[] for _ in lens], 1, flags=CO, label="co-issue asked for, a stream per tenant")], "bf16")
        # two streams: two pairs of tenants, one of every two operators runs inside its mate's launch; one stream: the
        # four tenants form one group and three of every four operators do
        assert fused[0] == fused[1] == fused[3] == 2 * lens[0] and fused[2] == 3 * lens[0]
        assert fused[4] == 0                              # nothing shares a stream
        with pytest.raises(B.MtError):
            ctx.schedule([[] for _ in lens], 1, concurrency=[2], flags=CO | B.MT_SCHED_GRAPH)
    finally:
        mix.close()


def test_mixed_tenants_pair_where_they_can_and_stay_in_order_where_not():
    # ResNet-18 twice and MobileNetV2 twice on one stream: neighbours (0, 1) and (2, 3) are walked together; with the
    # fused pairs of one tenant (1x1 + depthwise, convolution + pooling) the operators of such a pair are not co-issued
    # and are launched one tenant after the other, inside the same walk
    print("case r18 r18 mbv2 mbv2 f16", flush=True)
    mix = Mix([zoo.resnet18("f16", 1), zoo.resnet18("f16", 1), zoo.BUILDERS["mobilenetv2"]("f16", 1), zoo.BUILDERS["mobilenetv2"]("f16", 1)], seed=922)
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        FE = B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_POOL
        fused = compare(mix, ctx.sequential(),
                        [ctx.schedule([[] for _ in lens], 1, concurrency=[1], flags=CO, label="co-issue, one stream"),
                         ctx.schedule([[] for _ in lens], 1, concurrency=[1], flags=CO | FE, label="co-issue and fused pairs"),
                         ctx.schedule([[] for _ in lens], 1, concurrency=[2], flags=CO | PAR, label="co-issue, unequal neighbours")], "f16")
        assert fused[0] == lens[0] + lens[2]              # every operator of tenants 1 and 3 runs inside its mate's launch
        assert fused[1] > 0
        assert fused[2] == 0                              # longest first puts a ResNet-18 beside a MobileNetV2: nothing to pair
    finally:
        mix.close()


def test_same_length_different_shapes_are_not_paired():
    def net(c):
        g = GraphBuilder("n%d" % c, "f16", 2, 12, 12, 16)
        t = g.conv(0, c, 3, pad=1, bn=True)
        t = g.conv(t, 32, 1, bn=True)
        t = g.gap(t)
        g.fc(t, 10)
        return g.done()
    print("case same length, different widths", flush=True)
    mix = Mix([net(32), net(64)], seed=923)
    try:
        ctx = mix.ctx
        fused = compare(mix, ctx.sequential(), [ctx.schedule([[], []], 1, concurrency=[1], flags=CO, label="co-issue")], "f16")
        # the convolutions differ in width; pooling and classifier are the same operator in both tenants
        assert fused == [2]
    finally:
        mix.close()


def test_coissued_split_layers_in_the_fixed_scratch_array():
    # both tenants' layers are split along the reduction: the pair's partial sums and arrival counters live side by
    # side, in the arenas (mt_run) or in the library's fixed array (mt_run_static_scratch)
    def net():
        g = GraphBuilder("small_split", "f16", 1, 7, 7, 256)
        t = g.conv(0, 256, 3, pad=1, bn=True)
        t = g.conv(t, 512, 3, pad=1, bn=True)
        t = g.gap(t)
        g.fc(t, 100)
        return g.done()
    print("case three split-K tenants", flush=True)
    mix = Mix([net(), net(), net()], seed=924)
    try:
        ctx = mix.ctx
        assert any(ctx.op_info(0, i).split_k > 1 for i in range(ctx.lens()[0]))
        s = ctx.schedule([[], [], []], 1, concurrency=[1], flags=CO, label="co-issue")
        fused = compare(mix, ctx.sequential(), [s], "f16")
        assert fused[0] == 2 * ctx.lens()[0]              # one group of three: two of every three operators
        ref, _ = mix.run(ctx.sequential())
        for _ in range(2):
            outs = [ctx.make_output(t) for t in range(3)]
            for o in outs:
                o.fill_(float("nan"))
            tm = ctx.run_static_scratch(s, mix.inputs, outs)
            assert tm["n_fused"] == fused[0]
            for t in range(3):
                np.testing.assert_array_equal(ctx.output_to_numpy(t, outs[t]), ref[t])
    finally:
        mix.close()


@pytest.mark.parametrize("arch,dtype", [("alexnet_published", "bf16"), ("inceptionv3", "bf16"), ("vgg16", "f16"), ("tinyD", "f16")])
def test_every_kernel_family_in_its_two_operator_form(arch, dtype):
    # grouped convolutions and normalisation (AlexNet as published), asymmetric windows, average pooling and concat
    # writes (Inception-v3), the weight-streaming classifier and the pooled epilogue (VGG-16), add and 5x5 depthwise (tinyD)
    print("case 2 x", arch, dtype, flush=True)
    mix = Mix([zoo.BUILDERS[arch](dtype, 1), zoo.BUILDERS[arch](dtype, 1)], seed=925)
    try:
        ctx = mix.ctx
        lens = ctx.lens()
        fused = compare(mix, ctx.sequential(),
                        [ctx.schedule([[], []], 1, concurrency=[1], flags=CO, label="co-issue"),
                         ctx.schedule([[], []], 1, concurrency=[1], flags=CO | B.MT_SCHED_FUSE_POOL | B.MT_SCHED_FUSE_EXPAND, label="co-issue and fused pairs"),
                         ctx.schedule([[lens[0] // 3, 2 * lens[0] // 3]] * 2, 3, concurrency=[1, 1, 1], flags=CO | PAR, label="co-issue, three stages")], dtype)
        assert 0 < fused[0] <= lens[0] and fused[2] == fused[0]
        print("  operators inside the mate's launch: %d of %d" % (fused[0], lens[0]), flush=True)
    finally:
        mix.close()
