"""Pins for the oracle's graph walker and the synthetic model zoo."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from synth import zoo, weights, GraphBuilder
from oracle import forward as F, ops

GMAC = {"resnet18": 1.814, "resnet34": 3.664, "resnet50": 4.089, "resnet101": 7.801, "vgg16": 15.470,
        "mobilenetv2": 0.301, "alexnet": 1.135, "inceptionv3": 5.713, "alexnet_published": 0.724}
NOPS = {"tinyA": 8, "tinyB": 5, "tinyC": 9, "resnet18": 23, "resnet50": 56, "resnet101": 107, "vgg16": 21,
        "mobilenetv2": 54, "alexnet": 11, "inceptionv3": 109, "alexnet_published": 13, "tinyD": 8, "resnet34": 39}


@pytest.mark.parametrize("name", sorted(GMAC))
def test_mac_totals(name):
    m = zoo.BUILDERS[name]("f16", 1)
    assert abs(m.macs() / 1e9 - GMAC[name]) < 6e-4
    assert zoo.BUILDERS[name]("f16", 8).macs() == 8 * m.macs()


@pytest.mark.parametrize("name", sorted(NOPS))
def test_op_counts_and_serial_order(name):
    m = zoo.BUILDERS[name]("f16", 1)
    assert len(m.ops) == NOPS[name]
    written = {0}
    for op in m.ops:
        assert op.in_tensor in written
        if op.res_tensor >= 0:
            assert op.res_tensor in written
        written.add(op.out_tensor)


def _sizes(m):
    out = []
    for op in m.ops:
        if not out or out[-1] != op.out_shape[0]:
            out.append(op.out_shape[0])
    return out


def test_spatial_size_chains():
    # the projection shortcut of a down-sampling block is serialised before the block's branch,
    # so compare the sizes at which each new resolution first appears
    first_seen = list(dict.fromkeys(_sizes(zoo.resnet50())))
    assert first_seen == [112, 56, 28, 14, 7, 1]
    assert list(dict.fromkeys(_sizes(zoo.resnet18()))) == [112, 56, 28, 14, 7, 1]
    v = [op.out_shape[0] for op in zoo.vgg16().ops if op.kind == "maxpool"]
    assert v == [112, 56, 28, 14, 7]
    a = [op.out_shape[0] for op in zoo.alexnet().ops][:8]
    assert a == [55, 27, 27, 13, 13, 13, 13, 6]
    inc = zoo.inception_v3()
    stem = [op.out_shape[0] for op in inc.ops[:7]]
    assert stem == [149, 147, 147, 73, 73, 71, 35]
    assert {op.out_shape[0] for op in inc.ops} == {149, 147, 73, 71, 35, 17, 8, 1}
    widths = sorted({inc_t for inc_t in (op.out_c_total for op in inc.ops) if inc_t})
    assert widths == [256, 288, 768, 1280, 2048]
    assert zoo.tiny_b().ops[-1].in_shape == (5, 5, 64)


def test_concat_channels_fully_covered():
    inc = zoo.inception_v3()
    cover = {}
    for op in inc.ops:
        if op.out_c_total:
            cover.setdefault(op.out_tensor, []).append((op.out_c_offset, op.out_c_offset + op.out_shape[2], op.out_c_total))
    assert len(cover) == 11
    for spans in cover.values():
        spans.sort()
        assert spans[0][0] == 0 and spans[-1][1] == spans[0][2]
        for a, b in zip(spans, spans[1:]):
            assert a[1] == b[0]


def _torch_forward(model, params, x):
    """The same graph through torch's float64 CPU operators (library routines)."""
    t = {0: torch.from_numpy(x).double().permute(0, 3, 1, 2)}
    for op, p in zip(model.ops, params):
        xin = t[op.in_tensor]
        st, pd, kk = (op.stride_h, op.stride_w), (op.pad_h, op.pad_w), (op.r, op.s)
        if op.kind == "conv":
            y = TF.conv2d(xin, torch.from_numpy(p[0]).double().permute(0, 3, 1, 2),
                          None if p[1] is None else torch.from_numpy(p[1]).double(), st, pd, 1, op.groups)
            if op.res_tensor >= 0:
                y = y + t[op.res_tensor][:, : y.shape[1]]
        elif op.kind == "dwconv":
            c = xin.shape[1]
            y = TF.conv2d(xin, torch.from_numpy(p[0]).double().reshape(c, 1, op.r, op.s),
                          None if p[1] is None else torch.from_numpy(p[1]).double(), st, pd, groups=c)
        elif op.kind == "maxpool":
            y = TF.max_pool2d(xin, kk, st, pd)
        elif op.kind == "avgpool":
            y = TF.avg_pool2d(xin, kk, st, pd, count_include_pad=False)
        elif op.kind == "gap":
            y = xin.mean(dim=(2, 3), keepdim=True)
        elif op.kind == "fc":
            flat = xin.permute(0, 2, 3, 1).reshape(xin.shape[0], -1)
            y = TF.linear(flat, torch.from_numpy(p[0]).double(), None if p[1] is None else torch.from_numpy(p[1]).double())
            y = y.reshape(y.shape[0], -1, 1, 1)
        elif op.kind == "lrn":
            y = TF.local_response_norm(xin, op.r, op.lrn_alpha * op.r, op.lrn_beta, op.lrn_k)   # torch divides alpha by the size
        elif op.kind == "add":
            y = xin + t[op.res_tensor]
        if op.act == "relu":
            y = y.clamp(min=0)
        elif op.act == "relu6":
            y = y.clamp(0, 6)
        if op.out_c_total:
            buf = t.get(op.out_tensor)
            if buf is None:
                buf = torch.zeros(y.shape[0], op.out_c_total, y.shape[2], y.shape[3], dtype=torch.float64)
            buf[:, op.out_c_offset: op.out_c_offset + y.shape[1]] = y
            y = buf
        t[op.out_tensor] = y
    last = t[model.ops[-1].out_tensor]
    return last.permute(0, 2, 3, 1).reshape(last.shape[0], -1).numpy()


def _mini_graph():
    """Residual block with projection shortcut, an inverted-residual block and a 3-branch concat."""
    g = GraphBuilder("mini", "f32", 2, 12, 10, 3)
    t = g.conv(0, 8, 3, stride=2, pad=1, bn=True)
    short = g.conv(t, 16, 1, act="none", bn=True)
    u = g.conv(t, 8, 3, pad=1, bn=True)
    t = g.conv(u, 16, 3, pad=1, bn=True, gain=0.25, res=short, act="relu")
    u = g.conv(t, 32, 1, act="relu6", bn=True)
    u = g.dwconv(u, 3, 1, 1, act="relu6", bn=True)
    t = g.conv(u, 16, 1, act="none", bn=True, res=t)
    d = g.new_tensor()
    g.conv(t, 8, 1, dst=d, c_off=0, c_tot=8 + 8 + 16)
    u = g.conv(t, 4, (1, 3), pad=(0, 1))
    g.conv(u, 8, (3, 1), pad=(1, 0), dst=d, c_off=8, c_tot=32)
    u = g.avgpool(t, 3, 1, 1)
    g.conv(u, 16, 1, dst=d, c_off=16, c_tot=32)
    t = g.maxpool(d, 3, 2, 1)
    t = g.gap(t)
    g.fc(t, 5)
    return g.done()


@pytest.mark.parametrize("builder", [zoo.tiny_a, zoo.tiny_b, zoo.tiny_c, zoo.tiny_d, _mini_graph])
def test_forward_matches_torch_composition(builder):
    m = builder() if builder is _mini_graph else builder("f32", 1)
    raw = weights.make_params(m, 7, 0)
    x = weights.make_input(m, 7, 0, "uniform")
    params = F.prepare_params(m, raw)
    y = F.forward(m, params, x)
    ref = _torch_forward(m, params, x)
    assert y.shape == ref.shape == (m.batch, m.out_features)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-5 * max(1.0, np.abs(ref).max()))


def test_low_precision_forward_close_to_fp32_and_representable():
    for dt, tol in (("f16", 2e-2), ("bf16", 8e-2)):
        m = _mini_graph()
        m.dtype = dt
        raw = weights.make_params(m, 9, 0)
        x = weights.make_input(m, 9, 0, "normal")
        y, tensors = F.forward(m, F.prepare_params(m, raw), x, keep=True)
        for v in tensors.values():
            np.testing.assert_array_equal(ops.round_array(v, dt), v)     # stored values are representable
        m32 = _mini_graph()
        y32 = F.forward(m32, F.prepare_params(m32, raw), x)
        assert np.abs(y - y32).max() <= tol * np.abs(y32).max()


def test_distinct_seeds_per_tenant():
    m = zoo.tiny_a()
    a = weights.make_params(m, 1, 0)[0]["w"]
    b = weights.make_params(m, 1, 1)[0]["w"]
    c = weights.make_params(m, 1, 0)[0]["w"]
    assert not np.array_equal(a, b) and np.array_equal(a, c)
    std = weights.make_params(zoo.vgg16(), 1, 0)[1]["w"].std()
    assert abs(std - np.sqrt(2 / (9 * 64))) < 0.01 * np.sqrt(2 / (9 * 64))


@pytest.mark.parametrize("name,dt", [("resnet50", "f16"), ("mobilenetv2", "f16"), ("inceptionv3", "bf16")])
def test_deep_models_stay_finite(name, dt):
    m = zoo.BUILDERS[name](dt, 1)
    raw = weights.make_params(m, 3, 0)
    y = F.forward(m, F.prepare_params(m, raw), weights.make_input(m, 3, 0, "normal"))
    assert np.isfinite(y).all() and 1e-3 < np.abs(y).max() < 1e3
