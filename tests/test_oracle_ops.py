"""Pins for the CPU oracle's operators: brute force, library routines, closed forms."""
import itertools
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import ops, fold


def rnd(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def brute_conv(x, w, stride, pad, groups=1):
    """Seven nested loops (n, k, p, q, c, r, s), float64, written independently of ops.c."""
    n_, h, wd, c_ = x.shape
    k_, r_, s_, cg = w.shape
    assert cg * groups == c_ and k_ % groups == 0
    p_ = (h + 2 * pad[0] - r_) // stride[0] + 1
    q_ = (wd + 2 * pad[1] - s_) // stride[1] + 1
    y = np.zeros((n_, p_, q_, k_), dtype=np.float64)
    kpg = k_ // groups
    for n in range(n_):
        for k in range(k_):
            g = k // kpg
            for p in range(p_):
                for q in range(q_):
                    acc = 0.0
                    for c in range(cg):
                        for r in range(r_):
                            for s in range(s_):
                                ih = p * stride[0] + r - pad[0]
                                iw = q * stride[1] + s - pad[1]
                                if 0 <= ih < h and 0 <= iw < wd:
                                    acc += float(x[n, ih, iw, g * cg + c]) * float(w[k, r, s, c])
                    y[n, p, q, k] = acc
    return y


CONV_CASES = [
    # n, h, w, c, k, r, s, stride, pad
    (1, 5, 5, 3, 4, 3, 3, (1, 1), (1, 1)),
    (2, 7, 6, 3, 5, 3, 3, (2, 2), (1, 1)),
    (1, 9, 9, 2, 3, 5, 5, (1, 1), (2, 2)),
    (1, 11, 13, 3, 2, 7, 7, (2, 2), (3, 3)),
    (1, 15, 15, 3, 2, 11, 11, (4, 4), (0, 0)),
    (1, 6, 8, 4, 3, 1, 7, (1, 1), (0, 3)),
    (1, 8, 6, 4, 3, 7, 1, (1, 1), (3, 0)),
    (1, 5, 5, 2, 3, 1, 3, (1, 1), (0, 1)),
    (1, 5, 5, 2, 3, 3, 1, (1, 1), (1, 0)),
    (2, 4, 4, 8, 6, 1, 1, (1, 1), (0, 0)),
    (1, 7, 7, 5, 4, 1, 1, (2, 2), (0, 0)),
    (1, 6, 5, 3, 2, 3, 2, (2, 1), (1, 0)),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_brute_force_and_torch(case):
    n, h, w, c, k, r, s, st, pd = case
    x = rnd((n, h, w, c), 1)
    wt = rnd((k, r, s, c), 2)
    y = ops.conv(x, wt, None, st, pd, "none", None, "f32")
    ref = brute_conv(x, wt, st, pd)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-6 * max(1.0, np.abs(ref).max()))
    t = TF.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                  torch.from_numpy(wt).double().permute(0, 3, 1, 2), stride=st, padding=pd)
    np.testing.assert_allclose(y, t.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-6 * max(1.0, np.abs(ref).max()))


@pytest.mark.parametrize("st,pd,r", [((1, 1), (1, 1), 3), ((2, 2), (1, 1), 3), ((1, 1), (0, 0), 3), ((2, 2), (2, 2), 5)])
def test_dwconv_matches_grouped_brute_force_and_torch(st, pd, r):
    c = 5
    x = rnd((2, 7, 6, c), 3)
    wt = rnd((c, r, r), 4)
    b = rnd((c,), 5)
    y = ops.dwconv(x, wt, b, st, pd, "none", "f32")
    ref = brute_conv(x, wt.reshape(c, r, r, 1), st, pd, groups=c) + b.astype(np.float64)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-6)
    t = TF.conv2d(torch.from_numpy(x).double().permute(0, 3, 1, 2),
                  torch.from_numpy(wt).double().reshape(c, 1, r, r), torch.from_numpy(b).double(),
                  stride=st, padding=pd, groups=c)
    np.testing.assert_allclose(y, t.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-6)


def test_conv_identity_closed_forms():
    x = rnd((1, 6, 7, 4), 6)
    eye = np.eye(4, dtype=np.float32).reshape(4, 1, 1, 4)
    np.testing.assert_array_equal(ops.conv(x, eye), x)
    # centre-tap delta kernel of a 3x3, pad 1 => identity
    w = np.zeros((4, 3, 3, 4), dtype=np.float32)
    for k in range(4):
        w[k, 1, 1, k] = 1.0
    np.testing.assert_array_equal(ops.conv(x, w, pad=(1, 1)), x)
    # off-centre tap shifts the image: pins the sign convention ih = p*stride - pad + r
    w2 = np.zeros((4, 3, 3, 4), dtype=np.float32)
    for k in range(4):
        w2[k, 0, 2, k] = 1.0          # r=0, s=2 : reads (p-1, q+1)
    y = ops.conv(x, w2, pad=(1, 1))
    np.testing.assert_array_equal(y[0, 1:, :-1], x[0, :-1, 1:])
    assert np.all(y[0, 0] == 0) and np.all(y[0, :, -1] == 0)


@pytest.mark.parametrize("r,s,c,pad", [(3, 3, 3, 0), (5, 5, 2, 0), (3, 3, 4, 1), (1, 7, 2, 3), (7, 1, 2, 3)])
def test_conv_all_ones_counts_taps(r, s, c, pad):
    ph, pw = (pad if r > 1 else 0), (pad if s > 1 else 0)
    h, w = 9, 8
    x = np.ones((1, h, w, c), dtype=np.float32)
    wt = np.ones((2, r, s, c), dtype=np.float32)
    y = ops.conv(x, wt, pad=(ph, pw))
    for p, q in itertools.product(range(y.shape[1]), range(y.shape[2])):
        rows = sum(1 for i in range(r) if 0 <= p - ph + i < h)
        cols = sum(1 for j in range(s) if 0 <= q - pw + j < w)
        assert y[0, p, q, 0] == rows * cols * c
    if ph == 0 and pw == 0:
        assert np.all(y == r * s * c)


def test_conv_bias_residual_activation_order():
    x = rnd((1, 4, 4, 3), 7)
    w = np.zeros((2, 3, 3, 3), dtype=np.float32)
    b = np.array([0.5, -0.25], dtype=np.float32)
    res = rnd((1, 4, 4, 2), 8)
    y = ops.conv(x, w, b, pad=(1, 1), act="relu", res=res)
    np.testing.assert_array_equal(y, np.maximum(res + b, 0).astype(np.float32))
    y6 = ops.conv(x, w, b * 40, pad=(1, 1), act="relu6", res=res)
    np.testing.assert_array_equal(y6, np.clip(res.astype(np.float64) + (b * 40), 0, 6).astype(np.float32))
    # residual read from a wider tensor uses that tensor's channel stride
    wide = rnd((1, 4, 4, 5), 9)
    yw = ops.conv(x, w, None, pad=(1, 1), res=wide)
    np.testing.assert_array_equal(yw, wide[..., :2])


def test_channel_offset_write_leaves_other_channels():
    x = rnd((1, 4, 4, 3), 10)
    w = rnd((2, 1, 1, 3), 11)
    y = np.full((1, 4, 4, 6), 7.0, dtype=np.float32)
    ops.conv(x, w, y=y, c_off=3, c_tot=6)
    np.testing.assert_array_equal(y[..., 3:5], ops.conv(x, w))
    assert np.all(y[..., :3] == 7.0) and np.all(y[..., 5] == 7.0)
    ops.maxpool(rnd((1, 8, 8, 2), 12), (2, 2), (2, 2), y=y, c_off=0, c_tot=6)
    assert np.all(y[..., 2] == 7.0)


def test_pools_closed_forms_and_torch():
    ones = np.ones((2, 7, 7, 3), dtype=np.float32)
    assert np.all(ops.maxpool(ones, (3, 3), (2, 2), (1, 1)) == 1)
    assert np.all(ops.avgpool(ones, (3, 3), (1, 1), (1, 1)) == 1)      # in-bounds divisor
    assert np.all(ops.global_avgpool(ones) == 1)
    ramp = np.arange(6 * 6, dtype=np.float32).reshape(1, 6, 6, 1)
    mp = ops.maxpool(ramp, (2, 2), (2, 2))
    assert mp.shape == (1, 3, 3, 1)
    for p, q in itertools.product(range(3), range(3)):
        assert mp[0, p, q, 0] == (2 * p + 1) * 6 + 2 * q + 1
    assert ops.global_avgpool(ramp)[0, 0, 0, 0] == 17.5
    # negative inputs with padding: padding must never win the max
    neg = -np.abs(rnd((1, 5, 5, 2), 13)) - 1
    y = ops.maxpool(neg, (3, 3), (2, 2), (1, 1))
    assert np.all(y < 0)
    x = rnd((2, 9, 8, 3), 14)
    xt = torch.from_numpy(x).double().permute(0, 3, 1, 2)
    for k, s, p in [((2, 2), (2, 2), (0, 0)), ((3, 3), (2, 2), (0, 0)), ((3, 3), (2, 2), (1, 1))]:
        t = TF.max_pool2d(xt, k, s, p).permute(0, 2, 3, 1).numpy()
        np.testing.assert_array_equal(ops.maxpool(x, k, s, p), t.astype(np.float32))
    t = TF.avg_pool2d(xt, 3, 1, 1, count_include_pad=False).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(ops.avgpool(x, (3, 3), (1, 1), (1, 1)), t, rtol=0, atol=1e-6)
    np.testing.assert_allclose(ops.global_avgpool(x)[:, 0, 0, :], x.astype(np.float64).mean(axis=(1, 2)), atol=1e-6)


def test_fc_pins():
    x = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32).reshape(2, 1, 1, 3)
    w = np.array([[1, 0, -1], [0.5, 0.5, 0.5]], dtype=np.float32)
    b = np.array([10, 20], dtype=np.float32)
    y = ops.fc(x, w, b)
    np.testing.assert_array_equal(y.reshape(2, 2), [[8, 23], [8, 27.5]])
    # fc == 1x1 conv on a 1x1 map; fc on a map flattens in H,W,C order == a conv with a full-size filter
    x4 = rnd((2, 3, 2, 5), 15)
    wf = rnd((4, 3 * 2 * 5), 16)
    y1 = ops.fc(x4, wf, None, "relu")
    y2 = ops.conv(x4, wf.reshape(4, 3, 2, 5), None, act="relu")
    np.testing.assert_array_equal(y1, y2)
    ref = np.maximum(x4.reshape(2, -1).astype(np.float64) @ wf.astype(np.float64).T, 0)
    np.testing.assert_allclose(y1.reshape(2, 4), ref, atol=1e-6)


def test_rounding_fp16_bf16():
    # hand-picked ties (round to even) and neighbours
    assert ops.round_store(1 + 2.0 ** -11, "f16") == 1.0                    # tie -> even (down)
    assert ops.round_store(1 + 3 * 2.0 ** -11, "f16") == 1 + 2.0 ** -9      # tie -> even (up)
    assert ops.round_store(1 + 2.0 ** -11 + 2.0 ** -30, "f16") == 1 + 2.0 ** -10
    assert ops.round_store(65504.0, "f16") == 65504.0
    assert ops.round_store(65519.9, "f16") == 65504.0
    assert ops.round_store(65520.0, "f16") == float("inf")                  # tie at the overflow threshold
    assert ops.round_store(2.0 ** -24, "f16") == 2.0 ** -24                 # smallest subnormal
    assert ops.round_store(2.0 ** -25, "f16") == 0.0                        # tie -> even (zero)
    assert ops.round_store(1.5 * 2.0 ** -24, "f16") == 2.0 ** -23
    assert ops.round_store(1 + 2.0 ** -8, "bf16") == 1.0
    assert ops.round_store(1 + 3 * 2.0 ** -8, "bf16") == 1 + 2.0 ** -6
    assert ops.round_store(-(1 + 2.0 ** -8 + 2.0 ** -20), "bf16") == -(1 + 2.0 ** -7)
    # library routines: numpy's double->half cast and torch's float->bfloat16 cast
    v = np.random.default_rng(0).standard_normal(4000) * np.exp(np.random.default_rng(1).uniform(-12, 11, 4000))
    mine = np.array([ops.round_store(t, "f16") for t in v])
    with np.errstate(over="ignore"):
        np.testing.assert_array_equal(mine, v.astype(np.float16).astype(np.float64))
    vf = v.astype(np.float32)
    mine_b = np.array([ops.round_store(float(t), "bf16") for t in vf])
    np.testing.assert_array_equal(mine_b, torch.from_numpy(vf).to(torch.bfloat16).double().numpy())
    # representable values survive
    h = np.random.default_rng(2).standard_normal(1000).astype(np.float16).astype(np.float32)
    np.testing.assert_array_equal(ops.round_array(h, "f16"), h)


def test_storage_rounding_applied_once_after_epilogue():
    x = np.full((1, 1, 1, 4), 0.1, dtype=np.float32)
    x = ops.round_array(x, "f16")
    w = ops.round_array(np.full((1, 1, 1, 4), 0.3, dtype=np.float32), "f16")
    b = np.array([1e-3], dtype=np.float32)
    y = ops.conv(x, w, b, dtype="f16")[0, 0, 0, 0]
    exact = 4 * float(x[0, 0, 0, 0]) * float(w[0, 0, 0, 0]) + float(b[0])
    assert y == np.float32(np.float16(exact))


def test_bn_fold_identity():
    x = rnd((2, 6, 6, 3), 20)
    w = rnd((5, 3, 3, 3), 21)
    g = np.random.default_rng(22)
    bn = {"gamma": g.uniform(0.5, 1.5, 5).astype(np.float32), "beta": g.standard_normal(5).astype(np.float32),
          "mean": g.standard_normal(5).astype(np.float32), "var": g.uniform(0.5, 1.5, 5).astype(np.float32), "eps": 1e-5}
    wf, bf = fold.fold_bn(w, bn)
    folded = ops.conv(x, wf, bf, pad=(1, 1))
    plain = fold.batchnorm(brute_conv(x, w, (1, 1), (1, 1)), bn)
    np.testing.assert_allclose(folded, plain, rtol=0, atol=2e-5)
    # depthwise weights [C,R,S] fold along the first axis too
    wd = rnd((3, 3, 3), 23)
    bn3 = {k: (v[:3] if k != "eps" else v) for k, v in bn.items()}
    wdf, bdf = fold.fold_bn(wd, bn3)
    plain = fold.batchnorm(brute_conv(x, wd.reshape(3, 3, 3, 1), (1, 1), (1, 1), groups=3), bn3)
    np.testing.assert_allclose(ops.dwconv(x, wdf, bdf, pad=(1, 1)), plain, rtol=0, atol=2e-5)


def test_conv_point_matches_full():
    x = rnd((2, 9, 9, 4), 30)
    w = rnd((3, 3, 3, 4), 31)
    y = ops.conv(x, w, stride=(2, 2), pad=(1, 1))
    for (n, p, q, k) in [(0, 0, 0, 0), (1, 4, 4, 2), (1, 2, 3, 1)]:
        assert abs(ops.conv_point(x, w, (2, 2), (1, 1), n, p, q, k) - y[n, p, q, k]) < 1e-6


# ---- grouped convolution, local response normalisation, stand-alone add ------------------------------------------
@pytest.mark.parametrize("groups,c,k,r,st,pd", [(2, 6, 4, 3, (1, 1), (1, 1)), (4, 8, 8, 3, (2, 2), (1, 1)), (2, 4, 6, 5, (1, 1), (2, 2)),
                                                 (3, 6, 3, 1, (1, 1), (0, 0))])
def test_grouped_conv_matches_brute_force_and_torch(groups, c, k, r, st, pd):
    x = rnd((2, 7, 6, c), 31)
    w = rnd((k, r, r, c // groups), 32, 0.3)
    b = rnd((k,), 33, 0.1)
    got = ops.conv(x, w, b, st, pd, "none", None, "f32", groups=groups).astype(np.float64)
    want = brute_conv(x, w, st, pd, groups) + b.astype(np.float64)
    assert np.abs(got - want).max() < 1e-5
    tx = torch.from_numpy(x).double().permute(0, 3, 1, 2)
    tw = torch.from_numpy(w).double().permute(0, 3, 1, 2)
    ty = TF.conv2d(tx, tw, torch.from_numpy(b).double(), st, pd, 1, groups).permute(0, 2, 3, 1).numpy()
    assert np.abs(got - ty).max() < 1e-5
    # a group must not see the other groups' channels: changing group 1's input leaves group 0's output alone
    x2 = x.copy()
    x2[..., c // groups:] += 1.0
    got2 = ops.conv(x2, w, b, st, pd, "none", None, "f32", groups=groups)
    assert np.array_equal(got2[..., :k // groups], got[..., :k // groups].astype(np.float32))
    assert not np.array_equal(got2[..., k // groups:], got[..., k // groups:].astype(np.float32))


def test_lrn_closed_forms_and_torch():
    # constant input a over 7 channels, window 5: interior channels see 5 squares, the edge channels 3 and 4
    a, k, alpha, beta = 2.0, 2.0, 1e-1, 0.75
    x = np.full((1, 2, 2, 7), a, dtype=np.float32)
    y = ops.lrn(x, 5, alpha, beta, k).astype(np.float64)
    counts = [3, 4, 5, 5, 5, 4, 3]
    for ch, cnt in enumerate(counts):
        assert abs(y[0, 0, 0, ch] - a / (k + alpha * cnt * a * a) ** beta) < 1e-6
    # a single non-zero channel: only channels within two of it are damped, and they are zero anyway
    x = np.zeros((1, 1, 1, 9), dtype=np.float32)
    x[0, 0, 0, 4] = 3.0
    y = ops.lrn(x, 5, 1e-4, 0.75, 2.0)
    assert abs(float(y[0, 0, 0, 4]) - 3.0 / (2.0 + 1e-4 * 9.0) ** 0.75) < 1e-6 and np.count_nonzero(y) == 1
    # torch divides alpha by the window size: alpha_torch = alpha * size gives the AlexNet-paper form
    rng = np.random.default_rng(3)
    for size in (3, 5):
        x = rng.standard_normal((2, 3, 4, 11)).astype(np.float32)
        got = ops.lrn(x, size, 2e-2, 0.75, 1.5).astype(np.float64)
        tx = torch.from_numpy(x).double().permute(0, 3, 1, 2)
        want = TF.local_response_norm(tx, size, 2e-2 * size, 0.75, 1.5).permute(0, 2, 3, 1).numpy()
        assert np.abs(got - want).max() < 1e-6
    # storage rounding happens once, at the end
    x = rng.standard_normal((1, 2, 2, 8)).astype(np.float32)
    xh = ops.round_array(x, "f16")
    exact = xh.astype(np.float64) / (2.0 + 1e-4 * np.stack([
        (xh.astype(np.float64) ** 2)[..., max(0, c - 2):min(7, c + 2) + 1].sum(-1) for c in range(8)], -1)) ** 0.75
    assert np.array_equal(ops.lrn(xh, 5, 1e-4, 0.75, 2.0, "f16"), exact.astype(np.float16).astype(np.float32))


def test_add_pins():
    x = np.array([[[[1.5, -2.0, 7.0, 0.25]]]], dtype=np.float32)
    o = np.array([[[[0.5, 1.0, 1.0, -0.25]]]], dtype=np.float32)
    assert ops.add(x, o).ravel().tolist() == [2.0, -1.0, 8.0, 0.0]
    assert ops.add(x, o, "relu").ravel().tolist() == [2.0, 0.0, 8.0, 0.0]
    assert ops.add(x, o, "relu6").ravel().tolist() == [2.0, 0.0, 6.0, 0.0]
    # one rounding of the exact sum: 2048 + 1 is a tie in fp16 (spacing 2) and goes to the even neighbour
    a = np.array([[[[2048.0, 2050.0]]]], dtype=np.float32)
    b = np.array([[[[1.0, 1.0]]]], dtype=np.float32)
    assert ops.add(a, b, "none", "f16").ravel().tolist() == [2048.0, 2052.0]
