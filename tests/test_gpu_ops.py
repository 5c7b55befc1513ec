"""Per-kernel parity on the GPU: small graphs chosen to hit every kernel family, tile shape, split-K path,
vector / scalar path and ragged tail, each compared element by element with the CPU oracle."""
import numpy as np
import pytest

from synth import GraphBuilder
from oracle import forward as OF
from paper_2111_14255_amd import binding as B
from gpu_harness import Mix, assert_close

pytestmark = pytest.mark.gpu

# kernel ids as reported by mt_op_info
DIRECT, IG128, IG64, IG16, DW, MAXP, AVGP, GAP, IG128x64, GEMV = range(10)
PW = 12
STEM = 13
ROWB = 14
PCONV = 15


def g_conv(dtype, n, h, w, c, k, r, stride=1, pad=0, act="relu", bn=True, res=False, coff=0, ctot=0):
    g = GraphBuilder("t", dtype, n, h, w, c)
    short = -1
    t = 0
    if res:
        # residual operand: another convolution with the same output geometry
        short = g.conv(0, k, r, stride=stride, pad=pad, act="none", bn=False)
    g.conv(t, k, r, stride=stride, pad=pad, act=act, bn=bn, res=short, c_off=coff, c_tot=ctot)
    if ctot:
        # fill the remaining channels so that the whole output tensor is defined
        d = g.m.ops[-1].out_tensor
        if coff:
            g.conv(t, coff, r, stride=stride, pad=pad, act="none", dst=d, c_off=0, c_tot=ctot)
        if coff + k < ctot:
            g.conv(t, ctot - coff - k, r, stride=stride, pad=pad, act="none", dst=d, c_off=coff + k, c_tot=ctot)
    return g.done()


CONV_CASES = [
    # name, builder args, expected kernel of the main conv (None = don't care)
    ("ig64_ragged", dict(n=1, h=13, w=13, c=16, k=40, r=3, pad=1), IG64),
    ("ig64_stride2_res", dict(n=2, h=15, w=15, c=24, k=72, r=3, stride=2, pad=1, res=True), IG64),
    ("ig64_1x1_relu6", dict(n=1, h=14, w=14, c=96, k=24, r=1, act="relu6"), IG64),
    ("ig64_1x7", dict(n=1, h=17, w=17, c=32, k=48, r=(1, 7), pad=(0, 3)), IG64),
    ("ig64_7x1", dict(n=1, h=17, w=17, c=32, k=48, r=(7, 1), pad=(3, 0)), IG64),
    ("ig64_5x5", dict(n=1, h=12, w=12, c=8, k=64, r=5, pad=2), IG64),
    ("ig64_splitk", dict(n=1, h=7, w=7, c=256, k=128, r=3, pad=1, res=True), IG64),
    ("ig64_first_layer_5x5", dict(n=1, h=41, w=41, c=3, k=64, r=5, stride=2, pad=2), IG64),
    ("ig64_first_layer_11x11s4", dict(n=1, h=67, w=67, c=3, k=96, r=11, stride=4), IG64),
    ("ig64_c12_scalar", dict(n=1, h=9, w=9, c=12, k=20, r=3, pad=1, act="none"), IG64),
    ("ig64_concat_unaligned", dict(n=1, h=8, w=8, c=16, k=10, r=3, pad=1, coff=3, ctot=18), IG64),
    ("ig64_concat_aligned", dict(n=1, h=8, w=8, c=16, k=32, r=1, coff=64, ctot=128), IG64),
    ("ig16_conv_tiny_map", dict(n=2, h=4, w=4, c=64, k=70, r=3, pad=1), IG16),
    ("ig64_splitk_wide", dict(n=1, h=66, w=66, c=128, k=64, r=3, pad=1, res=True), IG64),
    ("gemv_1x1_m1", dict(n=1, h=1, w=1, c=1280, k=1000, r=1, act="none"), GEMV),
    ("gemv_1x1_m5_res", dict(n=5, h=1, w=1, c=520, k=77, r=1, res=True), GEMV),
    ("pw_1x1_m12", dict(n=12, h=1, w=1, c=512, k=100, r=1), PW),
    ("pw_stride2_res", dict(n=2, h=15, w=15, c=64, k=128, r=1, stride=2, res=True), PW),
    ("pw_four_slices_res", dict(n=1, h=7, w=7, c=960, k=160, r=1, act="none", res=True), PW),
    ("pw_four_slices_two_chunks_per_wave", dict(n=1, h=7, w=7, c=2048, k=72, r=1), PW),
    ("pw_c24_partial_step_scalar_store", dict(n=1, h=9, w=9, c=24, k=18, r=1, act="none"), PW),
    ("pw_concat_unaligned", dict(n=1, h=8, w=8, c=16, k=10, r=1, coff=3, ctot=18), PW),
    ("pw_largest_map_64x64", dict(n=1, h=64, w=64, c=32, k=48, r=1, act="relu6"), PW),
    ("ig64_1x1_c12_element_gather", dict(n=1, h=10, w=10, c=12, k=32, r=1), IG64),
    ("ig128x64", dict(n=1, h=128, w=128, c=8, k=100, r=3, pad=1), IG128x64),
    ("ig128x64_long_reduction_eight_waves", dict(n=1, h=128, w=128, c=128, k=128, r=3, pad=1, res=True), IG128x64),
    ("ig128", dict(n=2, h=182, w=182, c=8, k=128, r=3, pad=1, res=True), IG128),
    ("ig128_first_layer", dict(n=2, h=200, w=200, c=3, k=120, r=3, pad=1), IG128),
    # first-layer kernel: three input channels, even horizontal stride, even width, 32 or 64 output channels
    ("stem_7x7_ragged_tile", dict(n=1, h=40, w=40, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_7x7_three_images", dict(n=3, h=38, w=46, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_7x7_all_border", dict(n=2, h=8, w=8, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_7x7_one_pixel_row", dict(n=1, h=2, w=2, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_7x7_k32_no_act", dict(n=2, h=30, w=34, c=3, k=32, r=7, stride=2, pad=3, act="none", bn=False), STEM),
    ("stem_7x7_224", dict(n=2, h=224, w=224, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_7x7_grid_stride", dict(n=9, h=224, w=224, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_3x3_k32_relu6", dict(n=2, h=34, w=30, c=3, k=32, r=3, stride=2, pad=1, act="relu6"), STEM),
    ("stem_3x3_k64", dict(n=1, h=224, w=224, c=3, k=64, r=3, stride=2, pad=1), STEM),
    ("stem_3x3_all_border", dict(n=3, h=2, w=4, c=3, k=32, r=3, stride=2, pad=1), STEM),
    ("stem_7x7_concat", dict(n=1, h=36, w=36, c=3, k=64, r=7, stride=2, pad=3, coff=64, ctot=136), STEM),
    # filters resident in LDS, activations straight from memory: 1x1 / 3x3 on 64 or 256 channels, maps of 8192 pixels or more
    ("rowb_1x1_c64_n64", dict(n=1, h=96, w=96, c=64, k=64, r=1), ROWB),
    ("rowb_1x1_c64_n256_res", dict(n=1, h=92, w=92, c=64, k=256, r=1, res=True), ROWB),
    ("rowb_1x1_c256_n64_ragged", dict(n=1, h=91, w=93, c=256, k=64, r=1, act="relu6"), ROWB),
    ("rowb_1x1_c256_n128", dict(n=2, h=66, w=66, c=256, k=128, r=1, act="none", bn=False), ROWB),
    ("rowb_1x1_stride2", dict(n=4, h=100, w=100, c=64, k=256, r=1, stride=2), ROWB),
    ("rowb_3x3_res_ragged", dict(n=1, h=95, w=97, c=64, k=64, r=3, pad=1, res=True), ROWB),
    ("rowb_3x3_patch_three_images", dict(n=3, h=60, w=52, c=64, k=64, r=3, pad=1, act="relu6"), ROWB),
    ("rowb_3x3_patch_grid_stride", dict(n=5, h=112, w=112, c=64, k=64, r=3, pad=1, res=True), ROWB),
    ("rowb_3x3_stride2", dict(n=3, h=120, w=116, c=64, k=64, r=3, stride=2, pad=1), ROWB),
    ("rowb_3x3_no_padding", dict(n=1, h=100, w=100, c=64, k=64, r=3), ROWB),
    ("rowb_1x1_c128_n512_sliced_res", dict(n=1, h=92, w=92, c=128, k=512, r=1, res=True), ROWB),
    ("rowb_1x1_c256_n512_stride2", dict(n=4, h=100, w=100, c=256, k=512, r=1, stride=2), ROWB),
    ("rowb_1x1_c64_n128_two_slices", dict(n=1, h=96, w=96, c=64, k=128, r=1, act="none"), ROWB),
    ("rowb_1x1_c256_n192_three_slices", dict(n=1, h=91, w=93, c=256, k=192, r=1), ROWB),
    ("rowb_concat", dict(n=1, h=96, w=96, c=64, k=64, r=1, coff=64, ctot=192), ROWB),
    # 3x3 / stride 1 / padding 1 on 64 k channels, 150 or more 64x64 tiles: activations staged as an input patch
    ("pconv_w56_two_channel_tiles", dict(n=2, h=56, w=56, c=64, k=128, r=3, pad=1), PCONV),
    ("pconv_w31_res_ragged", dict(n=3, h=27, w=31, c=128, k=256, r=3, pad=1, res=True), PCONV),
    ("pconv_w14_tiles_span_rows", dict(n=16, h=14, w=14, c=256, k=256, r=3, pad=1, res=True), PCONV),
    ("pconv_w7_tiles_span_images", dict(n=40, h=7, w=7, c=64, k=320, r=3, pad=1, act="relu6"), PCONV),
    ("pconv_w112_large_patch", dict(n=1, h=112, w=112, c=64, k=128, r=3, pad=1, act="none", bn=False), PCONV),
    ("pconv_partial_channel_tile", dict(n=8, h=28, w=28, c=64, k=72, r=3, pad=1), PCONV),
    ("pconv_concat", dict(n=8, h=28, w=28, c=64, k=128, r=3, pad=1, coff=64, ctot=256), PCONV),
    # general form: runs that start on odd elements (odd stride, odd width, even 3 * pad)
    ("stem_general_3x3_s1_vgg_like", dict(n=2, h=30, w=30, c=3, k=64, r=3, pad=1), STEM),
    ("stem_general_3x3_s2_odd_map_ends_on_half_dword", dict(n=1, h=35, w=35, c=3, k=32, r=3, stride=2), STEM),
    ("stem_general_7x7_odd_width", dict(n=3, h=41, w=41, c=3, k=64, r=7, stride=2, pad=3), STEM),
    ("stem_general_3x3_s1_odd_width_all_border", dict(n=3, h=3, w=5, c=3, k=32, r=3, pad=1, act="none", bn=False), STEM),
    ("stem_general_7x7_s1_even_pad", dict(n=1, h=36, w=38, c=3, k=32, r=7, stride=1, pad=2), STEM),
    ("stem_general_3x3_224", dict(n=1, h=224, w=224, c=3, k=64, r=3, pad=1), STEM),
    ("stem_general_3x3_s2_299", dict(n=1, h=299, w=299, c=3, k=32, r=3, stride=2), STEM),
    ("stem_7x7_row_stride_1", dict(n=1, h=20, w=44, c=3, k=64, r=7, stride=(1, 2), pad=3), STEM),
]


def _expand_cases():
    """Small problems (<= 4096 pixels and <= 3e8 MACs) run on the 64x16 tile; every case written for the 64x64
    tile is therefore run twice: as is (64x16 kernel) and on a map of more than 4096 output pixels (64x64 kernel)."""
    out = []
    for name, kw, kid in CONV_CASES:
        if kid != IG64:
            out.append((name, kw, kid))
            continue
        if name == "ig64_first_layer_5x5":
            out.append((name + "_small", kw, IG16))
            out.append((name + "_big", dict(kw, h=139, w=139), IG64))
            continue
        op = g_conv("f16", **kw).ops[1 if kw.get("res") else 0]
        if kw["n"] * op.out_shape[0] * op.out_shape[1] > 4096:
            out.append((name, kw, kid))
            continue
        pointwise = kw["r"] == 1 and not kw.get("pad") and kw["c"] % 8 == 0
        out.append((name + "_small", kw, PW if pointwise else IG16))
        big = dict(kw)
        stride = kw.get("stride", 1)
        r = kw["r"] if isinstance(kw["r"], int) else max(kw["r"])
        side = 66 * stride + (r if not kw.get("pad") else 0)
        big["h"] = big["w"] = side
        big["n"] = 1
        if big["c"] > 64:
            big["c"] = 64                      # keep the oracle fast; the channel-mode of the case is preserved below
            if kw["c"] % 64 != 0:
                big["c"] = kw["c"]
        out.append((name + "_big", big, IG64))
    return out


ALL_CONV_CASES = _expand_cases()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("name,kw,kid", ALL_CONV_CASES, ids=[c[0] for c in ALL_CONV_CASES])
def test_conv_igemm(name, kw, kid, dtype):
    spec = g_conv(dtype, **kw)
    print("case", name, dtype, flush=True)
    mix = Mix([spec], seed=11)
    try:
        main = 1 if kw.get("res") else 0
        info = mix.ctx.op_info(0, main)
        if kid is not None:
            assert info.kernel_id == kid, (info.kernel_id, info.split_k, info.out_h, info.out_w)
        if "splitk" in name and not name.endswith("_big"):   # the enlarged copy has enough tiles without a split
            assert info.split_k > 1
        if "four_slices" in name:
            assert info.split_k == 4
        got, _ = mix.run(mix.ctx.sequential())
        assert_close(got[0], mix.oracle()[0], dtype, name)
    finally:
        mix.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("name,kw", [
    ("aligned_7x7", dict(n=2, h=20, w=24, c=3, k=64, r=7, stride=2, pad=3)),
    ("aligned_3x3", dict(n=1, h=18, w=16, c=3, k=32, r=3, stride=2, pad=1)),
    ("general_3x3", dict(n=1, h=12, w=13, c=3, k=32, r=3, pad=1)),
    ("general_7x7_odd_width", dict(n=1, h=21, w=23, c=3, k=64, r=7, stride=2, pad=3)),
])
def test_first_layer_masks_keep_non_finite_pixels_out_of_foreign_windows(name, kw, dtype):
    """The first-layer kernel loads whole 16-byte groups, which also hold elements of neighbouring pixels (the dummy
    in front of a run, the padding behind it, columns beyond the border).  Their filter weights are zero, but only
    clearing them in registers keeps a NaN next to a window out of that window's output."""
    spec = g_conv(dtype, act="none", bn=False, **kw)
    mix = Mix([spec], seed=5)
    try:
        assert mix.ctx.op_info(0, 0).kernel_id == STEM
        x = mix.x[0]
        h, w = kw["h"], kw["w"]
        for (r, c) in ((5, 7), (9, 0), (3, w - 1), (h - 1, w // 2), (0, 1)):
            x[0, r, c, :] = np.nan
        mix.inputs[0] = mix.ctx.make_input(0, x)
        mix._oracle = None
        got, _ = mix.run(mix.ctx.sequential())
        ref = mix.oracle()[0]
        bad = ~np.isfinite(ref)
        assert bad.any() and not bad.all()
        assert np.array_equal(~np.isfinite(got[0]), bad), name
        scale = float(np.abs(ref[~bad]).max())
        err = float(np.abs(got[0][~bad].astype(np.float64) - ref[~bad].astype(np.float64)).max())
        assert err <= 2e-2 * scale, (name, err, scale)
    finally:
        mix.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_patch_staged_kernel_masks_taps_that_leave_the_image(dtype):
    """In the flattened patch the pixel left of column 0 is the last pixel of the row above, and the row above row 0
    is the last row of the image before: a NaN there must not reach windows that do not contain it."""
    kw = dict(n=16, h=14, w=14, c=64, k=256, r=3, pad=1)
    spec = g_conv(dtype, act="none", bn=False, **kw)
    mix = Mix([spec], seed=6)
    try:
        assert mix.ctx.op_info(0, 0).kernel_id == PCONV
        x = mix.x[0]
        for (n, r, c) in ((0, 3, 13), (1, 13, 5), (2, 0, 0), (5, 13, 13), (6, 0, 7), (9, 6, 0)):
            x[n, r, c, 17] = np.nan
        mix.inputs[0] = mix.ctx.make_input(0, x)
        mix._oracle = None
        got, _ = mix.run(mix.ctx.sequential())
        ref = mix.oracle()[0]
        bad = ~np.isfinite(ref)
        assert bad.any() and not bad.all()
        assert np.array_equal(~np.isfinite(got[0]), bad)
        scale = float(np.abs(ref[~bad]).max())
        err = float(np.abs(got[0][~bad].astype(np.float64) - ref[~bad].astype(np.float64)).max())
        assert err <= 2e-2 * scale, (err, scale)
    finally:
        mix.close()


def g_fc(dtype, n, h, w, c, k, act="none"):
    g = GraphBuilder("t", dtype, n, h, w, c)
    g.fc(0, k, act=act)
    return g.done()


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("n,h,w,c,k", [(1, 7, 7, 32, 100), (3, 1, 1, 1000, 70), (8, 2, 2, 64, 10), (40, 1, 1, 256, 130), (1, 5, 5, 3, 10)])
def test_fc(dtype, n, h, w, c, k):
    spec = g_fc(dtype, n, h, w, c, k, act="relu")
    print("case fc", dtype, n, h, w, c, k, flush=True)
    mix = Mix([spec], seed=12)
    try:
        got, _ = mix.run(mix.ctx.sequential())
        assert_close(got[0], mix.oracle()[0], dtype)
    finally:
        mix.close()


@pytest.mark.parametrize("n,h,w,c,k,r,stride,pad", [(2, 9, 9, 3, 16, 3, 1, 1), (1, 12, 12, 5, 7, 5, 2, 0), (1, 6, 6, 16, 32, 1, 1, 0)])
def test_conv_fp32_direct(n, h, w, c, k, r, stride, pad):
    spec = g_conv("f32", n, h, w, c, k, r, stride, pad, res=True)
    mix = Mix([spec], seed=13, input_dist="uniform")
    try:
        assert mix.ctx.op_info(0, 1).kernel_id == DIRECT
        got, _ = mix.run(mix.ctx.sequential())
        assert_close(got[0], mix.oracle()[0], "f32")
    finally:
        mix.close()


def g_chain(dtype, n, h, w, c, build):
    g = GraphBuilder("t", dtype, n, h, w, c)
    build(g)
    return g.done()


CHANNELWISE = [
    ("dw_c32", 1, 20, 20, 32, lambda g: g.dwconv(0, 3, 1, 1, act="relu6", bn=True)),
    ("dw_c64_ragged", 2, 7, 9, 64, lambda g: g.dwconv(0, 3, 1, 1, act="relu", bn=True)),
    ("dw_c8", 1, 5, 37, 8, lambda g: g.dwconv(0, 3, 1, 1, act="none", bn=True)),
    ("dw_stride2", 1, 15, 15, 96, lambda g: g.dwconv(0, 3, 2, 1, act="relu6", bn=True)),
    ("dw_c96_stride1", 1, 14, 14, 96, lambda g: g.dwconv(0, 3, 1, 1, act="relu6", bn=True)),
    ("dw_c960", 1, 7, 7, 960, lambda g: g.dwconv(0, 3, 1, 1, act="relu6", bn=True)),
    # large maps: the banded kernel (several output rows per thread, neighbouring columns by wavefront shuffles)
    ("dw_banded_c32_two_rows", 2, 64, 128, 32, lambda g: g.dwconv(0, 3, 1, 1, act="relu6", bn=True)),          # 4 vectors per pixel
    ("dw_banded_c96_four_rows_ragged", 4, 61, 59, 96, lambda g: g.dwconv(0, 3, 1, 1, act="relu", bn=True)),     # 12 per pixel, bands of 4 over 61 rows
    ("dw_banded_c144_stride2", 8, 57, 57, 144, lambda g: g.dwconv(0, 3, 2, 1, act="relu6", bn=True)),           # 18 per pixel, odd width, stride 2
    ("dw_banded_c576_no_neighbour_in_wave", 4, 30, 31, 576, lambda g: g.dwconv(0, 3, 1, 1, act="none", bn=True)),   # 72 per pixel: every neighbour is loaded
    ("dw_banded_c64_stride2_even", 16, 32, 32, 64, lambda g: g.dwconv(0, 3, 2, 1, act="relu", bn=True)),
    ("dw_scalar_c20", 1, 9, 9, 20, lambda g: g.dwconv(0, 3, 1, 1, act="relu", bn=False)),
    ("dw_5x5", 1, 11, 11, 16, lambda g: g.dwconv(0, 5, 1, 2, act="relu", bn=False)),
    ("dw_7x7_generic", 1, 9, 10, 24, lambda g: g.dwconv(0, 7, 1, 3, act="relu", bn=True)),
    ("maxpool_2x2", 2, 14, 14, 64, lambda g: g.maxpool(0, 2, 2)),
    ("maxpool_3x3s2p1", 1, 17, 17, 64, lambda g: g.maxpool(0, 3, 2, 1)),
    ("maxpool_3x3s2_scalar", 1, 13, 13, 12, lambda g: g.maxpool(0, 3, 2)),
    ("avgpool_3x3s1p1", 1, 8, 8, 40, lambda g: g.avgpool(0, 3, 1, 1)),
    ("avgpool_scalar", 1, 6, 7, 5, lambda g: g.avgpool(0, 3, 1, 1)),
    ("gap_7x7", 2, 7, 7, 512, lambda g: g.gap(0)),
    ("gap_8x8_c2048", 1, 8, 8, 2048, lambda g: g.gap(0)),
    ("gap_16x16_c24", 3, 16, 16, 24, lambda g: g.gap(0)),
    ("gap_scalar_c10", 1, 5, 5, 10, lambda g: g.gap(0)),
    ("lrn_5_c96", 1, 9, 9, 96, lambda g: g.lrn(0, 5, 1e-2, 0.75, 2.0)),
    ("lrn_3_c8_single_vector", 2, 5, 6, 8, lambda g: g.lrn(0, 3, 5e-2, 0.5, 1.0)),
    ("lrn_15_c32_widest_window", 1, 4, 4, 32, lambda g: g.lrn(0, 15, 1e-2, 0.75, 1.0)),
    ("lrn_5_scalar_c11", 1, 6, 5, 11, lambda g: g.lrn(0, 5, 1e-2, 0.75, 2.0)),
    ("add_relu_c64", 2, 7, 9, 64, lambda g: g.add(g.maxpool(0, 3, 1, 1), 0, act="relu")),
    ("add_none_scalar_c5", 1, 6, 7, 5, lambda g: g.add(g.avgpool(0, 3, 1, 1), 0)),
    ("conv_groups2_c96_5x5", 1, 13, 13, 96, lambda g: g.conv(0, 256, 5, pad=2, groups=2)),
    ("conv_groups2_c384_3x3", 1, 13, 13, 384, lambda g: g.conv(0, 256, 3, pad=1, groups=2)),
    ("conv_groups4_scalar_gather", 2, 9, 8, 12, lambda g: g.conv(0, 20, 3, pad=1, groups=4, act="none")),
    ("conv_groups2_residual", 1, 8, 8, 32, lambda g: g.conv(g.conv(0, 32, 1), 32, 3, pad=1, groups=2, res=0)),
    ("conv_groups3_1x1_on_1x1_map", 4, 1, 1, 48, lambda g: g.conv(0, 24, 1, groups=3)),
    ("conv_groups2_1x1_pointwise_kernel", 2, 6, 6, 64, lambda g: g.conv(0, 48, 1, groups=2)),
    ("maxpool_into_concat", 1, 9, 9, 16, lambda g: (lambda d: (g.maxpool(0, 3, 2, dst=d, c_off=8, c_tot=24),
                                                               g.conv(0, 8, 3, stride=2, dst=d, c_off=0, c_tot=24)))(g.new_tensor())),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("name,n,h,w,c,build", CHANNELWISE, ids=[c[0] for c in CHANNELWISE])
def test_channelwise(name, n, h, w, c, build, dtype):
    spec = g_chain(dtype, n, h, w, c, build)
    print("case", name, dtype, flush=True)
    mix = Mix([spec], seed=14)
    try:
        got, _ = mix.run(mix.ctx.sequential())
        assert_close(got[0], mix.oracle()[0], dtype, name)
    finally:
        mix.close()


def test_empty_slices_and_single_op_tenant():
    """Degenerate schedules: a tenant with one operator, stages in which some or all tenants have no work."""
    a = g_fc("f16", 1, 1, 1, 64, 16)
    b = g_conv("f16", 1, 8, 8, 8, 16, 3, pad=1)
    mix = Mix([a, b], seed=15)
    try:
        ref = mix.oracle()
        for rho in ([[0, 0, 1], [0, 0, 0]], [[1, 1, 1], [1, 1, 1]], [[0, 0, 0], [1, 1, 1]], [[0, 1, 1], [0, 0, 1]]):
            for flags in (0, B.MT_SCHED_PARALLEL_ISSUE):
                got, tm = mix.run(mix.ctx.schedule(rho, 4, flags=flags))
                assert tm["n_launches"] == 2
                for t in range(2):
                    assert_close(got[t], ref[t], "f16")
                # a stage lasts from the end of the one before to the latest end on its streams; one that launches
                # nothing takes no time, and the stages add up to the makespan
                work = [any((rho[t][st - 1] if st else 0) < (rho[t][st] if st < 3 else 1) for t in range(2)) for st in range(4)]
                assert len(tm["stage_ms"]) == 4
                for st in range(4):
                    assert (tm["stage_ms"][st] > 0) == work[st], (rho, st, tm["stage_ms"])
                assert abs(sum(tm["stage_ms"]) - tm["makespan_ms"]) <= 1e-3 * tm["makespan_ms"] + 1e-6
    finally:
        mix.close()


def test_split_k_is_deterministic_and_counters_reset():
    """The split-K reduction adds partial sums in split order whatever the arrival order: repeated runs of
    the same operator, alone and next to a busy neighbour stream, give identical bits."""
    a = g_conv("f16", 1, 7, 7, 512, 512, 3, pad=1, res=True)
    b = g_conv("f16", 2, 56, 56, 64, 64, 3, pad=1)
    mix = Mix([a, b], seed=16)
    try:
        assert mix.ctx.op_info(0, 1).split_k >= 8
        ref = mix.oracle()
        first = None
        for rep in range(25):
            sched = mix.ctx.sequential() if rep % 2 else mix.ctx.all_concurrent()
            got, _ = mix.run(sched)
            assert_close(got[0], ref[0], "f16")
            if first is None:
                first = got
            assert np.array_equal(first[0], got[0]) and np.array_equal(first[1], got[1])
    finally:
        mix.close()


# ---- depthwise convolution fused into the 1x1 convolution that reads it --------------------------------------------
FUSED_BLOCKS = [
    # name, n, h, w, c_in, hidden, c_out, stride, residual
    ("c96_s1_res", 1, 14, 14, 16, 96, 16, 1, True),
    ("c144_s2", 1, 15, 15, 24, 144, 32, 2, False),
    ("c192_s1_ragged_pixels", 2, 7, 9, 32, 192, 32, 1, True),
    ("c384_s1_n96", 1, 14, 14, 64, 384, 96, 1, False),
    ("c960_s1_n160_two_channel_tiles", 1, 7, 7, 160, 960, 160, 1, True),
    ("c32_single_tile_padded", 1, 10, 10, 8, 32, 16, 1, False),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("name,n,h,w,cin,hid,cout,stride,resid", FUSED_BLOCKS, ids=[c[0] for c in FUSED_BLOCKS])
def test_fused_depthwise_pointwise_equals_separate_launches(name, n, h, w, cin, hid, cout, stride, resid, dtype):
    g = GraphBuilder("blk", dtype, n, h, w, cin)
    e = g.conv(0, hid, 1, act="relu6", bn=True)
    d = g.dwconv(e, 3, stride, 1, act="relu6", bn=True)
    g.conv(d, cout, 1, act="none", bn=True, res=0 if resid else -1)
    spec = g.done()
    print("case", name, dtype, flush=True)
    mix = Mix([spec], seed=21)
    try:
        ctx = mix.ctx
        fused, tm = mix.run(ctx.sequential(flags=B.MT_SCHED_FUSE_DEPTHWISE))
        assert tm["n_fused"] == (1 if hid <= 256 else 0), tm     # longer reductions are cut into four ranges: not fused
        dshape = (n,) + tuple(spec.ops[1].out_shape)
        dw_fused = ctx.read_tensor(0, d, dshape)
        plain, tm = mix.run(ctx.sequential())
        assert tm["n_fused"] == 0
        dw_plain = ctx.read_tensor(0, d, dshape)
        split, tm = mix.run(ctx.schedule([[2]], 2, flags=B.MT_SCHED_FUSE_DEPTHWISE))   # a stage boundary between the two operators: no fusion either
        assert tm["n_fused"] == 0
        assert np.array_equal(fused[0].view(np.uint32), plain[0].view(np.uint32))
        assert np.array_equal(fused[0].view(np.uint32), split[0].view(np.uint32))
        assert np.array_equal(dw_fused.view(np.uint32), dw_plain.view(np.uint32))      # the intermediate tensor stays valid
        ref, tensors = OF.forward(spec, OF.prepare_params(spec, mix.raw[0]), mix.x[0], keep=True)
        assert_close(fused[0], ref, dtype, name)
        assert_close(dw_fused.reshape(n, -1), tensors[d].reshape(n, -1), dtype, name + " depthwise output")
    finally:
        mix.close()


# ---- 1x1 convolution fused with the depthwise convolution that reads it (small maps) ---------------------------------
EXPAND_BLOCKS = [
    # name, n, h, w, c_in, hidden, c_out, stride, residual, fused
    ("c64_h384_14x14", 1, 14, 14, 64, 384, 64, 1, True, True),
    ("c96_h576_14x14_s2", 1, 14, 14, 96, 576, 160, 2, False, True),
    ("c160_h960_7x7", 1, 7, 7, 160, 960, 320, 1, False, True),
    ("c32_h192_7x9_two_images", 2, 7, 9, 32, 192, 32, 1, True, True),
    ("c24_h144_13x13_partial_chunk", 1, 13, 13, 24, 144, 24, 1, True, True),
    ("c128_h64_16x16_largest_map", 1, 16, 16, 128, 64, 32, 1, False, True),
    ("c8_h8_2x2_map", 3, 2, 2, 8, 8, 8, 1, True, True),
    ("c8_h8_1x1_map_matrix_vector_form", 3, 1, 1, 8, 8, 8, 1, True, False),
    ("c256_h64_8x8_deep_reduction", 1, 8, 8, 256, 64, 16, 2, False, True),
    ("c32_h192_28x28_four_bands", 1, 28, 28, 32, 192, 32, 1, True, True),
    ("c32_h192_28x28_s2", 1, 28, 28, 32, 192, 64, 2, False, True),
    ("c24_h144_56x56_wide_rows", 1, 56, 56, 24, 144, 24, 1, True, True),
    ("c24_h144_57x55_s2_odd", 1, 57, 55, 24, 144, 32, 2, False, True),
    ("c136_h64_12x12_deep_reduction_many_bands", 1, 12, 12, 136, 64, 16, 1, False, True),
    ("c160_h64_8x32_rows_too_wide", 1, 8, 32, 160, 64, 16, 1, False, False),
    ("c264_h64_6x6_reduction_too_deep", 1, 6, 6, 264, 64, 16, 1, False, False),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("name,n,h,w,cin,hid,cout,stride,resid,fusable", EXPAND_BLOCKS, ids=[c[0] for c in EXPAND_BLOCKS])
def test_fused_pointwise_depthwise_equals_separate_launches(name, n, h, w, cin, hid, cout, stride, resid, fusable, dtype):
    g = GraphBuilder("blk", dtype, n, h, w, cin)
    pre = g.conv(0, cin, 1, act="none", bn=True)          # the block input is an arena tensor, as inside a network
    e = g.conv(pre, hid, 1, act="relu6", bn=True)
    d = g.dwconv(e, 3, stride, 1, act="relu6", bn=True)
    g.conv(d, cout, 1, act="none", bn=True, res=pre if resid and stride == 1 and cout == cin else -1)
    spec = g.done()
    print("case", name, dtype, flush=True)
    mix = Mix([spec], seed=23)
    try:
        ctx = mix.ctx
        eshape = (n,) + tuple(spec.ops[1].out_shape)
        dshape = (n,) + tuple(spec.ops[2].out_shape)
        fused, tm = mix.run(ctx.sequential(flags=B.MT_SCHED_FUSE_EXPAND))
        assert tm["n_fused"] == (1 if fusable else 0), tm
        assert tm["n_launches"] == 4
        e_fused, d_fused = ctx.read_tensor(0, e, eshape), ctx.read_tensor(0, d, dshape)
        plain, tm = mix.run(ctx.sequential())
        assert tm["n_fused"] == 0
        e_plain, d_plain = ctx.read_tensor(0, e, eshape), ctx.read_tensor(0, d, dshape)
        both, tm = mix.run(ctx.sequential(flags=B.MT_SCHED_FUSE_EXPAND | B.MT_SCHED_FUSE_DEPTHWISE))
        assert tm["n_fused"] >= (1 if fusable else 0)
        split, tm = mix.run(ctx.schedule([[2]], 2, flags=B.MT_SCHED_FUSE_EXPAND))   # a stage boundary inside the pair: no fusion
        assert tm["n_fused"] == 0
        for other in (plain, both, split):
            assert np.array_equal(fused[0].view(np.uint32), other[0].view(np.uint32))
        assert np.array_equal(e_fused.view(np.uint32), e_plain.view(np.uint32))        # both intermediate tensors stay valid
        assert np.array_equal(d_fused.view(np.uint32), d_plain.view(np.uint32))
        ref, tensors = OF.forward(spec, OF.prepare_params(spec, mix.raw[0]), mix.x[0], keep=True)
        assert_close(fused[0], ref, dtype, name)
        assert_close(e_fused.reshape(n, -1), tensors[e].reshape(n, -1), dtype, name + " widened tensor")
        assert_close(d_fused.reshape(n, -1), tensors[d].reshape(n, -1), dtype, name + " depthwise output")
    finally:
        mix.close()


# ---- 2x2 max pooling applied in the epilogue of the convolution that feeds it ---------------------------------------
POOL_BLOCKS = [
    # name (starts with the kernel expected), n, h, w, c_in, c_out, window, stride, pad, act, fusable
    ("igemm_64x16_16x16", 1, 16, 16, 64, 64, 3, 1, 1, "relu", True),
    ("igemm_64x64_two_wave_groups_56x56", 1, 56, 56, 128, 128, 3, 1, 1, "relu", True),
    ("igemm_64x64_split_14x14_c512", 1, 14, 14, 512, 512, 3, 1, 1, "relu", True),
    ("igemm_128x64_batch4_56x56", 4, 56, 56, 128, 256, 3, 1, 1, "relu6", True),
    ("igemm_128x128_batch8_112x112", 8, 112, 112, 64, 128, 3, 1, 1, "relu", True),
    ("ragged_6x10_c24_k40", 3, 6, 10, 24, 40, 3, 1, 1, "none", True),
    ("pointwise_stride2_conv_large_map", 2, 140, 100, 32, 72, 1, 2, 0, "relu", True),
    ("pointwise_small_map_direct_operand_kernel_not_fused", 2, 20, 12, 32, 72, 1, 2, 0, "relu", False),
    ("first_layer_c3_element_gather", 1, 32, 32, 3, 48, 3, 1, 1, "relu", True),
    ("first_layer_kernel_is_not_fused", 1, 32, 32, 3, 64, 3, 1, 1, "relu", False),
    ("odd_map_15x15_not_fused", 1, 15, 15, 64, 64, 3, 1, 1, "relu", False),
    ("k_not_multiple_of_8_not_fused", 1, 16, 16, 64, 36, 3, 1, 1, "relu", False),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("name,n,h,w,cin,cout,win,stride,pad,act,fusable", POOL_BLOCKS, ids=[c[0] for c in POOL_BLOCKS])
def test_pooling_in_the_convolution_epilogue_equals_separate_launches(name, n, h, w, cin, cout, win, stride, pad, act, fusable, dtype):
    g = GraphBuilder("blk", dtype, n, h, w, cin)
    c = g.conv(0, cout, win, stride, pad, act=act, bn=True)
    pl = g.maxpool(c, 2, 2, 0)
    g.conv(pl, 16, 1, act="none", bn=True)
    spec = g.done()
    print("case", name, dtype, flush=True)
    mix = Mix([spec], seed=29)
    try:
        ctx = mix.ctx
        if name.startswith("igemm_"):
            kname = B.load().mt_kernel_name(ctx.op_info(0, 0).kernel_id).decode()
            assert name.startswith(kname), kname
        if "split" in name:
            assert ctx.op_info(0, 0).split_k > 1
        pshape = (n,) + tuple(spec.ops[1].out_shape)
        fused, tm = mix.run(ctx.sequential(flags=B.MT_SCHED_FUSE_POOL))
        assert tm["n_fused"] == (1 if fusable else 0), tm
        assert tm["n_launches"] == 3
        p_fused = ctx.read_tensor(0, pl, pshape)
        plain, tm = mix.run(ctx.sequential())
        assert tm["n_fused"] == 0
        p_plain = ctx.read_tensor(0, pl, pshape)
        split, tm = mix.run(ctx.schedule([[1]], 2, flags=B.MT_SCHED_FUSE_POOL))     # a stage boundary inside the pair: no fusion
        assert tm["n_fused"] == 0
        assert np.array_equal(fused[0].view(np.uint32), plain[0].view(np.uint32))
        assert np.array_equal(fused[0].view(np.uint32), split[0].view(np.uint32))
        assert np.array_equal(p_fused.view(np.uint32), p_plain.view(np.uint32))
        ref, tensors = OF.forward(spec, OF.prepare_params(spec, mix.raw[0]), mix.x[0], keep=True)
        assert_close(fused[0], ref, dtype, name)
        assert_close(p_fused.reshape(n, -1), tensors[pl].reshape(n, -1), dtype, name + " pooled tensor")
    finally:
        mix.close()
