// Host runtime: model construction and shape inference, kernel planning, registration (weight packing and
// upload), schedule deployment on per-tenant HIP streams with event barriers, timing, profile-driven search.
// Paper: Sec. III-A (problem), III-B (IR: stream, pointer, stage, schedule), III-C (search), III-D (issue order).
#include <hip/hip_runtime_api.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <array>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <set>
#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <memory>

#include "internal.h"

using namespace mt;

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline int elt_size(int dtype) { return dtype == MT_F32 ? 4 : 2; }

struct TensorInfo {
    int h = 0, w = 0, c = 0;
    bool defined = false;
    size_t offset = 0, bytes = 0;
};

struct OpRec {
    mt_op_desc d{};
    int in_h = 0, in_w = 0, in_c = 0, out_h = 0, out_w = 0, out_c = 0;
    OpArgs plan{};                 // shape part filled by mt_model_end
    std::vector<uint8_t> w_host;   // raw weights as given
    std::vector<float> bias_host;
    bool has_weights = false;
    size_t w_off = 0, w_bytes = 0, bias_off = 0, ws_off = 0, ws_bytes = 0, cnt_off = 0, cnt_bytes = 0;
    double flops = 0, bytes = 0;
};

}  // namespace

struct mt_model {
    int dtype = 0, batch = 0, in_h = 0, in_w = 0, in_c = 0;
    std::vector<OpRec> ops;
    std::vector<TensorInfo> tensors;
    bool finalized = false;
    size_t arena_bytes = 0;
    int final_tensor = -1;
};

namespace {

// Pixel range of the resident-filter kernel.  Below 8192 pixels there are too few 32-pixel wave tiles to fill the chip
// (ResNet-50 256 -> 1024 on a 14x14 map at batch 16: 10.9 us against 8.7 us on the 128x64 tile).  A 3x3 window reads every
// input line nine times through the L1, which bounds it on large maps (64 -> 64 on 56x56 at batch 16 / 128: 12.1 / 70.4 us
// against 15.0 / 65.7 us on the tile kernel).
constexpr int ROWB_MIN_PIXELS = 8192, ROWB_MAX_PIXELS_3X3 = 131072;
constexpr int PCONV_MIN_TILES = 150;

bool needs_weights(int kind) { return kind == MT_CONV || kind == MT_DWCONV || kind == MT_FC; }

// Kernel, tile and split choice of a convolution / fully connected layer: a pure function of the GEMM shape.
void plan_igemm(OpArgs &p, int M, int Kc, int gemm_k) {
    auto cdiv = [](int a, int b) { return (a + b - 1) / b; };
    p.k_pad = cdiv(gemm_k, IGEMM_BK) * IGEMM_BK;
    p.grid_y = p.grid_z = 1;
    p.block = 256;
    p.split_k = 1;
    if (M <= 8 && p.H == 1 && p.W == 1 && p.R == 1 && p.S == 1 && p.vec_a && p.groups <= 1) {
        p.kernel_id = K_GEMV;
        p.n_pad = cdiv(Kc, 64) * 64;
        p.grid_x = cdiv(cdiv(Kc, 2), 4);          // two output channels per wavefront, four wavefronts per workgroup
        return;
    }
    const double macs_pw = (double)M * Kc * gemm_k;
    if (p.kind == MT_CONV && p.R == 1 && p.S == 1 && p.ph == 0 && p.pw == 0 && p.vec_a != 0 && M <= 4096 && macs_pw <= 3.0e8) {
        // 1x1 convolution on a small map: operands straight from memory, one wave per 16 x 16 output tile.  Up to eight
        // 32-deep reduction steps a wave walks alone (split_k 1); longer reductions are cut into four ranges, one per
        // wave of the workgroup (recorded as split_k 4; no workspace: the partial sums meet in LDS).
        // Measured on MI355X (MobileNetV2 at batch 1, in the chain): 5.4-7.8 us per layer on the 64x16 tile.
        p.kernel_id = K_IGEMM_PW;
        p.n_pad = cdiv(Kc, 64) * 64;
        const int tiles = cdiv(M, 16) * cdiv(Kc, 16);
        p.split_k = (p.k_pad / 32 > 8) ? 4 : 1;
        p.grid_x = p.split_k == 1 ? cdiv(tiles, 4) : tiles;
        make_divisor((uint32_t)p.Q, p.divq_m, p.divq_s1, p.divq_s2);
        make_divisor((uint32_t)p.P * (uint32_t)p.Q, p.divpq_m, p.divpq_s1, p.divpq_s2);
        return;
    }
    int bn, bm, kid;
    // Small problems (few multiply-accumulates on a small map) are latency bound: narrow pixel tiles give more,
    // shorter workgroups.  Measured on MI355X: ResNet-18 3x3 layers (115 M MACs) 9-11 us -> 7.3-8.6 us.
    const double macs = (double)M * Kc * gemm_k;
    if (M <= 32 || (M <= 4096 && macs <= 3.0e8)) {
        kid = K_IGEMM_64x16; bn = 64; bm = 16;
    } else if (Kc >= 96 && cdiv(M, 128) * cdiv(Kc, 128) >= 512) {
        kid = K_IGEMM_128x128; bn = 128; bm = 128;
    } else if (Kc >= 96 && cdiv(M, 64) * cdiv(Kc, 128) >= 256) {
        kid = K_IGEMM_128x64; bn = 128; bm = 64;
    } else {
        kid = K_IGEMM_64x64; bn = 64; bm = 64;
    }
    p.kernel_id = kid;
    p.n_pad = cdiv(Kc, bn) * bn;
    const int tiles = cdiv(M, bm) * (p.n_pad / bn);
    const int nkt = p.k_pad / IGEMM_BK;
    int target = (kid == K_IGEMM_64x16) ? 2048 : 768;
    int max_split = 8, min_kt = 6;    // a split below 6 reduction tiles costs more in the partial-sum exchange than it saves
    int split = 1;
    p.wk = 1;
    // Long reductions on the 128x64 tile are bound by the matrix cores: eight waves per tile (two per SIMD) overlap LDS
    // reads with MFMA better than four.  Measured on MI355X at batch 8: 3x3 layers of 128 / 256 / 512 channels on
    // 112^2 / 56^2 / 28^2 maps 62.9 -> 56.5, 62.2 -> 54.9, 59.5 -> 52.1 us; the short reductions of 1x1 layers lose
    // (17.3 -> 19.3 us) and keep four waves.  The same change on the 128x128 tile loses everywhere.
        if (kid == K_IGEMM_128x64 && p.vec_a != 0 && nkt >= 18) p.wk = 2;
    int wk_tiles = 512;
    if (kid == K_IGEMM_64x64 && p.vec_a != 0 && tiles <= wk_tiles) {
        // Few workgroups per compute unit: eight waves per tile (two per SIMD, the MFMA steps of every LDS tile split
        // between two wave groups) and only as many splits as keep about one workgroup per unit.  Measured on MI355X,
        // VGG-16 at batch 1: conv3_2 18.9 -> 13.9 us, conv4_1 15.2 -> 11.8 us, conv4_2 19.7 -> 16.1 us.
        p.wk = 2;
        split = std::max(1, std::min({256 / tiles, std::max(1, nkt / 4), max_split}));
        const int per = cdiv(nkt, split);
        split = cdiv(nkt, per);
    } else if (tiles < target / 2) {
        split = std::min({cdiv(target, tiles), std::max(1, nkt / min_kt), max_split});
        const int per = cdiv(nkt, split);
        split = cdiv(nkt, per);            // no empty split
    }
    p.split_k = std::max(1, split);
    // Only where the 64x64 tile would run unsplit on 150 tiles or more.  On larger problems the patch form is level with
    // the wide tiles on maps up to 28 pixels wide and loses on wider ones, whose patch leaves room for one workgroup per
    // compute unit (batch 8, 256 channels on 56x56: 72 against 57 us; 128 channels on 112x112: 90 against 53 us).
    const bool pconv_size = kid == K_IGEMM_64x64 && p.split_k == 1 && tiles >= PCONV_MIN_TILES;
    if (pconv_size && p.kind == MT_CONV && p.groups <= 1 && p.R == 3 && p.S == 3 && p.sh == 1 && p.sw == 1 && p.ph == 1 && p.pw == 1 &&
        p.C % 64 == 0 && p.K % 8 == 0 && p.y_ct % 8 == 0 && p.y_coff % 8 == 0 && p.res_ct % 8 == 0 && pconv_patch_pixels(p.W) > 0) {
        // 3x3 layers that would run on the 64x64 tile unsplit: same tile, activations staged as an input patch
        p.kernel_id = K_PCONV;
        p.wk = 1;
        p.block = 512;
        p.k_pad = gemm_k;
        p.split_k = 1;
        p.n_pad = cdiv(Kc, 64) * 64;
        p.tile_order = 0;
        make_divisor((uint32_t)p.Q, p.divq_m, p.divq_s1, p.divq_s2);
        make_divisor((uint32_t)p.P * (uint32_t)p.Q, p.divpq_m, p.divpq_s1, p.divpq_s2);
        p.grid_x = cdiv(cdiv(M, 64) * (p.n_pad / 64), 8) * 8;
        return;
    }
    // Which operand each XCD's L2 keeps to itself: consecutive tiles (one XCD) walk the channel tiles of one pixel
    // tile (0) when the activations are the larger operand, the pixel tiles of one channel tile (1) otherwise.
    p.tile_order = ((double)Kc * gemm_k > (double)p.N * p.H * p.W * p.C) ? 1 : 0;
    make_divisor((uint32_t)p.Q, p.divq_m, p.divq_s1, p.divq_s2);
    make_divisor((uint32_t)p.P * (uint32_t)p.Q, p.divpq_m, p.divpq_s1, p.divpq_s2);
    const int total = tiles * p.split_k;
    p.grid_x = cdiv(total, 8) * 8;
}

int32_t finalize_model(mt_model *m) {
    m->tensors.clear();
    m->tensors.resize(1);
    m->tensors[0].h = m->in_h; m->tensors[0].w = m->in_w; m->tensors[0].c = m->in_c; m->tensors[0].defined = true;
    const int es = elt_size(m->dtype);
    for (size_t i = 0; i < m->ops.size(); ++i) {
        OpRec &o = m->ops[i];
        const mt_op_desc &d = o.d;
        auto bad = [&](const std::string &why) { return fail(MT_ERR_SHAPE_MISMATCH, "op " + std::to_string(i) + ": " + why); };
        if (d.in_tensor < 0 || d.in_tensor >= (int)m->tensors.size() || !m->tensors[d.in_tensor].defined)
            return bad("input tensor is not produced by an earlier operator");
        if (d.out_tensor < 1) return bad("output tensor id must be >= 1");
        if (d.out_tensor > 2 * (int)m->ops.size() + 16) return bad("output tensor id is too large for a model of this many operators");
        if (d.out_tensor == d.in_tensor) return bad("in-place operators are not supported");
        const TensorInfo in = m->tensors[d.in_tensor];
        o.in_h = in.h; o.in_w = in.w; o.in_c = in.c;
        int R = d.r, S = d.s, sh = d.stride_h, sw = d.stride_w, ph = d.pad_h, pw = d.pad_w;
        if (d.kind == MT_GLOBAL_AVGPOOL || d.kind == MT_FC) { R = in.h; S = in.w; sh = sw = 1; ph = pw = 0; }
        const int lrn_size = d.r;
        if (d.kind == MT_LRN || d.kind == MT_ADD) { R = S = 1; sh = sw = 1; ph = pw = 0; }
        const int groups = (d.kind == MT_CONV && d.groups > 1) ? d.groups : 1;
        if (d.kind != MT_CONV && d.groups > 1) return bad("groups are supported on CONV only");
        if (R < 1 || S < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return bad("bad window / stride / padding");
        if (ph >= R || pw >= S) return bad("padding must be smaller than the window");
        if (in.h + 2 * ph < R || in.w + 2 * pw < S) return bad("window larger than the padded input");
        o.out_h = (in.h + 2 * ph - R) / sh + 1;
        o.out_w = (in.w + 2 * pw - S) / sw + 1;
        o.out_c = (d.kind == MT_CONV || d.kind == MT_FC) ? d.out_c : in.c;
        if (o.out_c < 1) return bad("output channels must be >= 1");
        if (d.act < MT_ACT_NONE || d.act > MT_ACT_RELU6) return bad("unknown activation");
        const int ctot = d.out_c_total ? d.out_c_total : o.out_c;
        if (d.out_c_offset < 0 || d.out_c_offset + o.out_c > ctot) return bad("channel range exceeds the output tensor");
        if ((int)m->tensors.size() <= d.out_tensor) m->tensors.resize(d.out_tensor + 1);
        TensorInfo &out = m->tensors[d.out_tensor];
        if (out.defined) {
            if (out.h != o.out_h || out.w != o.out_w || out.c != ctot) return bad("output tensor shape disagrees with an earlier writer");
        } else {
            out.h = o.out_h; out.w = o.out_w; out.c = ctot; out.defined = true;
        }
        int res_ct = 0;
        if (d.res_tensor >= 0) {
            if (d.kind != MT_CONV && d.kind != MT_ADD) return bad("a second input is supported on CONV (residual) and ADD only");
            if (d.res_tensor >= (int)m->tensors.size() || !m->tensors[d.res_tensor].defined || d.res_tensor == d.out_tensor)
                return bad("residual tensor is not produced by an earlier operator");
            const TensorInfo &rt = m->tensors[d.res_tensor];
            if (rt.h != o.out_h || rt.w != o.out_w || rt.c < o.out_c) return bad("residual tensor shape mismatch");
            res_ct = rt.c;
        }
        if (d.kind == MT_ADD && (d.res_tensor < 0 || res_ct != in.c)) return bad("ADD needs a second tensor of the input's shape");
        if (d.kind == MT_ADD && (d.act < MT_ACT_NONE || d.act > MT_ACT_RELU6)) return bad("unknown activation");
        if (d.kind == MT_LRN && (lrn_size < 1 || lrn_size % 2 == 0 || lrn_size > 15)) return bad("LRN window must be odd and at most 15");
        if (groups > 1 && (in.c % groups || o.out_c % groups)) return bad("channel counts must be multiples of the group count");
        OpArgs &p = o.plan;
        p = OpArgs{};
        p.kind = d.kind; p.dtype = m->dtype;
        p.N = m->batch; p.H = in.h; p.W = in.w; p.C = in.c / groups;
        p.x_ct = in.c; p.x_coff = 0; p.groups = groups;
        p.lrn_alpha = d.lrn_alpha; p.lrn_beta = d.lrn_beta; p.lrn_k = d.lrn_k;
        p.K = o.out_c / groups; p.R = d.kind == MT_LRN ? lrn_size : R; p.S = S; p.P = o.out_h; p.Q = o.out_w;
        p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.act = d.act;
        p.res_ct = res_ct; p.y_coff = d.out_c_offset; p.y_ct = ctot;
        p.split_k = 1; p.block = 256; p.vec = 1;
        const int vmax = 16 / es;
        const double out_elems = (double)m->batch * o.out_h * o.out_w * o.out_c;
        const double in_elems = (double)m->batch * in.h * in.w * in.c;
        switch (d.kind) {
            case MT_CONV:
            case MT_FC: {
                const int gemm_k = R * S * (in.c / groups);
                p.gemm_k = gemm_k;
                o.flops = 2.0 * out_elems * gemm_k;
                o.bytes = (in_elems + out_elems + (double)o.out_c * gemm_k + (res_ct ? out_elems : 0)) * es + 4.0 * o.out_c;
                if (m->dtype == MT_F32) {
                    p.kernel_id = K_CONV_DIRECT;
                } else {
                    // a fully connected layer is a 1x1 convolution over a 1x1 map with H*W*C channels
                    if (d.kind == MT_FC) { p.H = p.W = 1; p.C = gemm_k; p.x_ct = gemm_k; p.R = p.S = 1; }
                    // im2col gather mode: 2 = tile inside one tap (C % 64 == 0, at most 64 taps), 1 = 16-byte chunks, 0 = element-wise
                    p.vec_a = (p.C % IGEMM_BK == 0 && p.R * p.S <= 64) ? 2 : (p.C % 8 == 0) ? 1 : 0;
                    const int sform = (d.kind == MT_CONV && groups == 1 && in.c == 3 && res_ct == 0 && ctot % 8 == 0 && d.out_c_offset % 8 == 0)
                                          ? stem_form(R, S, sw, in.w, pw, o.out_c) : 0;
                    const StemGeom sg = stem_geom(R, S, sform);
                    if (sform > 0) {
                        // first layer: the im2col rows are contiguous runs of an input row and go straight into the
                        // MFMA operand registers.  Measured on MI355X (ResNet-50 stem, bf16, batch 1 / 16 / 128): 4.8 / 12.6 /
                        // 58 us against 7 / 45.7 / 303 us with the element-wise gather of the tile kernel.
                        p.kernel_id = K_STEM;
                        p.n_pad = o.out_c;
                        p.k_pad = sg.ksteps * 16;
                        const int n_tiles = (m->batch * o.out_h * o.out_w + 31) / 32;
                                                // as many workgroups as stay resident (3 per compute unit for the 7x7 window with 64 channels, by
                        // registers and LDS; 6 or more for the lighter forms); the waves walk the tiles with a grid stride
                        p.grid_x = std::min((n_tiles + 3) / 4, (R == 7 && o.out_c == 64) ? 768 : 1536);
                        p.grid_y = p.grid_z = 1;
                        make_divisor((uint32_t)p.Q, p.divq_m, p.divq_s1, p.divq_s2);
                        make_divisor((uint32_t)p.P * (uint32_t)p.Q, p.divpq_m, p.divpq_s1, p.divpq_s2);
                        break;
                    }
                    const int M = m->batch * o.out_h * o.out_w;
                    const int rw = (d.kind == MT_CONV && groups == 1 && ph < R && (R == 3 || (ph == 0 && pw == 0))) ? rowb_waves(R, S, in.c, o.out_c) : 0;
                    if (rw > 0 && res_ct % 8 == 0 && ctot % 8 == 0 && d.out_c_offset % 8 == 0 && M >= ROWB_MIN_PIXELS &&
                        (R == 1 || M <= ROWB_MAX_PIXELS_3X3 || (sh == 1 && sw == 1))) {
                        // few output channels or a short reduction on a large map: filters resident in LDS, one wave per 32 pixels
                        p.kernel_id = K_ROWB;
                        p.n_pad = o.out_c;
                        p.k_pad = gemm_k;
                        p.block = 64 * rw;
                        // one workgroup per (slice of output channels, chunk of rw pixel tiles); chunks beyond what stays
                        // resident are walked with a stride
                        const int n_tiles = (M + 31) / 32;
                        const int slices = o.out_c / (32 * rowb_tiles(R, S, in.c, o.out_c));
                        p.grid_x = slices * std::max(1, std::min((n_tiles + rw - 1) / rw, 512 / slices));
                        if (rowb_patch_form(p)) {
                            // 4 x 8 pixel tiles, eight per workgroup, one workgroup per compute unit (143 KB of LDS)
                            const int t2 = m->batch * ((o.out_h + 3) / 4) * ((o.out_w + 7) / 8);
                            p.grid_x = std::max(1, std::min((t2 + rw - 1) / rw, 256));
                        }
                        p.grid_y = p.grid_z = 1;
                        make_divisor((uint32_t)p.Q, p.divq_m, p.divq_s1, p.divq_s2);
                        make_divisor((uint32_t)p.P * (uint32_t)p.Q, p.divpq_m, p.divpq_s1, p.divpq_s2);
                        break;
                    }
                    plan_igemm(p, M, o.out_c / groups, gemm_k);
                }
                break;
            }
            case MT_DWCONV:
                p.kernel_id = K_DWCONV;
                p.vec = (in.c % vmax == 0 && ctot % vmax == 0 && d.out_c_offset % vmax == 0) ? vmax : 1;
                o.flops = 2.0 * out_elems * R * S;
                o.bytes = (in_elems + out_elems + (double)in.c * R * S) * es + 4.0 * in.c;
                break;
            case MT_MAXPOOL:
            case MT_AVGPOOL:
            case MT_GLOBAL_AVGPOOL:
                p.kernel_id = d.kind == MT_MAXPOOL ? K_MAXPOOL : d.kind == MT_AVGPOOL ? K_AVGPOOL : K_GAP;
                p.vec = (in.c % vmax == 0 && ctot % vmax == 0 && d.out_c_offset % vmax == 0) ? vmax : 1;
                o.flops = 0;
                o.bytes = (in_elems + out_elems) * es;
                break;
            case MT_LRN:
                p.kernel_id = K_LRN;
                p.vec = (in.c % vmax == 0) ? vmax : 1;
                o.flops = out_elems * (2.0 * lrn_size + 3);
                o.bytes = (in_elems + out_elems) * es;
                break;
            case MT_ADD:
                p.kernel_id = K_ADD;
                p.vec = (in.c % vmax == 0) ? vmax : 1;
                o.flops = out_elems;
                o.bytes = (2 * in_elems + out_elems) * es;
                break;
            default:
                return bad("unknown operator kind");
        }
    }
    if (m->ops.empty()) return fail(MT_ERR_SHAPE_MISMATCH, "model has no operators");
    m->final_tensor = m->ops.back().d.out_tensor;

    // ---- arena layout: weights, activations, split-K workspaces -----------------------------
    size_t off = 0;
    for (OpRec &o : m->ops) {
        const OpArgs &p = o.plan;
        if (needs_weights(p.kind)) {
            bool igemm = is_gemm_kernel(p.kernel_id) || p.kernel_id == K_STEM || p.kernel_id == K_ROWB || p.kernel_id == K_PCONV;
            size_t wcount = igemm ? (size_t)p.groups * p.n_pad * p.k_pad
                                  : (p.kind == MT_DWCONV ? (size_t)p.C * p.R * p.S : (size_t)p.groups * p.K * o.plan.R * o.plan.S * p.C);
            if (p.kind == MT_FC && !igemm) wcount = (size_t)p.K * o.in_h * o.in_w * o.in_c;
            o.w_off = off; o.w_bytes = wcount * es; off += align_up(o.w_bytes);
            const size_t nb = (size_t)p.groups * (igemm ? p.n_pad : p.K);
            o.bias_off = off; off += align_up(nb * sizeof(float));
        }
        if (p.split_k > 1 && p.kernel_id != K_IGEMM_PW) {
            const int bn = p.kernel_id == K_IGEMM_64x16 || p.kernel_id == K_IGEMM_64x64 ? 64 : 128;
            const int bm = p.kernel_id == K_IGEMM_64x16 ? 16 : p.kernel_id == K_IGEMM_128x128 ? 128 : 64;
            const int M = p.N * p.P * p.Q;
            const size_t tiles = (size_t)((M + bm - 1) / bm) * (p.n_pad / bn);
            o.ws_off = off; o.ws_bytes = tiles * p.split_k * bn * bm * sizeof(float); off += align_up(o.ws_bytes);
            o.cnt_off = off; o.cnt_bytes = tiles * sizeof(uint32_t); off += align_up(o.cnt_bytes);
        }
    }
    for (size_t t = 1; t < m->tensors.size(); ++t) {
        TensorInfo &ti = m->tensors[t];
        if (!ti.defined) continue;
        ti.bytes = (size_t)m->batch * ti.h * ti.w * ti.c * es;
        ti.offset = off;
        off += align_up(ti.bytes + 16);
    }
    m->tensors[0].bytes = (size_t)m->batch * m->in_h * m->in_w * m->in_c * es;
    // The kernels index tensors and packed filters with 32-bit offsets.
    const size_t limit = (size_t)1 << 31;
    for (size_t t = 0; t < m->tensors.size(); ++t)
        if (m->tensors[t].defined && m->tensors[t].bytes >= limit)
            return fail(MT_ERR_SHAPE_MISMATCH, "tensor " + std::to_string(t) + " is 2 GiB or larger: not supported");
    for (size_t i = 0; i < m->ops.size(); ++i)
        if (m->ops[i].w_bytes >= limit || m->ops[i].ws_bytes >= limit)
            return fail(MT_ERR_SHAPE_MISMATCH, "op " + std::to_string(i) + ": packed filters or split workspace of 2 GiB or more: not supported");
    m->arena_bytes = off;
    m->finalized = true;
    return MT_OK;
}

void fill_info(const mt_model *m, const OpRec &o, mt_op_info *out) {
    out->kind = o.d.kind;
    out->in_h = o.in_h; out->in_w = o.in_w; out->in_c = o.in_c;
    out->out_h = o.out_h; out->out_w = o.out_w; out->out_c = o.out_c;
    out->kernel_id = o.plan.kernel_id;
    out->split_k = o.plan.split_k;
    out->grid_blocks = o.plan.grid_x ? o.plan.grid_x : 0;
    out->flops = o.flops;
    out->bytes = o.bytes;
    (void)m;
}

}  // namespace

// ============================================================================================
struct Tenant {
    mt_model model;                 // private copy (host weights dropped after upload)
    uint8_t *arena = nullptr;
    bool owns_arena = false;
    std::vector<OpArgs> args;       // device pointers resolved; input/output patched per run
    std::vector<uint8_t> reads_input, res_input, writes_output;
    std::vector<uint8_t> fuse_next;  // operator i is a depthwise convolution that can run inside the launch of operator i + 1
    std::vector<uint8_t> fuse_pwdw;  // operator i is a 1x1 convolution that can run inside the launch of the depthwise operator i + 1
    std::vector<uint8_t> fuse_pool;  // operator i is a convolution whose epilogue can apply the 2x2 max pooling operator i + 1
    std::vector<OpArgs> pool_args;   // its arguments for that form (pooled output tensor, quad pixel walk)
    std::vector<uint8_t> short_kernel;   // operator runs on a short, latency-bound kernel (see MT_SCHED_PRIORITIZE_SHORT)
    // mt_run_static_scratch: where each split operator's counters and workspace sit inside the tenant's two blocks of the
    // fixed scratch array (byte offsets; blocks are laid out per call, counters of all tenants first)
    std::vector<size_t> st_cnt_off, st_ws_off;
    size_t st_cnt_bytes = 0, st_ws_bytes = 0;
};

struct StreamKey {
    int tenant, share;
    bool operator<(const StreamKey &o) const { return tenant != o.tenant ? tenant < o.tenant : share < o.share; }
};

struct mt_schedule;

// Issuing threads of MT_SCHED_PARALLEL_ISSUE: worker w launches everything that goes to tenant w's stream.
struct IssuePool {
    std::vector<std::thread> threads;
    std::mutex mu;
    std::condition_variable cv;
    uint64_t run_seq = 0;           // guarded by mu
    bool quit = false;              // guarded by mu
    mt_schedule *sched = nullptr;   // the run being issued
    const void *const *inputs = nullptr;
    void *const *outputs = nullptr;
    std::atomic<int> stage_posted{-1};            // stages up to this one may be issued (their gate event is recorded)
    std::atomic<int> stage_done[MT_MAX_STAGES];   // workers that finished issuing the stage
    std::atomic<int> finished{0};                 // workers that left the run
    std::atomic<int> error{0};
    std::string error_msg;                        // guarded by mu
};

struct mt_ctx {
    int device = 0;
    hipDeviceProp_t prop{};
    std::vector<std::unique_ptr<Tenant>> tenants;
    hipStream_t main_stream = nullptr;
    struct StreamEntry { hipStream_t stream = nullptr; int refs = 0; };
    std::map<StreamKey, StreamEntry> streams;   // tenant streams, shared by schedules (reference counted)
    hipEvent_t ev_start = nullptr;
    hipEvent_t ev_stage[MT_MAX_STAGES]{};
    hipEvent_t ev_done[MT_MAX_STAGES][MT_MAX_TENANTS]{};
    hipEvent_t ev_prof[2]{};
    hipEvent_t ev_first[MT_MAX_TENANTS]{};   // after the first operator of each tenant (MT_SCHED_TIME_FIRST_OP)
    hipEvent_t ev_last[MT_MAX_TENANTS]{};    // after the last operator of each tenant (MT_SCHED_TIME_TENANTS)
    // Graph executables of destroyed schedules.  They are released in batches after a device-wide synchronisation (at
    // the end of a search, every 64 candidates inside one, in mt_release_idle_streams and in mt_destroy): destroying one
    // right after its last launch has crashed inside the HIP runtime.
    std::vector<hipGraphExec_t> retired_graphs;
    // Schedules created from this context and not destroyed yet; mt_destroy detaches them so that a later
    // mt_schedule_destroy does not touch the freed context.
    std::set<mt_schedule *> live_schedules;
    IssuePool pool;
    // Masked streams whose hardware queue dispatches slowly (see get_stream) are parked: kept alive, never used.
    std::vector<hipStream_t> parked_streams;       // masked ones; released by purge_idle_streams
    uint32_t *probe_buf = nullptr;
    float best_dispatch_us = 0.f;
    uint32_t *barrier_word = nullptr;    // MT_SCHED_COUNTER_BARRIER: arrivals of the current run (borrowed from the process's pool)
};

struct StagePlan {
    std::vector<IssueItem> items;
    std::vector<int> streams;       // distinct streams used, ascending
    std::vector<std::vector<IssueItem>> by_stream;   // items of each stream (index = tenant that owns the stream), in issue order
    int prev_stage = -1;            // latest earlier stage that launched anything (-1: none)
};

struct mt_schedule {
    mt_ctx *ctx = nullptr;
    int n_tenants = 0, n_stages = 0, flags = 0;
    std::vector<StagePlan> stages;                 // non-empty stages only keep items; empty ones stay for timing
    // MT_SCHED_GRAPH with several tenants: the items of every stage in the other issue order (same operators, same
    // fused pairs), for the second capture
    std::vector<std::vector<IssueItem>> alt_items;
    // stream of (stage, stream owner); the same for every stage unless the shares are given per stage
    std::vector<std::array<hipStream_t, MT_MAX_TENANTS>> stream_at;
    std::vector<StreamKey> stream_keys;     // one reference in the context's pool per entry
    int n_launches = 0;
    int end_stage = -1;             // last stage that launches anything (-1: the schedule launches nothing)
    int n_fused = 0;                // operators that run inside the next operator's launch
    std::vector<uint32_t> arrivals_upto;   // MT_SCHED_COUNTER_BARRIER: streams that have ended stages 0 .. st, summed
    int32_t prio[MT_MAX_TENANTS] = {0};   // wave priority of a tenant's kernels, 0..3; -1: 3 for its short kernels, 0 for the others
    // graph replay
    hipGraphExec_t graph_exec = nullptr;
    std::vector<const void *> cap_in;
    std::vector<void *> cap_out;
    // MT_SCHED_STREAM_GRAPHS: one graph per (stage, stream) with the launches of that stream in that stage
    std::vector<std::array<hipGraphExec_t, MT_MAX_TENANTS>> slice_exec;
    // set for the duration of an mt_run_static_scratch call: base of the fixed scratch array and each tenant's blocks in it
    uint8_t *st_base = nullptr;
    size_t st_cnt_base[MT_MAX_TENANTS] = {}, st_ws_base[MT_MAX_TENANTS] = {};
};

// Hands every graph of a schedule to the context for release at mt_destroy.
static void retire_graphs(mt_ctx *ctx, mt_schedule *s);

namespace {

#define HIP_TRY(expr)                                                                                     \
    do {                                                                                                  \
        hipError_t e_ = (expr);                                                                           \
        if (e_ != hipSuccess) return fail(MT_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

// One kernel launch; returns a hipError_t as int.
int launch_kernel(const OpArgs &a, hipStream_t st, const OpArgs *mate = nullptr, int n_mates = 0) {
    if (a.kernel_id == K_STEM) return launch_stem(a, st, mate, n_mates);
    if (a.kernel_id == K_ROWB) return launch_rowb(a, st, mate, n_mates);
    if (a.kernel_id == K_PCONV) return launch_pconv(a, st, mate, n_mates);
    return is_gemm_kernel(a.kernel_id) ? launch_igemm(a, st, mate, n_mates) : launch_direct(a, st, mate, n_mates);
}

// Two operators can run in one launch if their kernel has a several-operator form and everything in their arguments
// but the buffers (and the wave priority, which the launch takes from the first) is equal: same kernel, tile, split, shape.
bool coissue_pair_ok(const OpArgs &a, const OpArgs &b) {
    if (!coissue_supported(a) || !coissue_supported(b)) return false;
    if ((a.res == nullptr) != (b.res == nullptr) || (a.ws == nullptr) != (b.ws == nullptr)) return false;
    OpArgs x = a, y = b;
    for (OpArgs *o : {&x, &y}) {
        o->x = nullptr; o->w = nullptr; o->bias = nullptr; o->res = nullptr; o->y = nullptr; o->ws = nullptr; o->counters = nullptr;
        o->prio = 0;
    }
    return std::memcmp(&x, &y, sizeof(OpArgs)) == 0;
}

// One operator; returns a hipError_t as int.  A grouped convolution is one operator of the sequence issued as one
// launch per group: each launch reads its slice of the input channels and its own filter bank and writes its slice of
// the output channels.
int launch_raw(const OpArgs &a, hipStream_t st) {
    if (a.groups <= 1) return launch_kernel(a, st);
    const size_t es = a.dtype == MT_F32 ? 4 : 2;
    const bool igemm = is_gemm_kernel(a.kernel_id);
    for (int g = 0; g < a.groups; ++g) {
        OpArgs b = a;
        b.groups = 1;
        b.x_coff = a.x_coff + g * a.C;
        b.y_coff = a.y_coff + g * a.K;
        b.w = (const uint8_t *)a.w + (size_t)g * (igemm ? (size_t)a.n_pad * a.k_pad : (size_t)a.K * a.R * a.S * a.C) * es;
        b.bias = a.bias + (size_t)g * (igemm ? a.n_pad : a.K);
        if (a.res) b.res = (const uint8_t *)a.res + (size_t)g * a.K * es;
        const int e = launch_kernel(b, st);
        if (e != 0) return e;
    }
    return 0;
}

}  // namespace

static void retire_graphs(mt_ctx *ctx, mt_schedule *s) {
    if (s->graph_exec) ctx->retired_graphs.push_back(s->graph_exec);
    s->graph_exec = nullptr;
    for (auto &row : s->slice_exec)
        for (hipGraphExec_t g : row)
            if (g) ctx->retired_graphs.push_back(g);
    s->slice_exec.clear();
}

namespace {

int32_t launch_op(const OpArgs &a, hipStream_t st) {
    const int e = launch_raw(a, st);
    if (e != 0) return fail(MT_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString((hipError_t)e));
    return MT_OK;
}

inline OpArgs patched(const Tenant &t, int op, const void *in, void *out) {
    OpArgs a = t.args[op];
    if (t.reads_input[op]) a.x = in;
    if (t.res_input[op]) a.res = in;
    if (t.writes_output[op]) a.y = out;
    return a;
}

int32_t dispatch_latency_us(mt_ctx *ctx, hipStream_t st, uint32_t *scratch, int n, float *us);
int32_t concurrent_latency_us(mt_ctx *ctx, const std::vector<hipStream_t> &streams, int n, float *us, float *host_us);

// One issue item on its stream; returns a hipError_t as int.  An operator that runs inside its successor's launch
// (fuse 1) is skipped here; its neighbour launches the pair (fuse 2: depthwise + 1x1, fuse 3: 1x1 + depthwise, both from
// the second operator; fuse 4: convolution with the next operator, a 2x2 max pooling, in its epilogue).
int launch_item(const mt_ctx *ctx, const mt_schedule *s, const IssueItem &it, const void *const *inputs, void *const *outputs, hipStream_t st) {
    if (it.fuse == 1) return 0;
    const Tenant &t = *ctx->tenants[it.tenant];
    const int tp = s->prio[it.tenant];
    OpArgs a = patched(t, it.op, inputs[it.tenant], outputs[it.tenant]);
    // partial sums and arrival counters from the fixed scratch array instead of the arena
    auto redirect = [&](OpArgs &o) {
        if (!s->st_base || !o.ws) return;
        o.ws = (float *)(s->st_base + s->st_ws_base[it.tenant] + t.st_ws_off[it.op]);
        o.counters = (uint32_t *)(s->st_base + s->st_cnt_base[it.tenant] + t.st_cnt_off[it.op]);
    };
    redirect(a);
    a.prio = tp >= 0 ? tp : (t.short_kernel[it.op] || it.fuse == 2 || it.fuse == 3) ? 3 : 0;
    if (it.fuse == 2 || it.fuse == 3) {
        OpArgs prev = patched(t, it.op - 1, inputs[it.tenant], outputs[it.tenant]);
        prev.prio = a.prio;
        return it.fuse == 2 ? launch_dwpw(prev, a, st) : launch_pwdw(prev, a, st);
    }
    if (it.mates[0] >= 0) {
        OpArgs b[COISSUE_MAX - 1];
        int nm = 0;
        for (int k = 0; k < COISSUE_MAX - 1 && it.mates[k] >= 0; ++k, ++nm) {
            const int m = it.mates[k];
            const Tenant &tm = *ctx->tenants[m];
            b[k] = patched(tm, it.op, inputs[m], outputs[m]);
            if (s->st_base && b[k].ws) {
                b[k].ws = (float *)(s->st_base + s->st_ws_base[m] + tm.st_ws_off[it.op]);
                b[k].counters = (uint32_t *)(s->st_base + s->st_cnt_base[m] + tm.st_cnt_off[it.op]);
            }
            b[k].prio = a.prio;
        }
        return launch_kernel(a, st, b, nm);
    }
    if (it.fuse == 4) {
        OpArgs b = t.pool_args[it.op];
        b.prio = a.prio;
        redirect(b);
        if (t.reads_input[it.op]) b.x = inputs[it.tenant];
        if (t.writes_output[it.op + 1]) b.y = outputs[it.tenant];
        return launch_raw(b, st);
    }
    return launch_raw(a, st);
}

// Destroys every masked stream no schedule refers to, and the parked ones with them (the next masked streams are
// timed again, so a slow queue slot that becomes free is parked again when it comes up).
int32_t purge_idle_streams(mt_ctx *ctx) {
    HIP_TRY(hipDeviceSynchronize());
    for (auto e = ctx->streams.begin(); e != ctx->streams.end();) {
        if (e->second.refs == 0 && e->first.share != 0) {
            (void)hipStreamDestroy(e->second.stream);
            e = ctx->streams.erase(e);
        } else {
            ++e;
        }
    }
    for (hipStream_t p : ctx->parked_streams) (void)hipStreamDestroy(p);
    ctx->parked_streams.clear();
    return MT_OK;
}

// Plain streams belong to the process, not to a context: the runtime deals its hardware queues to the plain streams
// of the process in creation order, so every plain stream a context created and destroyed moved the turn of the next
// one.  One main stream and one stream per tenant index exist per device, created on first use and never destroyed;
// contexts of one process therefore share them (their work is ordered, not wrong).
//
// Which streams can run side by side: the hardware queues behind the streams are served by four dispatch pipes, and
// two queues of one pipe take turns (measured with chains of one-workgroup kernels: a pair of streams takes either one
// launch time per round, 10 us, or two, 20 us, nothing in between; the relation is transitive and twelve streams fall
// into four classes of sizes like 4 / 4 / 2 / 2, in no fixed order of creation).  A new plain stream is therefore
// classified by running it beside one representative of every class found so far, and tenant index i gets a stream
// of class i % 4: the streams of up to four tenants run side by side, those of eight are spread two per pipe.  Streams
// of a class nobody asked for yet wait in `spare`.
constexpr int N_PIPES = 4;
struct PlainPool {
    hipStream_t main_stream = nullptr;
    hipStream_t tenant[MT_MAX_TENANTS] = {};
    std::vector<hipStream_t> parked;
    std::vector<hipStream_t> rep;                   // one stream of every class, in the order the classes were found
    std::vector<std::vector<hipStream_t>> spare;    // per class: classified streams not handed out yet
};
PlainPool &plain_pool(int device) {
    static std::map<int, PlainPool> pools;
    return pools[device];
}

// Words of signal memory (what the queues' wait-for-value packets poll) belong to the process and are never freed:
// contexts borrow them and hand them back.  Memory of this kind that a kernel has touched is not given back to the
// allocator while the process runs.
struct SignalPool {
    std::mutex mu;
    std::map<int, std::vector<uint32_t *>> idle;     // per device
};
SignalPool &signal_pool() {
    static SignalPool p;
    return p;
}
int32_t take_signal_word(int device, uint32_t **out) {
    SignalPool &p = signal_pool();
    std::lock_guard<std::mutex> lk(p.mu);
    auto &v = p.idle[device];
    if (!v.empty()) { *out = v.back(); v.pop_back(); return MT_OK; }
    int can = 0;
    HIP_TRY(hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, device));
    if (!can) return fail(MT_ERR_HIP, "the device does not support stream memory operations");
    uint32_t *w = nullptr;
    HIP_TRY(hipExtMallocWithFlags((void **)&w, 8, hipMallocSignalMemory));    // this kind of memory comes in 8-byte allocations
    HIP_TRY(hipMemset(w, 0, 8));
    *out = w;
    return MT_OK;
}
void return_signal_word(int device, uint32_t *w) {
    if (!w) return;
    SignalPool &p = signal_pool();
    std::lock_guard<std::mutex> lk(p.mu);
    p.idle[device].push_back(w);
}

// Class of a new stream: the first class whose representative it cannot run beside (a round of both takes more than
// 1.5 launch times), else a new class, of which a plain stream becomes the representative (a masked one is reported
// as class -1 then).
int32_t classify_stream(mt_ctx *ctx, PlainPool &pool, hipStream_t s, bool plain, int *cls) {
    float single = 0.f;
    int32_t rc = dispatch_latency_us(ctx, s, ctx->probe_buf, 8, &single);
    if (rc != MT_OK) return rc;
    if (ctx->best_dispatch_us == 0.f || single < ctx->best_dispatch_us) ctx->best_dispatch_us = single;
    for (size_t c = 0; c < pool.rep.size(); ++c) {
        float us = 0.f, host_us = 0.f;
        rc = concurrent_latency_us(ctx, {pool.rep[c], s}, 8, &us, &host_us);
        if (rc != MT_OK) return rc;
        if (us > 1.5f * single) { *cls = (int)c; return MT_OK; }
    }
    if (!plain) { *cls = -1; return MT_OK; }
    *cls = (int)pool.rep.size();
    pool.rep.push_back(s);
    pool.spare.emplace_back();
    return MT_OK;
}

// Makes sure a representative of every pipe class exists (new plain streams go to the spare lists), so that masked
// streams can be classified; gives up after 12 creations.
int32_t discover_classes(mt_ctx *ctx) {
    PlainPool &pool = plain_pool(ctx->device);
    if (!ctx->probe_buf) HIP_TRY(hipMalloc((void **)&ctx->probe_buf, 256));
    for (int attempt = 0; attempt < 12 && (int)pool.rep.size() < N_PIPES; ++attempt) {
        hipStream_t s = nullptr;
        HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        int cls = 0;
        int32_t rc = classify_stream(ctx, pool, s, true, &cls);
        if (rc != MT_OK) { (void)hipStreamDestroy(s); return rc; }
        pool.spare[cls].push_back(s);
    }
    return MT_OK;
}

// A plain stream of class `want` (of any class after 16 creations that did not produce one).
int32_t plain_stream_of_class(mt_ctx *ctx, int want, hipStream_t *out) {
    PlainPool &pool = plain_pool(ctx->device);
    if (!ctx->probe_buf) HIP_TRY(hipMalloc((void **)&ctx->probe_buf, 256));
    for (int attempt = 0; attempt <= 16; ++attempt) {
        if (want < (int)pool.spare.size() && !pool.spare[want].empty()) {
            *out = pool.spare[want].back();
            pool.spare[want].pop_back();
            return MT_OK;
        }
        if (attempt == 16) break;
        hipStream_t s = nullptr;
        HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        int cls = 0;
        int32_t rc = classify_stream(ctx, pool, s, true, &cls);
        if (rc != MT_OK) { (void)hipStreamDestroy(s); return rc; }
        pool.spare[cls].push_back(s);
    }
    for (auto &v : pool.spare)
        if (!v.empty()) {
            *out = v.back();
            v.pop_back();
            return MT_OK;
        }
    return fail(MT_ERR_HIP, "no plain stream could be created");
}

// A new stream for `share` units starting at first_cu (0 = all units: a plain stream of the class of the tenant index).
int32_t make_stream(mt_ctx *ctx, int tenant, int share, int first_cu, hipStream_t *out) {
    // A stream over all units is a plain stream on one of the runtime's own hardware queues (GPU_MAX_HW_QUEUES of them,
    // dealt to the plain streams of the process in turn).  Giving it a full CU mask, and with it a queue of its own,
    // was measured and dropped: after the queue creations and destructions of a share search such streams sometimes
    // ran three tenants in 0.9 ms instead of 0.32 ms.
    if (share == 0) return plain_stream_of_class(ctx, tenant % N_PIPES, out);
    hipStream_t s = nullptr;
    const int cus = ctx->prop.multiProcessorCount;
    std::vector<uint32_t> mask((cus + 31) / 32, 0u);
    for (int j = 0; j < share; ++j) {
        const int cu = (first_cu + j) % cus;
        mask[cu / 32] |= 1u << (cu % 32);
    }
    // A masked stream owns a hardware queue, which sits on one of the four dispatch pipes like any other: it is
    // classified like a plain stream, and one of another class than the tenant index asks for (i % 4) is parked (kept
    // alive so that the next queue lands on the next pipe; purge_idle_streams destroys it later) and replaced, up to
    // seven times.
    int32_t rc = discover_classes(ctx);
    if (rc != MT_OK) return rc;
    PlainPool &pool = plain_pool(ctx->device);
    for (int attempt = 0;; ++attempt) {
        HIP_TRY(hipExtStreamCreateWithCUMask(&s, (uint32_t)mask.size(), mask.data()));
        int cls = -1;
        rc = classify_stream(ctx, pool, s, false, &cls);
        if (rc != MT_OK) { (void)hipStreamDestroy(s); return rc; }
        if (cls == tenant % N_PIPES || (int)pool.rep.size() < N_PIPES || attempt == 7) break;
        ctx->parked_streams.push_back(s);
    }
    *out = s;
    return MT_OK;
}

// Stream of a tenant restricted to `share` compute units (0 = all).  Tenant i's units start where the
// shares of the tenants before it end, so disjoint shares give disjoint units.
int32_t get_stream(mt_ctx *ctx, int tenant, int share, int first_cu, hipStream_t *out, StreamKey *out_key, bool *created = nullptr) {
    StreamKey key{tenant, share == 0 ? 0 : (first_cu << 12) | share};
    *out_key = key;
    auto it = ctx->streams.find(key);
    if (created) *created = false;
    if (it != ctx->streams.end()) { it->second.refs++; *out = it->second.stream; return MT_OK; }
    // A search over CU shares creates many masked streams, each with a hardware queue of its own.  Too many
    // queues make the hardware scheduler time-slice them, which slows every stream of the process and adds
    // stalls of 10-20 ms every few dozen runs: release the unreferenced masked streams before they pile up.  With the 8
    // queues of the plain streams, five or six masked queues alive were already enough to run three tenants on masked
    // streams in 0.80 ms instead of 0.32 ms.
    if (share != 0) {
        int idle = (int)ctx->parked_streams.size();
        for (auto &e : ctx->streams)
            if (e.second.refs == 0 && e.first.share != 0) ++idle;
        if (idle >= 3) {
            int32_t rc = purge_idle_streams(ctx);
            if (rc != MT_OK) return rc;
        }
    }
    PlainPool &pool = plain_pool(ctx->device);
    hipStream_t s = nullptr;
    if (share == 0 && pool.tenant[tenant]) {
        s = pool.tenant[tenant];                    // created by an earlier context of the process
    } else {
        int32_t rc = make_stream(ctx, tenant, share, first_cu, &s);
        if (rc != MT_OK) return rc;
        if (share == 0) pool.tenant[tenant] = s;
        if (created) *created = true;
    }
    ctx->streams[key] = mt_ctx::StreamEntry{s, 1};
    *out = s;
    return MT_OK;
}

void release_streams(mt_schedule *s) {
    if (!s->ctx) { s->stream_keys.clear(); return; }
    for (const StreamKey &k : s->stream_keys) {
        auto it = s->ctx->streams.find(k);
        if (it != s->ctx->streams.end() && it->second.refs > 0) it->second.refs--;
    }
    s->stream_keys.clear();
}

// A stream about to run stage st waits for the start event (no earlier work) or, directly, for the end of every other
// stream of the latest earlier stage with work; those streams waited the same way, so all earlier stages are complete.
// One cross-queue hop per barrier instead of two through the main stream.
// Under graph capture the barrier goes through the main stream as before (every stream waits for the stage event the
// main stream recorded): capturing the direct form ended in a host crash of the capture/instantiate path whose cause
// is not known, so that combination is switched off.
hipError_t wait_for_previous_stage(mt_ctx *ctx, const mt_schedule *s, int st, int stream) {
    if (s->flags & MT_SCHED_GRAPH)
        return hipStreamWaitEvent(s->stream_at[st][stream], st == 0 ? ctx->ev_start : ctx->ev_stage[st - 1], 0);
    const int prev = s->stages[st].prev_stage;
    if (prev < 0) return hipStreamWaitEvent(s->stream_at[st][stream], ctx->ev_start, 0);
    if (s->flags & MT_SCHED_COUNTER_BARRIER)      // one wait per stream: every stream of the stages so far has bumped the word
        return hipStreamWaitValue32(s->stream_at[st][stream], ctx->barrier_word, s->arrivals_upto[prev], hipStreamWaitValueGte, 0xffffffffu);
    hipError_t e = hipSuccess;
    for (int pm : s->stages[prev].streams)
        if (s->stream_at[prev][pm] != s->stream_at[st][stream] && e == hipSuccess)     // the same stream is in order by itself
            e = hipStreamWaitEvent(s->stream_at[st][stream], ctx->ev_done[prev][pm], 0);
    return e;
}

// Outside whole-schedule graph capture the main stream takes no part in a run after the start event: the events that
// end a stage on its streams are timed, the streams of the next stage wait for them directly, the host waits for those
// of the last stage that launches anything, and stage times are differences of these events.  A queue that sits in a
// wait for another queue's event slows the dispatch of the others on this machine: with the main stream joining every
// stage for a stage event of its own, the sequential ResNet-18 + VGG-16 + MobileNetV2 pass took 0.62 instead of 0.56 ms
// and the concurrent one 0.325 instead of 0.30 ms.
inline bool ends_on_streams(const mt_schedule *s) { return !(s->flags & MT_SCHED_GRAPH) && s->end_stage >= 0; }

// MT_SCHED_STREAM_GRAPHS: the launches of one stream in one stage, captured on that stream (so that a CU mask of the
// stream applies at replay) into a graph of their own.  The barriers between stages stay ordinary events.
int32_t capture_slice_graphs(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs) {
    retire_graphs(ctx, s);
    s->slice_exec.assign(s->n_stages, {});
    for (int st = 0; st < s->n_stages; ++st) {
        const StagePlan &sp = s->stages[st];
        for (int sm : sp.streams) {
            hipStream_t stream = s->stream_at[st][sm];
            hipGraph_t graph = nullptr;
            HIP_TRY(hipStreamBeginCapture(stream, hipStreamCaptureModeRelaxed));
            int32_t rc = MT_OK;
            for (const IssueItem &it : sp.by_stream[sm]) {
                const int e = launch_item(ctx, s, it, inputs, outputs, stream);
                if (e != 0) { rc = fail(MT_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString((hipError_t)e)); break; }
            }
            hipError_t e = hipStreamEndCapture(stream, &graph);
            if (rc != MT_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
            if (e != hipSuccess) return fail(MT_ERR_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
            e = hipGraphInstantiate(&s->slice_exec[st][sm], graph, nullptr, nullptr, 0);
            (void)hipGraphDestroy(graph);
            if (e != hipSuccess) return fail(MT_ERR_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e));
        }
    }
    s->cap_in.assign(inputs, inputs + s->n_tenants);
    s->cap_out.assign(outputs, outputs + s->n_tenants);
    return MT_OK;
}

// Issues the whole schedule on the tenant streams.  Barrier between stages: every stream of the stage records an
// event and the streams of the next stage wait for all of them.  Under whole-schedule graph capture the main stream
// waits for them too and records a stage event that the next stage waits for (a capture has to join its origin).
int32_t issue_schedule(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, int *n_launch, bool alt = false) {
    if (s->flags & MT_SCHED_COUNTER_BARRIER) HIP_TRY(hipStreamWriteValue32(ctx->main_stream, ctx->barrier_word, 0u, 0));
    HIP_TRY(hipEventRecord(ctx->ev_start, ctx->main_stream));
    int launches = 0;
    for (int st = 0; st < s->n_stages; ++st) {
        const StagePlan &sp = s->stages[st];
        for (int sm : sp.streams) HIP_TRY(wait_for_previous_stage(ctx, s, st, sm));
        if (s->flags & MT_SCHED_STREAM_GRAPHS) {
            for (int sm : sp.streams) HIP_TRY(hipGraphLaunch(s->slice_exec[st][sm], s->stream_at[st][sm]));
            launches += (int)sp.items.size();
        } else
        for (const IssueItem &it : (alt ? s->alt_items[st] : sp.items)) {
            ++launches;                              // counts operators issued, fused or not
            const int e = launch_item(ctx, s, it, inputs, outputs, s->stream_at[st][it.stream]);
            if (e != 0) return fail(MT_ERR_HIP, std::string("kernel launch: ") + hipGetErrorString((hipError_t)e));
            if ((s->flags & MT_SCHED_TIME_FIRST_OP) && it.op == 0) HIP_TRY(hipEventRecord(ctx->ev_first[it.tenant], s->stream_at[st][it.stream]));
            if ((s->flags & MT_SCHED_TIME_TENANTS) && it.op + 1 == (int)ctx->tenants[it.tenant]->model.ops.size())
                HIP_TRY(hipEventRecord(ctx->ev_last[it.tenant], s->stream_at[st][it.stream]));
        }
        if (ends_on_streams(s)) {
            for (int sm : sp.streams) HIP_TRY(hipEventRecord(ctx->ev_done[st][sm], s->stream_at[st][sm]));
            if ((s->flags & MT_SCHED_COUNTER_BARRIER) && st < s->end_stage)
                for (int sm : sp.streams) {
                    const int e = launch_arrive(ctx->barrier_word, s->stream_at[st][sm]);
                    if (e != 0) return fail(MT_ERR_HIP, std::string("arrival kernel: ") + hipGetErrorString((hipError_t)e));
                }
            continue;
        }
        for (int sm : sp.streams) {
            HIP_TRY(hipEventRecord(ctx->ev_done[st][sm], s->stream_at[st][sm]));
            HIP_TRY(hipStreamWaitEvent(ctx->main_stream, ctx->ev_done[st][sm], 0));
        }
        HIP_TRY(hipEventRecord(ctx->ev_stage[st], ctx->main_stream));
    }
    if (n_launch) *n_launch = launches;
    return MT_OK;
}

inline void spin_pause() {
#if defined(__x86_64__)
    __builtin_ia32_pause();
#endif
}

// `seen` is the run counter at the time the thread was created: a worker added after earlier runs (a tenant
// registered later) must sleep until the next run is published, not wake for the last one, whose schedule may be gone.
void issue_worker(mt_ctx *ctx, int w, uint64_t seen) {
    IssuePool &pool = ctx->pool;
    (void)hipSetDevice(ctx->device);
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(pool.mu);
            pool.cv.wait(lk, [&] { return pool.quit || pool.run_seq != seen; });
            if (pool.quit) return;
            seen = pool.run_seq;
        }
        mt_schedule *s = pool.sched;
        if (w < s->n_tenants) {
            for (int st = 0; st < s->n_stages; ++st) {
                const StagePlan &sp = s->stages[st];
                if (sp.by_stream[w].empty()) continue;
                while (pool.stage_posted.load(std::memory_order_acquire) < st) spin_pause();
                hipError_t e = hipSuccess;
                const int prev = sp.prev_stage;
                if ((s->flags & MT_SCHED_HOST_BARRIER) && prev >= 0) {
                    // the barrier on the host: once every stream of the stage before has recorded its event, this
                    // thread waits for those of the other streams and only then launches
                    const StagePlan &pp = s->stages[prev];
                    while (pool.stage_done[prev].load(std::memory_order_acquire) < (int)pp.streams.size()) spin_pause();
                    for (int pm : pp.streams)
                        if (s->stream_at[prev][pm] != s->stream_at[st][w] && e == hipSuccess) e = hipEventSynchronize(ctx->ev_done[prev][pm]);
                } else {
                    e = wait_for_previous_stage(ctx, s, st, w);
                }
                for (const IssueItem &it : sp.by_stream[w]) {
                    if (e != hipSuccess) break;
                    const int rc = launch_item(ctx, s, it, pool.inputs, pool.outputs, s->stream_at[st][w]);
                    if (rc != 0) e = (hipError_t)rc;
                    else if ((s->flags & MT_SCHED_TIME_TENANTS) && it.op + 1 == (int)ctx->tenants[it.tenant]->model.ops.size())
                        e = hipEventRecord(ctx->ev_last[it.tenant], s->stream_at[st][w]);
                }
                if (e == hipSuccess) e = hipEventRecord(ctx->ev_done[st][w], s->stream_at[st][w]);
                if (e == hipSuccess && (s->flags & MT_SCHED_COUNTER_BARRIER) && st < s->end_stage)
                    e = (hipError_t)launch_arrive(ctx->barrier_word, s->stream_at[st][w]);
                if (e != hipSuccess) {
                    std::lock_guard<std::mutex> lk(pool.mu);
                    pool.error_msg = std::string("issuing thread: ") + hipGetErrorString(e);
                    pool.error.store(1);
                }
                pool.stage_done[st].fetch_add(1, std::memory_order_release);
            }
        }
        pool.finished.fetch_add(1, std::memory_order_release);
    }
}

int32_t ensure_pool(mt_ctx *ctx, int n) {
    while ((int)ctx->pool.threads.size() < n) {
        const int w = (int)ctx->pool.threads.size();
        uint64_t seq;
        {
            std::lock_guard<std::mutex> lk(ctx->pool.mu);
            seq = ctx->pool.run_seq;
        }
        ctx->pool.threads.emplace_back(issue_worker, ctx, w, seq);
    }
    return MT_OK;
}

void stop_pool(mt_ctx *ctx) {
    {
        std::lock_guard<std::mutex> lk(ctx->pool.mu);
        ctx->pool.quit = true;
    }
    ctx->pool.cv.notify_all();
    for (auto &t : ctx->pool.threads) t.join();
    ctx->pool.threads.clear();
}

// Same event structure as issue_schedule, with the launches of a stage spread over one host thread per stream.
int32_t issue_schedule_parallel(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, int *n_launch) {
    IssuePool &pool = ctx->pool;
    int32_t rc = ensure_pool(ctx, s->n_tenants);
    if (rc != MT_OK) return rc;
    const int n_workers = (int)pool.threads.size();
    pool.sched = s;
    pool.inputs = inputs;
    pool.outputs = outputs;
    pool.stage_posted.store(-1);
    for (int st = 0; st < MT_MAX_STAGES; ++st) pool.stage_done[st].store(0);
    pool.finished.store(0);
    pool.error.store(0);
    if (s->flags & MT_SCHED_COUNTER_BARRIER) HIP_TRY(hipStreamWriteValue32(ctx->main_stream, ctx->barrier_word, 0u, 0));
    HIP_TRY(hipEventRecord(ctx->ev_start, ctx->main_stream));
    {
        std::lock_guard<std::mutex> lk(pool.mu);
        ++pool.run_seq;
    }
    pool.cv.notify_all();
    hipError_t err = hipSuccess;
    for (int st = 0; st < s->n_stages; ++st) {
        const StagePlan &sp = s->stages[st];
        pool.stage_posted.store(st, std::memory_order_release);
        while (pool.stage_done[st].load(std::memory_order_acquire) < (int)sp.streams.size()) spin_pause();
        if (ends_on_streams(s)) continue;          // stages end on their own streams' events
        for (int sm : sp.streams)
            if (err == hipSuccess) err = hipStreamWaitEvent(ctx->main_stream, ctx->ev_done[st][sm], 0);
        if (err == hipSuccess) err = hipEventRecord(ctx->ev_stage[st], ctx->main_stream);
    }
    while (pool.finished.load(std::memory_order_acquire) < n_workers) spin_pause();
    pool.sched = nullptr;                      // every worker has left the run; nothing may look at the schedule again
    pool.inputs = nullptr;
    pool.outputs = nullptr;
    if (pool.error.load()) {
        std::lock_guard<std::mutex> lk(pool.mu);
        return fail(MT_ERR_HIP, pool.error_msg);
    }
    if (err != hipSuccess) return fail(MT_ERR_HIP, std::string("parallel issue: ") + hipGetErrorString(err));
    if (n_launch) *n_launch = s->n_launches;
    return MT_OK;
}

}  // namespace

// ============================================================================================
extern "C" {

const char *mt_kernel_name(int32_t id) {
    switch (id) {
        case K_CONV_DIRECT: return "conv_direct";
        case K_IGEMM_128x128: return "igemm_128x128";
        case K_IGEMM_128x64: return "igemm_128x64";
        case K_IGEMM_64x64: return "igemm_64x64";
        case K_IGEMM_64x16: return "igemm_64x16";
        case K_IGEMM_PW: return "igemm_pointwise";
        case K_STEM: return "stem_rows";
        case K_ROWB: return "igemm_resident_filters";
        case K_PCONV: return "igemm_patch_64x64";
        case K_DWCONV: return "dwconv";
        case K_MAXPOOL: return "maxpool";
        case K_AVGPOOL: return "avgpool";
        case K_GAP: return "global_avgpool";
        case K_GEMV: return "gemv";
        case K_LRN: return "lrn";
        case K_ADD: return "add";
    }
    return "unknown";
}

int32_t mt_create(int32_t device, mt_ctx **out) {
    if (!out) return fail(MT_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int count = 0;
    HIP_TRY(hipGetDeviceCount(&count));
    if (device < 0 || device >= count) return fail(MT_ERR_INVALID_ARG, "no such device");
    HIP_TRY(hipSetDevice(device));
    std::unique_ptr<mt_ctx> c(new mt_ctx);
    c->device = device;
    HIP_TRY(hipGetDeviceProperties(&c->prop, device));
    {
        PlainPool &pool = plain_pool(device);
        if (!pool.main_stream) HIP_TRY(hipStreamCreateWithFlags(&pool.main_stream, hipStreamNonBlocking));
        c->main_stream = pool.main_stream;
    }
    HIP_TRY(hipEventCreate(&c->ev_start));
    for (int s = 0; s < MT_MAX_STAGES; ++s) {
        HIP_TRY(hipEventCreate(&c->ev_stage[s]));
        for (int t = 0; t < MT_MAX_TENANTS; ++t) HIP_TRY(hipEventCreate(&c->ev_done[s][t]));
    }
    for (int t = 0; t < MT_MAX_TENANTS; ++t) HIP_TRY(hipEventCreate(&c->ev_first[t]));
    for (int t = 0; t < MT_MAX_TENANTS; ++t) HIP_TRY(hipEventCreate(&c->ev_last[t]));
    HIP_TRY(hipEventCreate(&c->ev_prof[0]));
    HIP_TRY(hipEventCreate(&c->ev_prof[1]));
    *out = c.release();
    return MT_OK;
}

int32_t mt_destroy(mt_ctx *ctx) {
    if (!ctx) return fail(MT_ERR_INVALID_ARG, "ctx is NULL");
    (void)hipSetDevice(ctx->device);
    stop_pool(ctx);
    (void)hipDeviceSynchronize();
    for (mt_schedule *ls : ctx->live_schedules) {
        retire_graphs(ctx, ls);
        ls->ctx = nullptr;
    }
    for (hipGraphExec_t g : ctx->retired_graphs) (void)hipGraphExecDestroy(g);
    for (auto &kv : ctx->streams)
        if (kv.first.share != 0) (void)hipStreamDestroy(kv.second.stream);       // plain streams belong to the process
    for (hipStream_t ps : ctx->parked_streams) (void)hipStreamDestroy(ps);
    if (ctx->probe_buf) (void)hipFree(ctx->probe_buf);
    return_signal_word(ctx->device, ctx->barrier_word);
    if (ctx->ev_start) (void)hipEventDestroy(ctx->ev_start);
    for (int s = 0; s < MT_MAX_STAGES; ++s) {
        if (ctx->ev_stage[s]) (void)hipEventDestroy(ctx->ev_stage[s]);
        for (int t = 0; t < MT_MAX_TENANTS; ++t)
            if (ctx->ev_done[s][t]) (void)hipEventDestroy(ctx->ev_done[s][t]);
    }
    for (auto e : ctx->ev_first)
        if (e) (void)hipEventDestroy(e);
    for (auto e : ctx->ev_last)
        if (e) (void)hipEventDestroy(e);
    for (auto e : ctx->ev_prof)
        if (e) (void)hipEventDestroy(e);
    for (auto &t : ctx->tenants)
        if (t->owns_arena && t->arena) (void)hipFree(t->arena);
    delete ctx;
    return MT_OK;
}

// Graph executables of destroyed schedules are released in batches, each after a device-wide synchronisation, so that a
// long search under graph replay (two instantiated graphs per candidate) does not keep them all until mt_destroy.
static int32_t release_retired_graphs(mt_ctx *ctx) {
    if (ctx->retired_graphs.empty()) return MT_OK;
    HIP_TRY(hipDeviceSynchronize());
    for (hipGraphExec_t g : ctx->retired_graphs) (void)hipGraphExecDestroy(g);
    ctx->retired_graphs.clear();
    return MT_OK;
}

int32_t mt_release_idle_streams(mt_ctx *ctx) {
    if (!ctx) return fail(MT_ERR_INVALID_ARG, "ctx is NULL");
    HIP_TRY(hipSetDevice(ctx->device));
    int32_t rc = release_retired_graphs(ctx);
    if (rc != MT_OK) return rc;
    return purge_idle_streams(ctx);
}

int32_t mt_get_device_info(const mt_ctx *ctx, mt_device_info *out) {
    if (!ctx || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    std::memset(out, 0, sizeof(*out));
    out->cu_count = ctx->prop.multiProcessorCount;
    out->wavefront_size = ctx->prop.warpSize;
    out->lds_bytes_per_block = (int32_t)ctx->prop.sharedMemPerBlock;
    out->clock_khz = ctx->prop.clockRate;
    out->l2_bytes = ctx->prop.l2CacheSize;
    out->hbm_bytes = (int64_t)ctx->prop.totalGlobalMem;
    std::strncpy(out->name, ctx->prop.name, sizeof(out->name) - 1);
    std::strncpy(out->arch, ctx->prop.gcnArchName, sizeof(out->arch) - 1);
    return MT_OK;
}

int32_t mt_probe_cu_mask(mt_ctx *ctx, int32_t share, int32_t first_cu, int32_t n_groups, uint32_t *hw_ids) {
    if (!ctx || !hw_ids) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    const int cus = ctx->prop.multiProcessorCount;
    if (share < 0 || share > cus || first_cu < 0 || first_cu >= cus || n_groups < 1 || n_groups > (1 << 20))
        return fail(MT_ERR_INVALID_ARG, "share, first_cu or n_groups out of range");
    HIP_TRY(hipSetDevice(ctx->device));
    hipStream_t st = nullptr;
    if (share == 0) {
        HIP_TRY(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    } else {
        std::vector<uint32_t> mask((cus + 31) / 32, 0u);
        for (int j = 0; j < share; ++j) {
            const int cu = (first_cu + j) % cus;
            mask[cu / 32] |= 1u << (cu % 32);
        }
        HIP_TRY(hipExtStreamCreateWithCUMask(&st, (uint32_t)mask.size(), mask.data()));
    }
    uint32_t *dev = nullptr;
    hipError_t e = hipMalloc((void **)&dev, sizeof(uint32_t) * 2 * n_groups);
    if (e == hipSuccess) {
        int rc = launch_probe(dev, n_groups, st);
        e = rc ? (hipError_t)rc : hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipMemcpy(hw_ids, dev, sizeof(uint32_t) * 2 * n_groups, hipMemcpyDeviceToHost);
        (void)hipFree(dev);
    }
    (void)hipStreamDestroy(st);
    if (e != hipSuccess) return fail(MT_ERR_HIP, std::string("probe: ") + hipGetErrorString(e));
    return MT_OK;
}

namespace {
// Mean time per launch of n dependent one-workgroup kernels on `st`, measured the way a stage runs: the main stream
// records a start event, the stream waits for it, runs, records its done event, the host waits for that.
int32_t dispatch_latency_us(mt_ctx *ctx, hipStream_t st, uint32_t *scratch, int n, float *us) {
    for (int rep = 0; rep < 2; ++rep) {          // first pass warms up
        HIP_TRY(hipEventRecord(ctx->ev_prof[0], ctx->main_stream));
        HIP_TRY(hipStreamWaitEvent(st, ctx->ev_prof[0], 0));
        for (int i = 0; i < n; ++i) {
            int rc = launch_probe(scratch, 1, st);
            if (rc) return fail(MT_ERR_HIP, std::string("probe launch: ") + hipGetErrorString((hipError_t)rc));
        }
        HIP_TRY(hipEventRecord(ctx->ev_done[0][0], st));
        HIP_TRY(hipEventSynchronize(ctx->ev_done[0][0]));
    }
    float ms = 0;
    HIP_TRY(hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_done[0][0]));
    *us = ms * 1e3f / n;
    return MT_OK;
}
// Time per round of n rounds in which every stream of the list launches one probe kernel, all chains running at once;
// host_us: the time the issuing thread needed per round (with many streams the launches themselves bound the round).
int32_t concurrent_latency_us(mt_ctx *ctx, const std::vector<hipStream_t> &streams, int n, float *us, float *host_us) {
    const int m = (int)streams.size();
    if (m < 1 || m > MT_MAX_TENANTS) return fail(MT_ERR_INVALID_ARG, "stream count out of range");
    if (!ctx->probe_buf) HIP_TRY(hipMalloc((void **)&ctx->probe_buf, 256));
    float host = 0.f, worst = 0.f;
    // Measured the way mt_run measures a stage: the main stream only records the start, every stream records its own
    // end, the host waits for those; no queue sits in a wait for another queue while the chains run.
    for (int rep = 0; rep < 2; ++rep) {
        HIP_TRY(hipEventRecord(ctx->ev_prof[0], ctx->main_stream));
        for (int j = 0; j < m; ++j) HIP_TRY(hipStreamWaitEvent(streams[j], ctx->ev_prof[0], 0));
        const auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < m; ++j) {
                int rc = launch_probe(ctx->probe_buf + 2 * j, 1, streams[j]);
                if (rc) return fail(MT_ERR_HIP, std::string("probe launch: ") + hipGetErrorString((hipError_t)rc));
            }
        host = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count() / n;
        for (int j = 0; j < m; ++j) HIP_TRY(hipEventRecord(ctx->ev_done[0][j], streams[j]));
        worst = 0.f;
        for (int j = 0; j < m; ++j) {
            HIP_TRY(hipEventSynchronize(ctx->ev_done[0][j]));
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_done[0][j]));
            worst = std::max(worst, ms);
        }
    }
    *us = worst * 1e3f / n;
    *host_us = host;
    return MT_OK;
}
}  // namespace

int32_t mt_probe_dispatch_latency(mt_ctx *ctx, int32_t n_streams, int32_t share, int32_t n_launches, float *us_per_launch) {
    if (!ctx || !us_per_launch) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    const int cus = ctx->prop.multiProcessorCount;
    if (n_streams < 1 || n_streams > 64 || n_launches < 1 || share < 0 || share > cus) return fail(MT_ERR_INVALID_ARG, "argument out of range");
    HIP_TRY(hipSetDevice(ctx->device));
    std::vector<hipStream_t> streams;
    uint32_t *dev = nullptr;
    HIP_TRY(hipMalloc((void **)&dev, 64));
    int32_t rc = MT_OK;
    for (int i = 0; i < n_streams && rc == MT_OK; ++i) {
        hipStream_t st = nullptr;
        hipError_t e;
        if (share == 0) {
            e = hipStreamCreateWithFlags(&st, hipStreamNonBlocking);
        } else {
            std::vector<uint32_t> mask((cus + 31) / 32, 0u);
            for (int j = 0; j < share; ++j) mask[j / 32] |= 1u << (j % 32);
            e = hipExtStreamCreateWithCUMask(&st, (uint32_t)mask.size(), mask.data());
        }
        if (e != hipSuccess) { rc = fail(MT_ERR_HIP, std::string("stream create: ") + hipGetErrorString(e)); break; }
        streams.push_back(st);
        rc = dispatch_latency_us(ctx, st, dev, n_launches, &us_per_launch[i]);
    }
    (void)hipDeviceSynchronize();
    for (hipStream_t st : streams) (void)hipStreamDestroy(st);
    (void)hipFree(dev);
    return rc;
}

int32_t mt_probe_stream_conflicts(mt_ctx *ctx, int32_t n_streams, int32_t n_launches, float *single_us, float *pair_us) {
    if (!ctx || !single_us || !pair_us) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_streams < 2 || n_streams > 32 || n_launches < 1 || n_launches > 256) return fail(MT_ERR_INVALID_ARG, "argument out of range");
    HIP_TRY(hipSetDevice(ctx->device));
    if (!ctx->probe_buf) HIP_TRY(hipMalloc((void **)&ctx->probe_buf, 256));
    std::vector<hipStream_t> streams;
    int32_t rc = MT_OK;
    for (int i = 0; i < n_streams && rc == MT_OK; ++i) {
        hipStream_t st = nullptr;
        hipError_t e = hipStreamCreateWithFlags(&st, hipStreamNonBlocking);
        if (e != hipSuccess) { rc = fail(MT_ERR_HIP, std::string("stream create: ") + hipGetErrorString(e)); break; }
        streams.push_back(st);
        rc = dispatch_latency_us(ctx, st, ctx->probe_buf, n_launches, &single_us[i]);
    }
    for (int i = 0; i < n_streams && rc == MT_OK; ++i)
        for (int j = 0; j < n_streams && rc == MT_OK; ++j) {
            if (j <= i) { pair_us[i * n_streams + j] = j == i ? single_us[i] : pair_us[j * n_streams + i]; continue; }
            float host_us = 0.f;
            rc = concurrent_latency_us(ctx, {streams[i], streams[j]}, n_launches, &pair_us[i * n_streams + j], &host_us);
        }
    (void)hipDeviceSynchronize();
    for (hipStream_t st : streams) (void)hipStreamDestroy(st);
    return rc;
}

int32_t mt_probe_barrier_cost(mt_ctx *ctx, int32_t n_streams, int32_t kind, int32_t rounds, float *us_per_round) {
    if (!ctx || !us_per_round) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (n_streams < 1 || n_streams > MT_MAX_TENANTS || kind < 0 || kind > 4 || rounds < 1 || rounds > 4096)
        return fail(MT_ERR_INVALID_ARG, "argument out of range");
    HIP_TRY(hipSetDevice(ctx->device));
    if (kind == 2 || kind == 3) {
        int can = 0;
        HIP_TRY(hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, ctx->device));
        if (!can) return fail(MT_ERR_HIP, "the device does not support stream memory operations");
    }
    // the plain tenant streams of the process, as mt_run uses them
    std::vector<hipStream_t> st(n_streams);
    std::vector<StreamKey> keys(n_streams);
    for (int i = 0; i < n_streams; ++i) {
        int32_t rc = get_stream(ctx, i, 0, 0, &st[i], &keys[i]);
        if (rc != MT_OK) return rc;
    }
    auto release = [&]() {
        for (int i = 0; i < n_streams; ++i) {
            auto it = ctx->streams.find(keys[i]);
            if (it != ctx->streams.end() && it->second.refs > 0) it->second.refs--;
        }
    };
    if (!ctx->probe_buf) HIP_TRY(hipMalloc((void **)&ctx->probe_buf, 256));
    // one word per stream (kind 2) or one in all (kind 3), borrowed from the process's pool and zeroed by the host
    uint32_t *words[MT_MAX_TENANTS] = {};
    auto free_words = [&]() {
        for (uint32_t *w : words) return_signal_word(ctx->device, w);
    };
    for (int i = 0; (kind == 2 || (kind == 3 && i == 0)) && i < n_streams; ++i) {
        int32_t rc = take_signal_word(ctx->device, &words[i]);
        hipError_t e = rc == MT_OK ? hipMemset(words[i], 0, 8) : hipSuccess;
        if (rc != MT_OK || e != hipSuccess) {
            free_words(); release();
            return rc != MT_OK ? rc : fail(MT_ERR_HIP, std::string("signal memory: ") + hipGetErrorString(e));
        }
    }
    hipError_t e = hipSuccess;
    float ms = 0.f;
    uint32_t epoch = 0;
    for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {                   // first pass warms up
        e = hipEventRecord(ctx->ev_prof[0], ctx->main_stream);
        for (int i = 0; i < n_streams && e == hipSuccess; ++i) e = hipStreamWaitEvent(st[i], ctx->ev_prof[0], 0);
        for (int r = 0; r < rounds && e == hipSuccess; ++r) {
            ++epoch;
            for (int i = 0; i < n_streams && e == hipSuccess; ++i) e = (hipError_t)launch_probe(ctx->probe_buf + 2 * i, 1, st[i]);
            if (kind == 1) {
                hipEvent_t *ev = ctx->ev_done[r & 1];                        // two event sets alternate between rounds
                for (int i = 0; i < n_streams && e == hipSuccess; ++i) e = hipEventRecord(ev[i], st[i]);
                for (int i = 0; i < n_streams; ++i)
                    for (int j = 0; j < n_streams && e == hipSuccess; ++j)
                        if (j != i) e = hipStreamWaitEvent(st[i], ev[j], 0);
            } else if (kind == 2) {
                for (int i = 0; i < n_streams && e == hipSuccess; ++i) e = hipStreamWriteValue32(st[i], words[i], epoch, 0);
                for (int i = 0; i < n_streams; ++i)
                    for (int j = 0; j < n_streams && e == hipSuccess; ++j)
                        if (j != i) e = hipStreamWaitValue32(st[i], words[j], epoch, hipStreamWaitValueGte, 0xffffffffu);
            }
            else if (kind == 3) {
                for (int i = 0; i < n_streams && e == hipSuccess; ++i) e = (hipError_t)launch_arrive(words[0], st[i]);
                for (int i = 0; i < n_streams && e == hipSuccess; ++i)
                    e = hipStreamWaitValue32(st[i], words[0], epoch * (uint32_t)n_streams, hipStreamWaitValueGte, 0xffffffffu);
            } else if (kind == 4) {
                hipEvent_t *ev = ctx->ev_done[r & 1];
                for (int i = 0; i < n_streams && e == hipSuccess; ++i) {
                    e = hipEventRecord(ev[i], st[i]);
                    if (e == hipSuccess) e = hipStreamWaitEvent(ctx->main_stream, ev[i], 0);
                }
                if (e == hipSuccess) e = hipEventRecord(ctx->ev_stage[r & 1], ctx->main_stream);
                for (int i = 0; i < n_streams && e == hipSuccess; ++i) e = hipStreamWaitEvent(st[i], ctx->ev_stage[r & 1], 0);
            }
        }
        for (int i = 0; i < n_streams && e == hipSuccess; ++i) {
            e = hipEventRecord(ctx->ev_done[2][i], st[i]);
            if (e == hipSuccess) e = hipStreamWaitEvent(ctx->main_stream, ctx->ev_done[2][i], 0);
        }
        if (e == hipSuccess) e = hipEventRecord(ctx->ev_prof[1], ctx->main_stream);
        if (e == hipSuccess) e = hipEventSynchronize(ctx->ev_prof[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_prof[1]);
    }
    (void)hipDeviceSynchronize();
    free_words();
    release();
    if (e != hipSuccess) return fail(MT_ERR_HIP, std::string("barrier probe: ") + hipGetErrorString(e));
    *us_per_round = ms * 1e3f / (float)rounds;
    return MT_OK;
}

int32_t mt_probe_peak_mfma(mt_ctx *ctx, int32_t dtype, int32_t iters, float *tflops) {
    if (!ctx || !tflops) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (dtype != MT_F16 && dtype != MT_BF16) return fail(MT_ERR_INVALID_ARG, "the matrix-instruction loop exists for fp16 and bf16");
    if (iters < 1 || iters > (1 << 20)) return fail(MT_ERR_INVALID_ARG, "iters out of range (1 .. 2^20)");
    HIP_TRY(hipSetDevice(ctx->device));
    const int n_groups = ctx->prop.multiProcessorCount * 2;        // two workgroups of four waves per unit: two waves per SIMD
    float *sink = nullptr;
    HIP_TRY(hipMalloc((void **)&sink, (size_t)n_groups * 256 * sizeof(float)));
    int32_t rc = MT_OK;
    float ms = 0;
    for (int rep = 0; rep < 2 && rc == MT_OK; ++rep) {             // first pass warms up
        hipError_t e = hipEventRecord(ctx->ev_prof[0], ctx->main_stream);
        if (e == hipSuccess) e = (hipError_t)launch_peak_mfma(dtype, sink, n_groups, iters, ctx->main_stream);
        if (e == hipSuccess) e = hipEventRecord(ctx->ev_prof[1], ctx->main_stream);
        if (e == hipSuccess) e = hipEventSynchronize(ctx->ev_prof[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_prof[1]);
        if (e != hipSuccess) rc = fail(MT_ERR_HIP, std::string("peak probe: ") + hipGetErrorString(e));
    }
    (void)hipFree(sink);
    if (rc != MT_OK) return rc;
    const double flops = (double)n_groups * 4 /*waves*/ * 4 /*accumulators*/ * (double)iters * 2.0 * 32 * 32 * 16;
    *tflops = (float)(flops / (ms * 1e-3) / 1e12);
    return MT_OK;
}

int32_t mt_probe_peak_stream(mt_ctx *ctx, int32_t mode, size_t bytes, int32_t groups_per_unit, int32_t reps, float *gbytes_per_s) {
    if (!ctx || !gbytes_per_s) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (mode != 0 && mode != 1) return fail(MT_ERR_INVALID_ARG, "mode is 0 (copy) or 1 (read)");
    if (bytes < ((size_t)1 << 20) || bytes > ((size_t)8 << 30) || bytes % 16 != 0)
        return fail(MT_ERR_INVALID_ARG, "bytes must be a multiple of 16 between 1 MiB and 8 GiB");
    if (reps < 1 || reps > 1000) return fail(MT_ERR_INVALID_ARG, "reps out of range (1 .. 1000)");
    if (groups_per_unit < 1 || groups_per_unit > 256) return fail(MT_ERR_INVALID_ARG, "groups_per_unit out of range (1 .. 256)");
    HIP_TRY(hipSetDevice(ctx->device));
    const int n_groups = ctx->prop.multiProcessorCount * groups_per_unit;
    const size_t dst_bytes = mode == 0 ? bytes : (size_t)n_groups * 256 * sizeof(uint32_t);
    void *src = nullptr, *dst = nullptr;
    HIP_TRY(hipMalloc(&src, bytes));
    if (hipMalloc(&dst, dst_bytes) != hipSuccess) { (void)hipFree(src); return fail(MT_ERR_OUT_OF_MEMORY, "peak probe: destination buffer"); }
    hipError_t e = (hipError_t)launch_fill_u32((uint32_t *)src, bytes / 4, 0x3c003c00u, ctx->main_stream);
    float ms = 0;
    for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {         // first pass warms up
        e = hipEventRecord(ctx->ev_prof[0], ctx->main_stream);
        for (int i = 0; i < reps && e == hipSuccess; ++i) e = (hipError_t)launch_peak_stream(mode, src, dst, bytes, n_groups, ctx->main_stream);
        if (e == hipSuccess) e = hipEventRecord(ctx->ev_prof[1], ctx->main_stream);
        if (e == hipSuccess) e = hipEventSynchronize(ctx->ev_prof[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_prof[1]);
    }
    (void)hipDeviceSynchronize();
    (void)hipFree(src);
    (void)hipFree(dst);
    if (e != hipSuccess) return fail(MT_ERR_HIP, std::string("peak probe: ") + hipGetErrorString(e));
    const double moved = (double)bytes * (mode == 0 ? 2.0 : 1.0) * reps;
    *gbytes_per_s = (float)(moved / (ms * 1e-3) / 1e9);
    return MT_OK;
}

// ---- model ---------------------------------------------------------------------------------
int32_t mt_model_begin(int32_t dtype, int32_t batch, int32_t in_h, int32_t in_w, int32_t in_c, mt_model **out) {
    if (!out) return fail(MT_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (dtype < MT_F32 || dtype > MT_BF16) return fail(MT_ERR_INVALID_ARG, "unknown storage type");
    if (batch < 1 || in_h < 1 || in_w < 1 || in_c < 1) return fail(MT_ERR_INVALID_ARG, "batch and input dimensions must be >= 1");
    mt_model *m = new mt_model;
    m->dtype = dtype; m->batch = batch; m->in_h = in_h; m->in_w = in_w; m->in_c = in_c;
    *out = m;
    return MT_OK;
}

int32_t mt_model_add_op(mt_model *m, const mt_op_desc *desc, int32_t *out_index) {
    if (!m || !desc) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (m->finalized) return fail(MT_ERR_INVALID_ARG, "model is already finalised");
    if (desc->kind < MT_CONV || desc->kind > MT_ADD) return fail(MT_ERR_INVALID_ARG, "unknown operator kind");
    OpRec o;
    o.d = *desc;
    m->ops.push_back(std::move(o));
    if (out_index) *out_index = (int32_t)m->ops.size() - 1;
    return MT_OK;
}

int32_t mt_model_end(mt_model *m) {
    if (!m) return fail(MT_ERR_INVALID_ARG, "model is NULL");
    if (m->finalized) return MT_OK;
    return finalize_model(m);
}

int32_t mt_model_destroy(mt_model *m) {
    if (!m) return fail(MT_ERR_INVALID_ARG, "model is NULL");
    delete m;
    return MT_OK;
}

int32_t mt_model_num_ops(const mt_model *m, int32_t *out) {
    if (!m || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    *out = (int32_t)m->ops.size();
    return MT_OK;
}

int32_t mt_model_op_info(const mt_model *m, int32_t i, mt_op_info *out) {
    if (!m || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (!m->finalized) return fail(MT_ERR_NOT_FINALIZED, "model is not finalised");
    if (i < 0 || i >= (int)m->ops.size()) return fail(MT_ERR_INVALID_ARG, "operator index out of range");
    fill_info(m, m->ops[i], out);
    return MT_OK;
}

int32_t mt_model_out_features(const mt_model *m, int64_t *out) {
    if (!m || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (!m->finalized) return fail(MT_ERR_NOT_FINALIZED, "model is not finalised");
    const TensorInfo &t = m->tensors[m->final_tensor];
    *out = (int64_t)t.h * t.w * t.c;
    return MT_OK;
}

int32_t mt_model_set_weights(mt_model *m, int32_t i, const void *w, size_t w_bytes, const float *bias, size_t n_bias) {
    if (!m || !w) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (!m->finalized) return fail(MT_ERR_NOT_FINALIZED, "call mt_model_end before setting weights");
    if (i < 0 || i >= (int)m->ops.size()) return fail(MT_ERR_INVALID_ARG, "operator index out of range");
    OpRec &o = m->ops[i];
    if (!needs_weights(o.d.kind)) return fail(MT_ERR_INVALID_ARG, "operator has no weights");
    const size_t es = elt_size(m->dtype);
    size_t count;
    if (o.d.kind == MT_DWCONV) count = (size_t)o.in_c * o.d.r * o.d.s;
    else if (o.d.kind == MT_FC) count = (size_t)o.out_c * o.in_h * o.in_w * o.in_c;
    else count = (size_t)o.out_c * o.d.r * o.d.s * (o.in_c / std::max(1, o.plan.groups));
    if (w_bytes != count * es) return fail(MT_ERR_SHAPE_MISMATCH, "weight size does not match the operator shape");
    if (bias && n_bias != (size_t)o.out_c) return fail(MT_ERR_SHAPE_MISMATCH, "bias length does not match the output channels");
    o.w_host.assign((const uint8_t *)w, (const uint8_t *)w + w_bytes);
    o.bias_host.assign(o.out_c, 0.f);
    if (bias) std::memcpy(o.bias_host.data(), bias, sizeof(float) * o.out_c);
    o.has_weights = true;
    return MT_OK;
}

int32_t mt_model_arena_bytes(const mt_model *m, size_t *out) {
    if (!m || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (!m->finalized) return fail(MT_ERR_NOT_FINALIZED, "model is not finalised");
    *out = m->arena_bytes;
    return MT_OK;
}

int32_t mt_fold_bn(float *w, int64_t k, int64_t per_k, const float *gamma, const float *beta, const float *mean,
                   const float *var, float eps, float *bias_out) {
    if (!w || !gamma || !beta || !mean || !var || !bias_out || k < 1 || per_k < 1)
        return fail(MT_ERR_INVALID_ARG, "bad argument");
    for (int64_t i = 0; i < k; ++i) {
        const float scale = gamma[i] / std::sqrt(var[i] + eps);
        for (int64_t j = 0; j < per_k; ++j) w[i * per_k + j] *= scale;
        const float ms = mean[i] * scale;
        bias_out[i] = beta[i] - ms;
    }
    return MT_OK;
}

// One round-to-nearest-even from fp32 to the storage type, written from the formats' definitions (host code: the
// device kernels round with the hardware conversions).
int32_t mt_round_to_storage(const float *src, int64_t n, int32_t dtype, void *dst) {
    if (!src || !dst || n < 0) return fail(MT_ERR_INVALID_ARG, "bad argument");
    if (dtype == MT_F32) {
        std::memcpy(dst, src, sizeof(float) * (size_t)n);
    } else if (dtype == MT_BF16) {
        uint16_t *o = (uint16_t *)dst;
        for (int64_t i = 0; i < n; ++i) {
            uint32_t u;
            std::memcpy(&u, src + i, 4);
            if ((u & 0x7fffffffu) > 0x7f800000u) o[i] = (uint16_t)((u >> 16) | 0x40u);          // NaN stays NaN (quiet)
            else o[i] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);                   // ties to even
        }
    } else if (dtype == MT_F16) {
        uint16_t *o = (uint16_t *)dst;
        for (int64_t i = 0; i < n; ++i) {
            uint32_t u;
            std::memcpy(&u, src + i, 4);
            const uint32_t sign = (u >> 16) & 0x8000u, mag = u & 0x7fffffffu;
            uint32_t h;
            if (mag > 0x7f800000u) h = 0x7e00u;                                               // NaN
            else if (mag >= 0x477ff000u) h = 0x7c00u;                                         // rounds to infinity (>= 65520)
            else if (mag >= 0x38800000u) {                                                    // normal half
                const uint32_t v = mag - 0x38000000u;                                         // rebias the exponent (127 -> 15)
                h = (v + 0xfffu + ((v >> 13) & 1u)) >> 13;
            } else if (mag >= 0x33000000u) {                                                  // subnormal half: multiples of 2^-24
                const uint32_t e = mag >> 23, m = (mag & 0x7fffffu) | 0x800000u;
                const uint32_t shift = 126u - e;                                              // 14 .. 24
                const uint32_t q = m >> shift, rem = m & ((1u << shift) - 1u), half = 1u << (shift - 1);
                h = q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u);
            } else h = 0;                                                                     // below half of the smallest subnormal
            o[i] = (uint16_t)(sign | h);
        }
    } else {
        return fail(MT_ERR_INVALID_ARG, "unknown storage type");
    }
    return MT_OK;
}

// ---- registration ----------------------------------------------------------------------------
int32_t mt_register(mt_ctx *ctx, const mt_model *m, void *device_arena, size_t arena_bytes, int32_t *out_tenant) {
    if (!ctx || !m || !out_tenant) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (!m->finalized) return fail(MT_ERR_NOT_FINALIZED, "model is not finalised");
    if ((int)ctx->tenants.size() >= MT_MAX_TENANTS) return fail(MT_ERR_INVALID_ARG, "too many tenants");
    for (size_t i = 0; i < m->ops.size(); ++i)
        if (needs_weights(m->ops[i].d.kind) && !m->ops[i].has_weights)
            return fail(MT_ERR_NOT_FINALIZED, "operator " + std::to_string(i) + " has no weights");
    if (device_arena) {
        if (arena_bytes < m->arena_bytes) return fail(MT_ERR_OUT_OF_MEMORY, "arena is smaller than mt_model_arena_bytes");
        if (((uintptr_t)device_arena) % ALIGN) return fail(MT_ERR_INVALID_ARG, "arena must be 256-byte aligned");
    }
    HIP_TRY(hipSetDevice(ctx->device));
    std::unique_ptr<Tenant> t(new Tenant);
    t->model = *m;
    if (device_arena) {
        t->arena = (uint8_t *)device_arena;
    } else {
        hipError_t e = hipMalloc((void **)&t->arena, std::max<size_t>(m->arena_bytes, ALIGN));
        if (e != hipSuccess) return fail(MT_ERR_OUT_OF_MEMORY, std::string("hipMalloc: ") + hipGetErrorString(e));
        t->owns_arena = true;
    }
    struct Guard {
        Tenant *t; bool armed = true;
        ~Guard() { if (armed && t->owns_arena && t->arena) { (void)hipFree(t->arena); t->arena = nullptr; } }
    } guard{t.get()};

    const int es = elt_size(m->dtype);
    const size_t nops = m->ops.size();
    t->args.resize(nops);
    t->reads_input.assign(nops, 0); t->res_input.assign(nops, 0); t->writes_output.assign(nops, 0);
    std::vector<uint8_t> packed;
    for (size_t i = 0; i < nops; ++i) {
        OpRec &o = t->model.ops[i];
        OpArgs a = o.plan;
        const bool igemm = is_gemm_kernel(a.kernel_id) || a.kernel_id == K_STEM || a.kernel_id == K_ROWB || a.kernel_id == K_PCONV;
        if (needs_weights(a.kind)) {
            const uint8_t *src = o.w_host.data();
            if (a.kernel_id == K_STEM) {
                // [K][R][S][3] -> [step][channel tile][lane][8]: the matrix-instruction fragments in reading order, zeros at
                // the dummy and padding positions of every filter row's run
                const StemGeom sg = stem_geom(a.R, a.S, stem_form(a.R, a.S, a.sw, a.W, a.pw, a.n_pad));
                const int tn = a.n_pad / 32;
                packed.assign((size_t)sg.ksteps * tn * 64 * 8 * es, 0);
                for (int t = 0; t < sg.ksteps; ++t)
                    for (int i = 0; i < tn; ++i)
                        for (int lane = 0; lane < 64; ++lane) {
                            const int k = 32 * i + lane % 32, G = 2 * t + lane / 32;
                            if (G >= sg.ng || k >= a.K) continue;
                            const int r = G / sg.gr, g = G % sg.gr;
                            for (int e = 0; e < 8; ++e) {
                                const int elem = 8 * g + e;
                                if (elem < sg.dummy || elem >= sg.seg) continue;
                                const int sc = elem - sg.dummy;    // s * 3 + c
                                std::memcpy(packed.data() + ((((size_t)t * tn + i) * 64 + lane) * 8 + e) * es,
                                            src + ((size_t)k * a.gemm_k + (size_t)r * a.S * 3 + sc) * es, es);
                            }
                        }
                src = packed.data();
            } else if (a.kernel_id == K_PCONV) {
                // [K][tap][C] -> [n_pad][chunk of 64 channels][tap][64], zero padded rows
                packed.assign((size_t)a.n_pad * a.k_pad * es, 0);
                const int ncc = a.C / 64;
                for (int k = 0; k < a.K; ++k)
                    for (int cc = 0; cc < ncc; ++cc)
                        for (int tap = 0; tap < 9; ++tap)
                            std::memcpy(packed.data() + ((size_t)k * a.k_pad + ((size_t)cc * 9 + tap) * 64) * es,
                                        src + ((size_t)k * a.gemm_k + (size_t)tap * a.C + cc * 64) * es, (size_t)64 * es);
                src = packed.data();
            } else if (a.kernel_id == K_ROWB) {
                // [K][gemm_k] -> [slice][step][channel tile][lane][8]: lane l of a step holds elements 16 * step + 8 * (l / 32)
                // .. + 7 of output channel 32 * (slice * tiles + tile) + l % 32
                const int steps = a.gemm_k / 16, tn = rowb_tiles(a.R, a.S, a.C, a.n_pad), slices = a.n_pad / (32 * tn);
                packed.assign((size_t)slices * steps * tn * 64 * 8 * es, 0);
                for (int sl = 0; sl < slices; ++sl)
                    for (int t = 0; t < steps; ++t)
                        for (int i = 0; i < tn; ++i)
                            for (int lane = 0; lane < 64; ++lane) {
                                const int k = 32 * (sl * tn + i) + lane % 32;
                                if (k >= a.K) continue;
                                std::memcpy(packed.data() + ((((size_t)sl * steps + t) * tn + i) * 64 + lane) * 8 * es,
                                            src + ((size_t)k * a.gemm_k + 16 * t + 8 * (lane / 32)) * es, (size_t)8 * es);
                            }
                src = packed.data();
            } else if (igemm) {
                // [groups][K][gemm_k] -> [groups][n_pad][k_pad], zero padded
                packed.assign((size_t)a.groups * a.n_pad * a.k_pad * es, 0);
                for (int g = 0; g < a.groups; ++g)
                    for (int k = 0; k < a.K; ++k)
                        std::memcpy(packed.data() + ((size_t)g * a.n_pad + k) * a.k_pad * es,
                                    src + ((size_t)g * a.K + k) * a.gemm_k * es, (size_t)a.gemm_k * es);
                src = packed.data();
            } else if (a.kind == MT_DWCONV) {
                // [C][R][S] -> [R][S][C]
                packed.assign((size_t)a.C * a.R * a.S * es, 0);
                for (int c = 0; c < a.C; ++c)
                    for (int rs = 0; rs < a.R * a.S; ++rs)
                        std::memcpy(packed.data() + ((size_t)rs * a.C + c) * es, src + ((size_t)c * a.R * a.S + rs) * es, es);
                src = packed.data();
            }
            HIP_TRY(hipMemcpy(t->arena + o.w_off, src, o.w_bytes, hipMemcpyHostToDevice));
            const size_t bstride = igemm ? a.n_pad : a.K;
            std::vector<float> b(bstride * a.groups, 0.f);
            for (int g = 0; g < a.groups; ++g)
                std::memcpy(b.data() + g * bstride, o.bias_host.data() + (size_t)g * a.K, sizeof(float) * a.K);
            HIP_TRY(hipMemcpy(t->arena + o.bias_off, b.data(), b.size() * sizeof(float), hipMemcpyHostToDevice));
            a.w = t->arena + o.w_off;
            a.bias = (const float *)(t->arena + o.bias_off);
        }
        if (a.split_k > 1 && a.kernel_id != K_IGEMM_PW) {
            a.ws = (float *)(t->arena + o.ws_off);
            a.counters = (uint32_t *)(t->arena + o.cnt_off);
            HIP_TRY(hipMemset(a.counters, 0, o.cnt_bytes));
        }
        auto tptr = [&](int id) -> uint8_t * { return t->arena + t->model.tensors[id].offset; };
        if (o.d.in_tensor == 0) t->reads_input[i] = 1; else a.x = tptr(o.d.in_tensor);
        if (o.d.res_tensor == 0) t->res_input[i] = 1; else if (o.d.res_tensor > 0) a.res = tptr(o.d.res_tensor);
        a.y = tptr(o.d.out_tensor);
        if (o.d.out_tensor == t->model.final_tensor) t->writes_output[i] = 1;
        t->args[i] = a;
        o.w_host.clear(); o.w_host.shrink_to_fit();
    }
    t->st_cnt_off.assign(nops, 0);
    t->st_ws_off.assign(nops, 0);
    for (size_t i = 0; i < nops; ++i) {
        const OpRec &o = t->model.ops[i];
        if (!t->args[i].ws) continue;
        t->st_cnt_off[i] = t->st_cnt_bytes; t->st_cnt_bytes += align_up(o.cnt_bytes);
        t->st_ws_off[i] = t->st_ws_bytes; t->st_ws_bytes += align_up(o.ws_bytes);
    }
    // short kernels: few workgroups of little work each, bound by launch and memory latency
    t->short_kernel.assign(nops, 0);
    for (size_t i = 0; i < nops; ++i) {
        const OpArgs &a = t->args[i];
        const int k = a.kernel_id;
        t->short_kernel[i] = k == K_IGEMM_64x16 || k == K_IGEMM_PW || k == K_DWCONV || k == K_MAXPOOL || k == K_AVGPOOL || k == K_GAP || k == K_LRN ||
                             k == K_ADD || (k == K_GEMV && (size_t)a.n_pad * a.k_pad * 2 < ((size_t)16 << 20));
    }
    // depthwise convolution followed by the 1x1 convolution that reads it: candidates for one fused launch
    t->fuse_next.assign(nops, 0);
    for (size_t i = 0; i + 1 < nops; ++i) {
        const mt_op_desc &d0 = t->model.ops[i].d, &d1 = t->model.ops[i + 1].d;
        if (d0.kind == MT_DWCONV && d1.kind == MT_CONV && d1.in_tensor == d0.out_tensor && !t->writes_output[i] &&
            dwpw_fusable(t->args[i], t->args[i + 1]))
            t->fuse_next[i] = 1;
    }
    // 1x1 convolution followed by the depthwise convolution that alone reads it, on a small map
    t->fuse_pwdw.assign(nops, 0);
    for (size_t i = 0; i + 1 < nops; ++i) {
        const mt_op_desc &d0 = t->model.ops[i].d, &d1 = t->model.ops[i + 1].d;
        if (d0.kind != MT_CONV || d1.kind != MT_DWCONV || d1.in_tensor != d0.out_tensor || t->writes_output[i] ||
            !pwdw_fusable(t->args[i], t->args[i + 1]))
            continue;
        bool sole_writer = true;                     // no other operator writes channels of the widened tensor
        for (size_t j = 0; j < nops; ++j)
            if (j != i && t->model.ops[j].d.out_tensor == d0.out_tensor) sole_writer = false;
        if (sole_writer) t->fuse_pwdw[i] = 1;
    }
    // convolution followed by the 2x2 / stride-2 max pooling that alone reads it: candidates for the pooled epilogue
    t->fuse_pool.assign(nops, 0);
    t->pool_args.assign(nops, OpArgs{});
    for (size_t i = 0; i + 1 < nops; ++i) {
        const mt_op_desc &d0 = t->model.ops[i].d, &d1 = t->model.ops[i + 1].d;
        const OpArgs &a0 = t->args[i], &a1 = t->args[i + 1];
        if (d0.kind != MT_CONV || d1.kind != MT_MAXPOOL || d1.in_tensor != d0.out_tensor || t->writes_output[i]) continue;
        if (!is_gemm_kernel(a0.kernel_id) || a0.kernel_id == K_GEMV || a0.kernel_id == K_IGEMM_PW || a0.groups > 1 || a0.res_ct != 0 || d0.res_tensor >= 0) continue;
        if (a0.K % 8 != 0 || a0.y_coff != 0 || a0.y_ct != a0.K || a0.P % 2 != 0 || a0.Q % 2 != 0) continue;
        if (a1.R != 2 || a1.S != 2 || a1.sh != 2 || a1.sw != 2 || a1.ph != 0 || a1.pw != 0 || a1.vec != 8) continue;
        bool only = true;                            // nothing else reads or writes the convolution's output tensor
        for (size_t j = 0; j < nops; ++j) {
            const mt_op_desc &dj = t->model.ops[j].d;
            if (j != i && dj.out_tensor == d0.out_tensor) only = false;
            if (j != i + 1 && (dj.in_tensor == d0.out_tensor || dj.res_tensor == d0.out_tensor)) only = false;
        }
        if (!only) continue;
        OpArgs b = a0;
        b.pool2 = 1;
        b.y = a1.y; b.y_ct = a1.y_ct; b.y_coff = a1.y_coff;
        make_divisor((uint32_t)(b.Q / 2), b.divq_m, b.divq_s1, b.divq_s2);
        make_divisor((uint32_t)(b.P / 2) * (uint32_t)(b.Q / 2), b.divpq_m, b.divpq_s1, b.divpq_s2);
        t->pool_args[i] = b;
        t->fuse_pool[i] = 1;
    }
    HIP_TRY(hipDeviceSynchronize());
    guard.armed = false;
    ctx->tenants.push_back(std::move(t));
    *out_tenant = (int32_t)ctx->tenants.size() - 1;
    return MT_OK;
}

int32_t mt_num_tenants(const mt_ctx *ctx, int32_t *out) {
    if (!ctx || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    *out = (int32_t)ctx->tenants.size();
    return MT_OK;
}

int32_t mt_tenant_num_ops(const mt_ctx *ctx, int32_t tenant, int32_t *out) {
    if (!ctx || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (tenant < 0 || tenant >= (int)ctx->tenants.size()) return fail(MT_ERR_INVALID_ARG, "no such tenant");
    *out = (int32_t)ctx->tenants[tenant]->model.ops.size();
    return MT_OK;
}

int32_t mt_tenant_op_info(const mt_ctx *ctx, int32_t tenant, int32_t i, mt_op_info *out) {
    if (!ctx || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (tenant < 0 || tenant >= (int)ctx->tenants.size()) return fail(MT_ERR_INVALID_ARG, "no such tenant");
    return mt_model_op_info(&ctx->tenants[tenant]->model, i, out);
}

int32_t mt_tenant_read_tensor(mt_ctx *ctx, int32_t tenant, int32_t tensor_id, void *host_dst, size_t bytes) {
    if (!ctx || !host_dst) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (tenant < 0 || tenant >= (int)ctx->tenants.size()) return fail(MT_ERR_INVALID_ARG, "no such tenant");
    Tenant &t = *ctx->tenants[tenant];
    if (tensor_id < 1 || tensor_id >= (int)t.model.tensors.size() || !t.model.tensors[tensor_id].defined)
        return fail(MT_ERR_INVALID_ARG, "no such tensor (tensor 0 and the final tensor live in caller memory)");
    if (tensor_id == t.model.final_tensor) return fail(MT_ERR_INVALID_ARG, "the final tensor is written to the caller's output buffer");
    if (bytes != t.model.tensors[tensor_id].bytes) return fail(MT_ERR_SHAPE_MISMATCH, "byte count does not match the tensor");
    HIP_TRY(hipSetDevice(ctx->device));
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host_dst, t.arena + t.model.tensors[tensor_id].offset, bytes, hipMemcpyDeviceToHost));
    return MT_OK;
}

// ---- schedule --------------------------------------------------------------------------------
int32_t mt_schedule_create(mt_ctx *ctx, int32_t n_tenants, int32_t n_stages, const int32_t *pointers,
                           const int32_t *stage_concurrency, const int32_t *cu_share, int32_t order, int32_t flags,
                           mt_schedule **out) {
    if (!ctx || !out) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    *out = nullptr;
    if (n_tenants != (int)ctx->tenants.size() || n_tenants < 1)
        return fail(MT_ERR_INVALID_SCHEDULE, "schedule must cover exactly the registered tenants");
    if (order != MT_ISSUE_BFS && order != MT_ISSUE_DFS) return fail(MT_ERR_INVALID_ARG, "unknown issue order");
    if ((flags & MT_SCHED_GRAPH) && (flags & MT_SCHED_PARALLEL_ISSUE))
        return fail(MT_ERR_INVALID_ARG, "graph replay and parallel issue cannot be combined");
    if ((flags & MT_SCHED_STREAM_GRAPHS) && (flags & (MT_SCHED_GRAPH | MT_SCHED_PARALLEL_ISSUE | MT_SCHED_TIME_FIRST_OP)))
        return fail(MT_ERR_INVALID_ARG, "per-stream graphs cannot be combined with whole-schedule replay, parallel issue or first-operator timing");
    if ((flags & MT_SCHED_TIME_FIRST_OP) && (flags & (MT_SCHED_GRAPH | MT_SCHED_PARALLEL_ISSUE)))
        return fail(MT_ERR_INVALID_ARG, "first-operator timing needs the single issuing thread and plain streams");
    if ((flags & MT_SCHED_COUNTER_BARRIER) && (flags & (MT_SCHED_GRAPH | MT_SCHED_STREAM_GRAPHS | MT_SCHED_HOST_BARRIER)))
        return fail(MT_ERR_INVALID_ARG, "the counter barrier runs on plain streams with device-side waits: not with graphs or the host-side barrier");
    if ((flags & MT_SCHED_COISSUE) && (flags & (MT_SCHED_GRAPH | MT_SCHED_STREAM_GRAPHS | MT_SCHED_TIME_FIRST_OP)))
        return fail(MT_ERR_INVALID_ARG, "co-issue runs on plain streams without first-operator timing");
    if ((flags & MT_SCHED_HOST_BARRIER) && !(flags & MT_SCHED_PARALLEL_ISSUE))
        return fail(MT_ERR_INVALID_ARG, "the host-side barrier needs one issuing thread per stream (MT_SCHED_PARALLEL_ISSUE)");
    if ((flags & MT_SCHED_TIME_TENANTS) && (flags & (MT_SCHED_GRAPH | MT_SCHED_STREAM_GRAPHS)))
        return fail(MT_ERR_INVALID_ARG, "per-tenant completion times cannot be read from captured graphs");
    int32_t lens[MT_MAX_TENANTS];
    for (int i = 0; i < n_tenants; ++i) lens[i] = (int32_t)ctx->tenants[i]->model.ops.size();
    int32_t rc = validate_pointers(n_tenants, lens, n_stages, pointers);
    if (rc != MT_OK) return rc;
    const int cus = ctx->prop.multiProcessorCount;
    for (int s = 0; s < n_stages; ++s)
        if (stage_concurrency && stage_concurrency[s] < 1) return fail(MT_ERR_INVALID_SCHEDULE, "stage concurrency must be >= 1");
    const int n_shares = (flags & MT_SCHED_SHARE_PER_STAGE) ? n_stages * n_tenants : n_tenants;
    if ((flags & MT_SCHED_SHARE_PER_STAGE) && !cu_share) return fail(MT_ERR_INVALID_ARG, "per-stage shares asked for but cu_share is NULL");
    for (int i = 0; i < n_shares; ++i)
        if (cu_share && (cu_share[i] < 0 || cu_share[i] > cus)) return fail(MT_ERR_INVALID_SCHEDULE, "CU share out of range");
    for (int i = 0; i < n_shares; ++i)
        if (cu_share && cu_share[i] > 0 && cu_share[i] < 8)
            return fail(MT_ERR_INVALID_SCHEDULE, "a CU share must be 0 (all units) or at least 8: a mask has to leave every one of the 8 XCDs a unit");
    HIP_TRY(hipSetDevice(ctx->device));
    std::unique_ptr<mt_schedule> s(new mt_schedule);
    s->ctx = ctx; s->n_tenants = n_tenants; s->n_stages = n_stages; s->flags = flags;
    for (int i = 0; i < n_tenants; ++i) s->prio[i] = (flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0;
    const bool per_stage = (flags & MT_SCHED_SHARE_PER_STAGE) != 0;
    s->stream_at.assign(n_stages, {});
    struct Acquired { StreamKey key; int share, first_cu; };
    std::vector<std::array<Acquired, MT_MAX_TENANTS>> acq(per_stage ? n_stages : 1);
    for (int st = 0; st < (per_stage ? n_stages : 1); ++st) {
        int first_cu = 0;
        for (int i = 0; i < n_tenants; ++i) {
            const int share = (cu_share && !(flags & MT_SCHED_GRAPH)) ? cu_share[(per_stage ? st * n_tenants : 0) + i] : 0;
            StreamKey key;
            rc = get_stream(ctx, i, share, first_cu, &s->stream_at[st][i], &key);
            if (rc != MT_OK) { release_streams(s.get()); return rc; }
            s->stream_keys.push_back(key);
            acq[st][i] = Acquired{key, share, first_cu};
            first_cu = (first_cu + share) % cus;
        }
    }
    if (!per_stage)
        for (int st = 1; st < n_stages; ++st) s->stream_at[st] = s->stream_at[0];
    std::vector<int32_t> slices((size_t)n_stages * n_tenants * 2);
    expand_pointers(n_tenants, lens, n_stages, pointers, slices.data());
    s->stages.resize(n_stages);
    for (int st = 0; st < n_stages; ++st) {
        const int conc = stage_concurrency ? stage_concurrency[st] : n_tenants;
        StagePlan &sp = s->stages[st];
        sp.items = issue_order(n_tenants, &slices[(size_t)st * n_tenants * 2], conc, order);
        // On request, two neighbouring operators issued in the same stage run as one launch.
        auto mark_pairs = [&](std::vector<IssueItem> &items, bool count) {
            for (int pass = 0; pass < 3; ++pass) {   // 1x1 + depthwise pairs before depthwise + 1x1: a depthwise operator joins one neighbour only
                const int want = pass == 0 ? MT_SCHED_FUSE_EXPAND : pass == 1 ? MT_SCHED_FUSE_DEPTHWISE : MT_SCHED_FUSE_POOL;
                if (!(flags & want)) continue;
                for (size_t k = 0; k < items.size(); ++k) {
                    IssueItem &it = items[k];
                    const Tenant &tt = *ctx->tenants[it.tenant];
                    const int end = slices[((size_t)st * n_tenants + it.tenant) * 2 + 1];
                    const bool can = pass == 0 ? tt.fuse_pwdw[it.op] != 0 : pass == 1 ? tt.fuse_next[it.op] != 0 : tt.fuse_pool[it.op] != 0;
                    if (it.fuse != 0 || it.op + 1 >= end || !can) continue;
                    for (size_t k2 = k + 1; k2 < items.size(); ++k2)
                        if (items[k2].tenant == it.tenant && items[k2].op == it.op + 1) {
                            if (items[k2].fuse == 0) {
                                // the absorbed operator is skipped; the other one launches the pair
                                items[k2].fuse = pass == 0 ? 3 : pass == 1 ? 2 : 1;
                                it.fuse = pass == 2 ? 4 : 1;
                                if (count) ++s->n_fused;
                            }
                            break;
                        }
                }
            }
        };
        mark_pairs(sp.items, true);
        // Co-issue: up to `group` tenants that share a stream and whose slices have the same operator range walk them
        // together; operator i of the others runs inside the launch of operator i of the first where they can
        // (coissue_pair_ok with the first), else right after it as a launch of its own.  The first tenant's items carry
        // the mates, the others' stay in the list (they count as issued and carry the end-of-tenant timing) and launch
        // nothing.
        if (flags & MT_SCHED_COISSUE) {
            const int group = COISSUE_MAX;
            int32_t hs[MT_MAX_TENANTS];
            stream_map(n_tenants, &slices[(size_t)st * n_tenants * 2], conc, hs);
            auto range = [&](int t, int which) { return slices[((size_t)st * n_tenants + t) * 2 + which]; };
            for (int sm = 0; sm < n_tenants; ++sm) {
                std::vector<int> on;                         // tenants of this stream, in tenant order
                for (int i = 0; i < n_tenants; ++i)
                    if (hs[i] == sm) on.push_back(i);
                for (size_t k = 0; k + 1 < on.size();) {
                    const int ta = on[k];
                    std::vector<int> rest;                   // the following tenants of the same operator range
                    while (k + 1 + rest.size() < on.size() && (int)rest.size() + 1 < group &&
                           range(on[k + 1 + rest.size()], 0) == range(ta, 0) && range(on[k + 1 + rest.size()], 1) == range(ta, 1))
                        rest.push_back(on[k + 1 + rest.size()]);
                    k += 1 + rest.size();
                    if (rest.empty()) continue;
                    const int ba = range(ta, 0), ea = range(ta, 1);
                    // operator i of the other tenants follows operator i of the first in the issue sequence
                    std::vector<std::vector<IssueItem>> others(rest.size(), std::vector<IssueItem>(ea - ba));
                    auto which = [&](int t) { for (size_t r = 0; r < rest.size(); ++r) if (rest[r] == t) return (int)r; return -1; };
                    for (const IssueItem &it : sp.items)
                        if (which(it.tenant) >= 0) others[which(it.tenant)][it.op - ba] = it;
                    std::vector<IssueItem> merged;
                    merged.reserve(sp.items.size());
                    for (const IssueItem &it : sp.items) {
                        if (which(it.tenant) >= 0) continue;
                        merged.push_back(it);
                        if (it.tenant != ta) continue;
                        const size_t head = merged.size() - 1;
                        int nm = 0;
                        for (size_t r = 0; r < rest.size(); ++r) {
                            IssueItem other = others[r][it.op - ba];
                            if (it.fuse == 0 && other.fuse == 0 &&
                                coissue_pair_ok(ctx->tenants[ta]->args[it.op], ctx->tenants[rest[r]]->args[it.op])) {
                                merged[head].mates[nm++] = rest[r];
                                other.fuse = 1;
                                ++s->n_fused;
                            }
                            merged.push_back(other);
                        }
                    }
                    sp.items.swap(merged);
                }
            }
        }
        if ((flags & MT_SCHED_GRAPH) && n_tenants > 1) {
            s->alt_items.resize(n_stages);
            s->alt_items[st] = issue_order(n_tenants, &slices[(size_t)st * n_tenants * 2], conc, order == MT_ISSUE_BFS ? MT_ISSUE_DFS : MT_ISSUE_BFS);
            mark_pairs(s->alt_items[st], false);
        }
        for (const IssueItem &it : sp.items)
            if (std::find(sp.streams.begin(), sp.streams.end(), it.stream) == sp.streams.end()) sp.streams.push_back(it.stream);
        std::sort(sp.streams.begin(), sp.streams.end());
        sp.by_stream.assign(n_tenants, {});
        for (const IssueItem &it : sp.items) sp.by_stream[it.stream].push_back(it);
        s->n_launches += (int)sp.items.size();
    }
    for (int st = 0, last = -1; st < n_stages; ++st) {
        s->stages[st].prev_stage = last;
        if (!s->stages[st].items.empty()) last = st;
        s->end_stage = last;
    }
    if (flags & MT_SCHED_COUNTER_BARRIER) {
        s->arrivals_upto.assign(n_stages, 0);
        uint32_t sum = 0;
        for (int st = 0; st < n_stages; ++st) {
            sum += (uint32_t)s->stages[st].streams.size();
            s->arrivals_upto[st] = sum;
        }
        if (!ctx->barrier_word) {
            rc = take_signal_word(ctx->device, &ctx->barrier_word);
            if (rc != MT_OK) { release_streams(s.get()); return rc; }
        }
    }
    // A schedule that uses masked streams checks its streams together (plain streams are placed by dispatch pipe when
    // they are created, see PlainPool; masked ones are not).  Every stream launches one probe kernel per round; a round
    // of more than 1.8 single-stream launches per started group of four streams, twice in a row and not explained by
    // the issuing thread's own launch time, means that streams of the set take turns on one pipe.  The stream whose
    // removal helps most is then parked and replaced (a masked one only if no other schedule holds it), up to three times.
    bool any_masked = false;
    for (const auto &row : acq)
        for (int i = 0; i < n_tenants; ++i) any_masked = any_masked || row[i].share != 0;
    if (!(flags & MT_SCHED_GRAPH) && any_masked) {
        struct Used { int row, idx; };
        std::vector<Used> used;
        std::vector<hipStream_t> all;
        auto collect = [&]() {
            used.clear();
            all.clear();
            for (int st = 0; st < n_stages; ++st)
                for (int sm : s->stages[st].streams) {
                    hipStream_t h = s->stream_at[st][sm];
                    if (std::find(all.begin(), all.end(), h) == all.end() && (int)all.size() < MT_MAX_TENANTS) {
                        all.push_back(h);
                        used.push_back(Used{per_stage ? st : 0, sm});
                    }
                }
        };
        auto measure = [&](const std::vector<hipStream_t> &set, float *us, bool *bad) -> int32_t {
            float host_us = 0.f;
            const float limit = 1.8f * ctx->best_dispatch_us * (float)((set.size() + 3) / 4);
            for (int rep = 0; rep < 2; ++rep) {          // a single high reading is measured again before it counts
                int32_t r = concurrent_latency_us(ctx, set, 8, us, &host_us);
                if (r != MT_OK) return r;
                *bad = ctx->best_dispatch_us > 0.f && *us > limit && *us > 1.3f * host_us;
                if (!*bad) break;
            }
            return MT_OK;
        };
        collect();
        for (int attempt = 0; attempt < 3 && all.size() > 1; ++attempt) {
            if (ctx->best_dispatch_us == 0.f) {         // a context that only met pooled streams so far has no reference yet
                float us1 = 0.f;
                if (!ctx->probe_buf) HIP_TRY(hipMalloc((void **)&ctx->probe_buf, 256));
                rc = dispatch_latency_us(ctx, all[0], ctx->probe_buf, 12, &us1);
                if (rc != MT_OK) { release_streams(s.get()); return rc; }
                ctx->best_dispatch_us = us1;
            }
            float us = 0.f;
            bool bad = false;
            rc = measure(all, &us, &bad);
            if (rc != MT_OK) { release_streams(s.get()); return rc; }
            if (!bad) break;
            // leave one out: the stream without which the rest runs fastest is the one to replace
            int culprit = (int)all.size() - 1;
            float best_rest = 1e30f;
            for (size_t j = 0; j < all.size() && all.size() > 2; ++j) {
                std::vector<hipStream_t> rest;
                for (size_t k = 0; k < all.size(); ++k)
                    if (k != j) rest.push_back(all[k]);
                float host_us = 0.f, r_us = 0.f;
                rc = concurrent_latency_us(ctx, rest, 8, &r_us, &host_us);
                if (rc != MT_OK) { release_streams(s.get()); return rc; }
                if (r_us < best_rest) { best_rest = r_us; culprit = (int)j; }
            }
            const Used u = used[culprit];
            const Acquired &aq = acq[u.row][u.idx];
            auto it = ctx->streams.find(aq.key);
            if (it == ctx->streams.end()) break;
            if (aq.share != 0 && it->second.refs != 1) break;          // another schedule launches on this masked stream
            hipStream_t fresh = nullptr;
            rc = make_stream(ctx, u.idx, aq.share, aq.first_cu, &fresh);
            if (rc != MT_OK) { release_streams(s.get()); return rc; }
            if (aq.share == 0) {
                PlainPool &pool = plain_pool(ctx->device);
                pool.parked.push_back(it->second.stream);           // never destroyed: other schedules may hold it
                pool.tenant[u.idx] = fresh;
            } else {
                ctx->parked_streams.push_back(it->second.stream);
            }
            it->second.stream = fresh;
            for (int st = 0; st < n_stages; ++st)
                if (!per_stage || st == u.row) s->stream_at[st][u.idx] = fresh;
            collect();
        }
    }
    ctx->live_schedules.insert(s.get());
    *out = s.release();
    return MT_OK;
}

int32_t mt_schedule_set_wave_priority(mt_schedule *s, const int32_t *prio) {
    if (!s || !prio) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    for (int i = 0; i < s->n_tenants; ++i)
        if (prio[i] < -1 || prio[i] > 3) return fail(MT_ERR_INVALID_ARG, "wave priority must be -1 (by kernel size) or 0..3");
    for (int i = 0; i < s->n_tenants; ++i) s->prio[i] = prio[i];
    if (s->ctx) retire_graphs(s->ctx, s);            // captured launches carry the old value
    s->cap_in.clear();
    s->cap_out.clear();
    return MT_OK;
}

int32_t mt_schedule_destroy(mt_schedule *s) {
    if (!s) return fail(MT_ERR_INVALID_ARG, "schedule is NULL");
    if (s->ctx) {
        retire_graphs(s->ctx, s);
        release_streams(s);
        s->ctx->live_schedules.erase(s);
    }
    delete s;
    return MT_OK;
}

// ---- run -------------------------------------------------------------------------------------
static int32_t run_pass(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, mt_timings *tm);

int32_t mt_run(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, mt_timings *tm) {
    return run_pass(ctx, s, inputs, outputs, tm);
}

int32_t mt_run_static_scratch(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, mt_timings *tm) {
    if (!ctx || !s || !inputs || !outputs) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (s->ctx != ctx) return fail(MT_ERR_INVALID_ARG, "schedule belongs to another (or a destroyed) context");
    if (s->flags & (MT_SCHED_GRAPH | MT_SCHED_STREAM_GRAPHS | MT_SCHED_PARALLEL_ISSUE))
        return fail(MT_ERR_INVALID_ARG, "graph replay and parallel issue allocate on their first run: not available without allocation");
    HIP_TRY(hipSetDevice(ctx->device));
    size_t cnt_total = 0, ws_total = 0;
    for (int i = 0; i < s->n_tenants; ++i) {
        cnt_total += ctx->tenants[i]->st_cnt_bytes;
        ws_total += ctx->tenants[i]->st_ws_bytes;
    }
    if (cnt_total + ws_total > (size_t)MT_STATIC_SCRATCH_BYTES)
        return fail(MT_ERR_OUT_OF_MEMORY, "the split workspaces of these tenants need " + std::to_string(cnt_total + ws_total) +
                                              " bytes, the fixed scratch array holds " + std::to_string((size_t)MT_STATIC_SCRATCH_BYTES));
    void *base = nullptr;
    const int e = static_scratch_address(ctx->device, &base);
    if (e != 0) return fail(MT_ERR_HIP, std::string("fixed scratch array: ") + hipGetErrorString((hipError_t)e));
    size_t cnt_at = 0, ws_at = cnt_total;                  // counters of all tenants first: one fill clears them
    for (int i = 0; i < s->n_tenants; ++i) {
        s->st_cnt_base[i] = cnt_at; cnt_at += ctx->tenants[i]->st_cnt_bytes;
        s->st_ws_base[i] = ws_at; ws_at += ctx->tenants[i]->st_ws_bytes;
    }
    if (cnt_total > 0) {
        // The array keeps what the last call (of any context) left; counters must start at zero.  The fill runs on the
        // main stream ahead of the start event that every tenant stream waits for.
        const int fe = launch_fill_u32((uint32_t *)base, cnt_total / sizeof(uint32_t), 0u, ctx->main_stream);
        if (fe != 0) return fail(MT_ERR_HIP, std::string("clearing the counters: ") + hipGetErrorString((hipError_t)fe));
    }
    s->st_base = (uint8_t *)base;
    const int32_t rc = run_pass(ctx, s, inputs, outputs, tm);
    s->st_base = nullptr;
    return rc;
}

static int32_t run_pass(mt_ctx *ctx, mt_schedule *s, const void *const *inputs, void *const *outputs, mt_timings *tm) {
    if (!ctx || !s || !inputs || !outputs) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (s->ctx != ctx) return fail(MT_ERR_INVALID_ARG, "schedule belongs to another (or a destroyed) context");
    for (int i = 0; i < s->n_tenants; ++i) {
        if (!inputs[i] || !outputs[i]) return fail(MT_ERR_INVALID_ARG, "NULL input or output buffer");
        if (((uintptr_t)inputs[i] % 16) || ((uintptr_t)outputs[i] % 16)) return fail(MT_ERR_INVALID_ARG, "buffers must be 16-byte aligned");
    }
    HIP_TRY(hipSetDevice(ctx->device));
    const auto t0 = std::chrono::steady_clock::now();
    int launches = 0;
    if (s->flags & MT_SCHED_GRAPH) {
        bool same = s->graph_exec && (int)s->cap_in.size() == s->n_tenants;
        for (int i = 0; same && i < s->n_tenants; ++i) same = s->cap_in[i] == inputs[i] && s->cap_out[i] == outputs[i];
        if (!same) {
            retire_graphs(ctx, s);
            // Replay does not know an issue order, only the capture does, and on this runtime the replay of a schedule
            // captured in one order is sometimes several times slower than that of the other (measured with more
            // than 4 hardware queues per process: 1 to 2.7 ms against 0.4 to 0.6 ms, in either direction).  Both orders
            // are therefore captured, each is replayed three times, and the faster graph is kept.
            const int n_orders = s->alt_items.empty() ? 1 : 2;
            hipGraphExec_t exec[2] = {nullptr, nullptr};
            float best_ms[2] = {0.f, 0.f};
            for (int o = 0; o < n_orders; ++o) {
                hipGraph_t graph = nullptr;
                HIP_TRY(hipStreamBeginCapture(ctx->main_stream, hipStreamCaptureModeRelaxed));
                int32_t rc = issue_schedule(ctx, s, inputs, outputs, &launches, o == 1);
                hipError_t e = hipStreamEndCapture(ctx->main_stream, &graph);
                if (rc == MT_OK && e != hipSuccess) rc = fail(MT_ERR_HIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
                if (rc == MT_OK) {
                    e = hipGraphInstantiate(&exec[o], graph, nullptr, nullptr, 0);
                    if (e != hipSuccess) rc = fail(MT_ERR_HIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e));
                }
                if (graph) (void)hipGraphDestroy(graph);
                if (rc != MT_OK) {
                    for (hipGraphExec_t g : exec)
                        if (g) ctx->retired_graphs.push_back(g);
                    return rc;
                }
            }
            int keep = 0;
            if (n_orders == 2) {
                for (int o = 0; o < 2; ++o)
                    for (int rep = 0; rep < 3; ++rep) {
                        float ms = 0.f;
                        HIP_TRY(hipEventRecord(ctx->ev_prof[0], ctx->main_stream));
                        HIP_TRY(hipGraphLaunch(exec[o], ctx->main_stream));
                        HIP_TRY(hipEventRecord(ctx->ev_prof[1], ctx->main_stream));
                        HIP_TRY(hipEventSynchronize(ctx->ev_prof[1]));
                        HIP_TRY(hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_prof[1]));
                        if (rep == 0 || ms < best_ms[o]) best_ms[o] = ms;
                    }
                keep = best_ms[1] < best_ms[0] ? 1 : 0;
                ctx->retired_graphs.push_back(exec[1 - keep]);
            }
            s->graph_exec = exec[keep];
            s->cap_in.assign(inputs, inputs + s->n_tenants);
            s->cap_out.assign(outputs, outputs + s->n_tenants);
        }
        launches = s->n_launches;
        HIP_TRY(hipEventRecord(ctx->ev_prof[0], ctx->main_stream));
        HIP_TRY(hipGraphLaunch(s->graph_exec, ctx->main_stream));
        HIP_TRY(hipEventRecord(ctx->ev_prof[1], ctx->main_stream));
    } else {
        if (s->flags & MT_SCHED_STREAM_GRAPHS) {
            bool same = !s->slice_exec.empty() && (int)s->cap_in.size() == s->n_tenants;
            for (int i = 0; same && i < s->n_tenants; ++i) same = s->cap_in[i] == inputs[i] && s->cap_out[i] == outputs[i];
            if (!same) {
                int32_t rc = capture_slice_graphs(ctx, s, inputs, outputs);
                if (rc != MT_OK) return rc;
            }
        }
        int32_t rc = (s->flags & MT_SCHED_PARALLEL_ISSUE) ? issue_schedule_parallel(ctx, s, inputs, outputs, &launches)
                                                          : issue_schedule(ctx, s, inputs, outputs, &launches);
        if (rc != MT_OK) return rc;
    }
    const auto t1 = std::chrono::steady_clock::now();
    if (s->flags & MT_SCHED_GRAPH) {
        HIP_TRY(hipEventSynchronize(ctx->ev_prof[1]));
    } else if (ends_on_streams(s)) {
        for (int sm : s->stages[s->end_stage].streams) HIP_TRY(hipEventSynchronize(ctx->ev_done[s->end_stage][sm]));
    } else {
        HIP_TRY(hipEventSynchronize(ctx->ev_stage[s->n_stages - 1]));
    }
    if (tm) {
        std::memset(tm, 0, sizeof(*tm));
        tm->n_launches = launches;
        tm->n_fused = s->n_fused;
        tm->n_stages = s->n_stages;
        tm->host_issue_ms = std::chrono::duration<float, std::milli>(t1 - t0).count();
        if (s->flags & MT_SCHED_GRAPH) {
            // events recorded inside a captured graph cannot be queried: only the end-to-end time is available
            HIP_TRY(hipEventElapsedTime(&tm->makespan_ms, ctx->ev_prof[0], ctx->ev_prof[1]));
        } else {
            if (ends_on_streams(s)) {
                float before = 0.f;                    // end of the stage before, from the start
                for (int st = 0; st <= s->end_stage; ++st) {
                    float end = before;
                    for (int sm : s->stages[st].streams) {             // the latest end over the streams of the stage
                        float ms = 0.f;
                        HIP_TRY(hipEventElapsedTime(&ms, ctx->ev_start, ctx->ev_done[st][sm]));
                        end = std::max(end, ms);
                    }
                    tm->stage_ms[st] = end - before;   // 0 for a stage that launches nothing
                    before = end;
                }
                tm->makespan_ms = before;
            } else {
                HIP_TRY(hipEventElapsedTime(&tm->makespan_ms, ctx->ev_start, ctx->ev_stage[s->n_stages - 1]));
            }
            if (s->flags & MT_SCHED_TIME_FIRST_OP)
                for (int i = 0; i < s->n_tenants; ++i)
                    if (!ctx->tenants[i]->model.ops.empty())
                        HIP_TRY(hipEventElapsedTime(&tm->first_op_done_ms[i], ctx->ev_start, ctx->ev_first[i]));
            if (s->flags & MT_SCHED_TIME_TENANTS)
                for (int i = 0; i < s->n_tenants; ++i)
                    if (!ctx->tenants[i]->model.ops.empty())
                        HIP_TRY(hipEventElapsedTime(&tm->tenant_done_ms[i], ctx->ev_start, ctx->ev_last[i]));
            hipEvent_t prev = ctx->ev_start;
            if (s->n_stages == 1) tm->stage_ms[0] = tm->makespan_ms;      // the same pair of events
            for (int st = 0; st < s->n_stages && s->n_stages > 1 && !ends_on_streams(s); ++st) {
                HIP_TRY(hipEventElapsedTime(&tm->stage_ms[st], prev, ctx->ev_stage[st]));
                prev = ctx->ev_stage[st];
            }
        }
    }
    return MT_OK;
}

int32_t mt_profile_ops(mt_ctx *ctx, int32_t tenant, const void *input, void *output, int32_t repeats, float *op_ms) {
    if (!ctx || !input || !output || !op_ms) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (tenant < 0 || tenant >= (int)ctx->tenants.size()) return fail(MT_ERR_INVALID_ARG, "no such tenant");
    if (repeats < 1) return fail(MT_ERR_INVALID_ARG, "repeats must be >= 1");
    HIP_TRY(hipSetDevice(ctx->device));
    const Tenant &t = *ctx->tenants[tenant];
    for (size_t i = 0; i < t.args.size(); ++i) {
        OpArgs a = patched(t, (int)i, input, output);
        int32_t rc = launch_op(a, ctx->main_stream);          // warm-up, also produces the next operator's input
        if (rc != MT_OK) return rc;
        HIP_TRY(hipEventRecord(ctx->ev_prof[0], ctx->main_stream));
        for (int r = 0; r < repeats; ++r) {
            rc = launch_op(a, ctx->main_stream);
            if (rc != MT_OK) return rc;
        }
        HIP_TRY(hipEventRecord(ctx->ev_prof[1], ctx->main_stream));
        HIP_TRY(hipEventSynchronize(ctx->ev_prof[1]));
        float ms = 0;
        HIP_TRY(hipEventElapsedTime(&ms, ctx->ev_prof[0], ctx->ev_prof[1]));
        op_ms[i] = ms / repeats;
    }
    return MT_OK;
}

// ---- search ----------------------------------------------------------------------------------
namespace {
struct ProfileCost {
    mt_ctx *ctx;
    const mt_search_opts *o;
    const void *const *inputs;
    void *const *outputs;
    int n_tenants;
    const int32_t *pointers = nullptr;     // fixed while shares are searched
    const int32_t *cu_share = nullptr;     // fixed while pointers are searched
    const int32_t *prio = nullptr;         // wave priorities applied to every candidate (NULL: what the flags give)
    const int32_t *conc = nullptr;         // per-stage concurrency applied to every candidate (NULL: one stream per tenant)
    int32_t rc = MT_OK;
};

double profile_schedule(ProfileCost *pc, const int32_t *pointers, const int32_t *cu_share) {
    if (pc->rc != MT_OK) return 1e30;
    mt_schedule *s = nullptr;
    pc->rc = mt_schedule_create(pc->ctx, pc->n_tenants, pc->o->n_stages, pointers, pc->conc, cu_share, pc->o->issue_order,
                                pc->o->flags, &s);
    if (pc->rc == MT_OK && pc->prio) pc->rc = mt_schedule_set_wave_priority(s, pc->prio);
    if (pc->rc != MT_OK) { if (s) mt_schedule_destroy(s); return 1e30; }
    // The profiled latency of a candidate is the median of its timed runs: one preempted run must not decide
    // a comparison between two schedules that differ by a few percent.
    std::vector<double> samples;
    for (int r = 0; r < pc->o->warmup + pc->o->runs && pc->rc == MT_OK; ++r) {
        mt_timings tm{};
        pc->rc = mt_run(pc->ctx, s, pc->inputs, pc->outputs, &tm);
        if (r >= pc->o->warmup) samples.push_back(tm.makespan_ms);
    }
    mt_schedule_destroy(s);
    if (pc->rc == MT_OK && pc->ctx->retired_graphs.size() >= 64) pc->rc = release_retired_graphs(pc->ctx);
    double c = 1e30;
    if (pc->rc == MT_OK && !samples.empty()) {
        std::sort(samples.begin(), samples.end());
        const size_t h = samples.size() / 2;
        c = samples.size() % 2 ? samples[h] : 0.5 * (samples[h - 1] + samples[h]);
    }
    return c;
}

double profile_cost(const int32_t *pointers, void *user) {
    ProfileCost *pc = (ProfileCost *)user;
    return profile_schedule(pc, pointers, pc->cu_share);
}

double profile_share_cost(const int32_t *cu_share, void *user) {
    ProfileCost *pc = (ProfileCost *)user;
    return profile_schedule(pc, pc->pointers, cu_share);
}

double profile_prio_cost(const int32_t *prio, void *user) {
    ProfileCost *pc = (ProfileCost *)user;
    const int32_t *keep = pc->prio;
    pc->prio = prio;
    const double c = profile_schedule(pc, pc->pointers, pc->cu_share);
    pc->prio = keep;
    return c;
}
}  // namespace

int32_t mt_search(mt_ctx *ctx, const mt_search_opts *opts, const void *const *inputs, void *const *outputs,
                  int32_t *best_pointers, int32_t *best_concurrency, int32_t *best_cu_share, int32_t *best_wave_priority, double *best_cost,
                  int32_t *rec_pointers, double *rec_cost, int32_t max_records, int32_t *n_records) {
    if (!ctx || !opts || !inputs || !outputs || !best_pointers) return fail(MT_ERR_INVALID_ARG, "NULL argument");
    if (opts->runs < 1 || opts->warmup < 0) return fail(MT_ERR_INVALID_ARG, "runs must be >= 1 and warmup >= 0");
    const int n = (int)ctx->tenants.size();
    if (n < 1) return fail(MT_ERR_INVALID_ARG, "no tenants registered");
    if (opts->cu_share_rounds > 0 && (opts->flags & MT_SCHED_GRAPH))
        return fail(MT_ERR_INVALID_ARG, "CU shares have no effect under graph replay");
    int32_t lens[MT_MAX_TENANTS];
    for (int i = 0; i < n; ++i) lens[i] = (int32_t)ctx->tenants[i]->model.ops.size();
    ProfileCost pc{ctx, opts, inputs, outputs, n};
    double cost = 0;
    // The play-off needs the whole record memory: when the caller's buffer is absent or may be too small the search
    // records into a buffer of its own, and the caller's one is filled from it afterwards.
    const int P = opts->n_stages - 1;
    const size_t width = (size_t)n * P;
    const bool playoff = opts->playoff_top > 0 && P > 0;
    const int32_t need = (int32_t)std::min<int64_t>((int64_t)opts->rounds * n * opts->candidates + 2, 1 << 24);
    std::vector<int32_t> own_p;
    std::vector<double> own_c;
    int32_t *rp = rec_pointers;
    double *rcst = rec_cost;
    int32_t cap = max_records;
    if (playoff && (!rec_pointers || !rec_cost || max_records < need)) {
        own_p.assign((size_t)need * std::max<size_t>(1, width), 0);
        own_c.assign((size_t)need, 0.0);
        rp = own_p.data(); rcst = own_c.data(); cap = need;
    }
    int32_t n_rec = 0;
    int32_t rc = search_pointers(n, lens, opts, profile_cost, &pc, best_pointers, &cost, rp, rcst, cap, &n_rec);
    if (pc.rc != MT_OK) return pc.rc;
    if (rc != MT_OK) return rc;
    if (n_records) *n_records = n_rec;
    if (rp != rec_pointers && rec_pointers && rec_cost) {
        const int32_t keep = std::min(std::min(n_rec, cap), max_records);
        if (keep > 0) {
            std::memcpy(rec_pointers, rp, sizeof(int32_t) * width * keep);
            std::memcpy(rec_cost, rcst, sizeof(double) * keep);
        }
    }
    if (playoff) {
        // Alg. 1 returns the best record as it was profiled once; schedules a few percent apart are not separated by
        // one short measurement, so the leaders (and the one-stage matrix) are measured again, longer.
        mt_search_opts longer = *opts;
        longer.runs = opts->playoff_runs >= 1 ? opts->playoff_runs : 21;
        ProfileCost pcf{ctx, &longer, inputs, outputs, n};
        rc = playoff_pointers(n, lens, opts->n_stages, rp, rcst, std::min(n_rec, cap), opts->playoff_top, profile_cost, &pcf,
                              best_pointers, &cost, nullptr);
        if (pcf.rc != MT_OK) return pcf.rc;
        if (rc != MT_OK) return rc;
    }
    // Streams in use at a time, the same number in every stage: the queues of this machine are served by four dispatch
    // pipes (see PlainPool), so with five tenants or more fewer streams than tenants can be faster.
    int32_t conc[MT_MAX_STAGES];
    for (int st = 0; st < opts->n_stages; ++st) conc[st] = n;
    if (opts->search_concurrency && n > 2) {
        int32_t trial[MT_MAX_STAGES];
        int best_c = n;
        pc.conc = trial;
        // `cost` comes from the longer runs of the play-off when there was one: the stream counts are then measured
        // the same way, so that one of them replaces "one stream per tenant" only on an equal footing
        mt_search_opts longer = *opts;
        if (playoff) longer.runs = opts->playoff_runs >= 1 ? opts->playoff_runs : 21;
        ProfileCost pcl{ctx, &longer, inputs, outputs, n};
        pcl.conc = trial;
        // Two passes over the counts, the lower figure of each counts: a stream set that runs for the first time can
        // stay slow for tens of milliseconds (measured: eight ResNet-50 on four streams 4.66 ms at first, 3.16 ms later)
        for (int pass = 0; pass < (playoff ? 2 : 1); ++pass)
            for (int c = 2; c < n; ++c) {
                for (int st = 0; st < opts->n_stages; ++st) trial[st] = c;
                const double cc = profile_schedule(&pcl, best_pointers, nullptr);
                if (pcl.rc != MT_OK) return pcl.rc;
                if (cc < cost) { cost = cc; best_c = c; }
            }
        for (int st = 0; st < opts->n_stages; ++st) conc[st] = best_c;
        pc.conc = best_c == n ? nullptr : conc;
    }
    int32_t shares[MT_MAX_TENANTS] = {0};
    const double unmasked_cost = cost;
    std::vector<int32_t> unmasked_pointers(best_pointers, best_pointers + (size_t)n * (opts->n_stages - 1));
    if (opts->cu_share_rounds > 0) {
        // Shares are searched under the pointers just found.  The descent starts from the best of four vectors:
        // all zeros (every tenant on every unit, whose cost is known), a disjoint split in proportion to the serial
        // latency of each tenant, and two uniform overlapping ones (below); a descent from all zeros alone rarely leaves it, because one masked tenant
        // among unmasked ones gains nothing.
        pc.pointers = best_pointers;
        const int cus = ctx->prop.multiProcessorCount;
        double weight[MT_MAX_TENANTS];
        std::vector<float> op_ms;
        for (int i = 0; i < n; ++i) {
            op_ms.assign((size_t)lens[i], 0.f);
            rc = mt_profile_ops(ctx, i, inputs[i], outputs[i], 3, op_ms.data());
            if (rc != MT_OK) return rc;
            weight[i] = 0;
            for (float v : op_ms) weight[i] += v;
        }
        int32_t start[MT_MAX_TENANTS];
        rc = proportional_cu_share(n, cus, weight, start);
        if (rc != MT_OK) return rc;
        // Two more start vectors give every tenant the same share, one half and three quarters of the units: the
        // shares then overlap (tenant i's units follow those of tenant i - 1, modulo the unit count), which keeps a
        // heavy tenant apart from some of the others without starving it.
        for (int cand = 0; cand < 3; ++cand) {
            if (cand > 0)
                for (int i = 0; i < n; ++i) start[i] = std::max(8, (cand == 1 ? cus / 2 : 3 * cus / 4) / 8 * 8);
            const double start_cost = profile_share_cost(start, &pc);
            if (pc.rc != MT_OK) return pc.rc;
            if (start_cost < cost) {
                std::memcpy(shares, start, sizeof(int32_t) * n);
                cost = start_cost;
            }
        }
        rc = search_cu_share(n, cus, opts->cu_share_rounds, profile_share_cost, &pc, shares, &cost);
        if (pc.rc != MT_OK) return pc.rc;
        if (rc != MT_OK) return rc;
        bool masked = false;
        for (int i = 0; i < n; ++i) masked = masked || shares[i] != 0;
        if (masked && opts->n_stages > 1) {
            // The stage boundaries were chosen while the tenants competed for every unit; search them once more under
            // the shares found and keep the result only if it is better.
            pc.cu_share = shares;
            std::vector<int32_t> rho2((size_t)n * (opts->n_stages - 1));
            double cost2 = 0;
            int32_t n2 = 0;
            rc = search_pointers(n, lens, opts, profile_cost, &pc, rho2.data(), &cost2, nullptr, nullptr, 0, &n2);
            if (pc.rc != MT_OK) return pc.rc;
            if (rc != MT_OK) return rc;
            if (cost2 < cost) {
                std::memcpy(best_pointers, rho2.data(), sizeof(int32_t) * rho2.size());
                cost = cost2;
            }
        }
    }
    if (opts->cu_share_rounds > 0) {
        rc = purge_idle_streams(ctx);     // leave the caller a process with few hardware queues
        if (rc != MT_OK) return rc;
        bool masked = false;
        for (int i = 0; i < n; ++i) masked = masked || shares[i] != 0;
        if (masked) {
            // The winner is measured once more on fresh streams, which stay in the pool for the caller's schedule:
            // a masked queue can come up slow, and a result that only held on the queues of the search is worth
            // nothing.  After three slow attempts the unmasked result of the pointer search is returned instead.
            pc.cu_share = nullptr;
            double again = 1e30;
            for (int attempt = 0; attempt < 3; ++attempt) {
                again = profile_schedule(&pc, best_pointers, shares);
                if (pc.rc != MT_OK) return pc.rc;
                if (again <= 1.1 * cost || again < unmasked_cost) break;
                rc = purge_idle_streams(ctx);
                if (rc != MT_OK) return rc;
            }
            if (again < unmasked_cost) {
                cost = again;
            } else {
                std::memcpy(best_pointers, unmasked_pointers.data(), sizeof(int32_t) * unmasked_pointers.size());
                std::memset(shares, 0, sizeof(shares));
                cost = unmasked_cost;
                rc = purge_idle_streams(ctx);
                if (rc != MT_OK) return rc;
            }
        }
    }
    int32_t prio[MT_MAX_TENANTS];
    for (int i = 0; i < n; ++i) prio[i] = (opts->flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0;
    if (opts->wave_priority_rounds > 0) {
        // Last coordinate set: the wave priority of each tenant's kernels, under the pointers and shares found.
        bool masked = false;
        for (int i = 0; i < n; ++i) masked = masked || shares[i] != 0;
        pc.pointers = best_pointers;
        pc.cu_share = masked ? shares : nullptr;
        rc = search_wave_priority(n, opts->wave_priority_rounds, profile_prio_cost, &pc, prio, &cost);
        if (pc.rc != MT_OK) return pc.rc;
        if (rc != MT_OK) return rc;
        if (masked) {
            // Priorities matter most where tenants share units, which masks prevent: the unmasked result of the pointer
            // search gets its own descent and wins if it ends lower.
            int32_t prio_u[MT_MAX_TENANTS];
            for (int i = 0; i < n; ++i) prio_u[i] = (opts->flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0;
            double cost_u = unmasked_cost;
            pc.pointers = unmasked_pointers.data();
            pc.cu_share = nullptr;
            rc = search_wave_priority(n, opts->wave_priority_rounds, profile_prio_cost, &pc, prio_u, &cost_u);
            if (pc.rc != MT_OK) return pc.rc;
            if (rc != MT_OK) return rc;
            if (cost_u < cost) {
                cost = cost_u;
                std::memcpy(prio, prio_u, sizeof(int32_t) * n);
                std::memcpy(best_pointers, unmasked_pointers.data(), sizeof(int32_t) * unmasked_pointers.size());
                std::memset(shares, 0, sizeof(shares));
                rc = purge_idle_streams(ctx);
                if (rc != MT_OK) return rc;
            }
        }
    }
    if (playoff && opts->wave_priority_rounds > 0) {
        // The descent over priorities accepts every candidate that measured lower, 4 n of them per round on short
        // runs: what it returns is measured against the default priorities with the longer runs, twice in turn, and
        // kept only if it is lower there too.
        bool changed = false;
        for (int i = 0; i < n; ++i) changed = changed || prio[i] != ((opts->flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0);
        if (changed) {
            mt_search_opts longer = *opts;
            longer.runs = opts->playoff_runs >= 1 ? opts->playoff_runs : 21;
            bool masked = false;
            for (int i = 0; i < n; ++i) masked = masked || shares[i] != 0;
            double with = 1e30, without = 1e30;
            for (int turn = 0; turn < 2; ++turn) {
                ProfileCost pa{ctx, &longer, inputs, outputs, n};
                pa.conc = conc[0] == n ? nullptr : conc;
                pa.prio = prio;
                with = std::min(with, profile_schedule(&pa, best_pointers, masked ? shares : nullptr));
                if (pa.rc != MT_OK) return pa.rc;
                ProfileCost pb{ctx, &longer, inputs, outputs, n};
                pb.conc = conc[0] == n ? nullptr : conc;
                without = std::min(without, profile_schedule(&pb, best_pointers, masked ? shares : nullptr));
                if (pb.rc != MT_OK) return pb.rc;
            }
            if (without <= with) {
                for (int i = 0; i < n; ++i) prio[i] = (opts->flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0;
                cost = without;
            } else {
                cost = with;
            }
        }
    }
    if (playoff) {
        // Last check: the result as a whole (pointers, stream count, shares, priorities) against the plain configuration
        // it started from (everything in stage 1, one stream per tenant, no shares, default priorities), both measured
        // twice in turn with the longer runs.  The coordinates were accepted one after the other on single
        // measurements; if together they do not beat the start, the start is returned.
        bool plain = true;
        for (int i = 0; i < n; ++i) plain = plain && shares[i] == 0 && prio[i] == ((opts->flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0);
        for (int st = 0; st < opts->n_stages; ++st) plain = plain && conc[st] == n;
        for (size_t k = 0; k < width; ++k) plain = plain && best_pointers[k] >= lens[k / P];
        if (!plain) {
            mt_search_opts longer = *opts;
            longer.runs = opts->playoff_runs >= 1 ? opts->playoff_runs : 21;
            std::vector<int32_t> all_first(width);
            for (size_t k = 0; k < width; ++k) all_first[k] = lens[k / P];
            bool masked = false;
            for (int i = 0; i < n; ++i) masked = masked || shares[i] != 0;
            double found = 1e30, start = 1e30;
            for (int turn = 0; turn < 2; ++turn) {
                ProfileCost pa{ctx, &longer, inputs, outputs, n};
                pa.conc = conc[0] == n ? nullptr : conc;
                pa.prio = prio;
                found = std::min(found, profile_schedule(&pa, best_pointers, masked ? shares : nullptr));
                if (pa.rc != MT_OK) return pa.rc;
                ProfileCost pb{ctx, &longer, inputs, outputs, n};
                start = std::min(start, profile_schedule(&pb, all_first.data(), nullptr));
                if (pb.rc != MT_OK) return pb.rc;
            }
            if (start < found) {
                std::memcpy(best_pointers, all_first.data(), sizeof(int32_t) * width);
                for (int st = 0; st < opts->n_stages; ++st) conc[st] = n;
                std::memset(shares, 0, sizeof(shares));
                for (int i = 0; i < n; ++i) prio[i] = (opts->flags & MT_SCHED_PRIORITIZE_SHORT) ? -1 : 0;
                cost = start;
            } else {
                cost = found;
            }
        }
    }
    rc = release_retired_graphs(ctx);          // what the candidates of a search under graph replay left behind
    if (rc != MT_OK) return rc;
    if (best_wave_priority) std::memcpy(best_wave_priority, prio, sizeof(int32_t) * n);
    if (best_concurrency) std::memcpy(best_concurrency, conc, sizeof(int32_t) * opts->n_stages);
    if (best_cu_share) std::memcpy(best_cu_share, shares, sizeof(int32_t) * n);
    if (best_cost) *best_cost = cost;
    return MT_OK;
}

}  // extern "C"
