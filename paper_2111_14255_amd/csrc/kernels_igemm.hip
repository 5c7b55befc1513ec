// Convolution and fully connected layers as an implicit GEMM on the gfx950 matrix cores.
//
//   D[k, m] = sum_j Wp[k, j] * A[m, j]        k: output channel, m: output pixel (n, p, q), j: (r, s, c)
//
// Wp is the filter bank packed at registration time as [n_pad][k_pad] (rows = output channels, zero padded
// to whole tiles), so its tiles are plain 16-byte loads.  A is never materialised: a tile row is gathered
// from the NHWC activation, where eight consecutive j with C % 8 == 0 are eight consecutive channels of one
// input pixel, i.e. one 16-byte load (or zeros in the padding halo).  Both tiles are staged in LDS with the
// reduction index contiguous, which is the operand layout of v_mfma_f32_32x32x16 / 16x16x32 (each lane feeds
// 8 consecutive j of one row).  The filter bank is the MFMA "A" operand, so a lane's accumulator registers
// hold four consecutive output channels of one pixel: the NHWC store is an 8-byte access per group.
//
// Pipeline: global loads run STAGES reduction tiles ahead in registers, LDS is double buffered, one
// workgroup barrier per tile.  fp16 / bf16 inputs, fp32 accumulation; bias, residual, activation in fp32;
// one rounding on store.
//
// Tiny-M layers are split along j across workgroups.  Partial sums go to a workspace with device-coherent
// (write-through) stores, and the workgroup that arrives last at the tile's counter adds them in split
// order, so the result does not depend on arrival order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <type_traits>
#include <utility>

#include "internal.h"
#include "device_types.h"
#include "mfma.h"

namespace mt {

constexpr int BK = IGEMM_BK;     // reduction elements per LDS tile
constexpr int LDK = BK + 8;      // padded LDS row (144 bytes: 16-byte reads of a wave fall in distinct banks)
constexpr int NXCD = 8;
constexpr int A_SCALAR = 0, A_VEC8 = 1, A_UNIFORM = 2;
constexpr uint32_t OOB_OFFSET = 0x80000000u;   // beyond any tensor: buffer loads return zeros
// Fused 1x1 + depthwise kernel: channels of the widened tensor per workgroup, workgroups wanted at least, and 8-channel
// chunks of depthwise output a workgroup takes at most (measured on MobileNetV2 at batch 1: 32 channels per workgroup
// are 7 % slower, 256 to 1024 chunks 1 to 4 % slower).
constexpr int PWDW_HC = 16, PWDW_WGS = 64, PWDW_ITEMS = 128;

// BN: output channels per workgroup, BM: pixels per workgroup, WN x WM: wave grid (4 waves), MF: MFMA edge,
// STAGES: reduction tiles whose global loads are in flight (register sets), even.
// AMODE: how a tile row of the im2col matrix is gathered:
//   A_UNIFORM  C % 64 == 0 and R*S <= 64: a 64-deep tile lies inside one filter tap, so the tap walks in
//              scalar registers and a lane only selects between its pixel's offset and "out of range"
//   A_VEC8     C % 8 == 0: every lane tracks the tap of its own 8-channel chunk
//   A_SCALAR   any C (first layers, C = 3): element-wise gather
// Filter tiles and (except A_SCALAR) im2col chunks are fetched with buffer loads: offsets are 32 bit, the
// tile walk is a scalar offset, and a chunk in the padding halo is given an out-of-range offset, for which
// the hardware returns zeros: no select and no 64-bit address arithmetic in the loop.
template <typename T, int BN, int BM, int WN, int WM, int MF, int STAGES, int AMODE, int WK = 1>
__device__ __forceinline__ void igemm_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    static_assert(WN * WM == 4, "four waves per output tile");
    // WK > 1: WK groups of four waves share the output tile and split the MFMA steps of every LDS tile between them
    // (a second wave per SIMD to overlap with when the grid gives a compute unit a single workgroup); their
    // accumulators are added through LDS after the main loop, in group order.
    constexpr int NT = 256 * WK;
    static_assert(STAGES >= 2 && STAGES % 2 == 0, "register sets rotate with the two LDS buffers");
    constexpr int SUBN = BN / WN, SUBM = BM / WM;          // wave tile
    constexpr int TN = SUBN / MF, TM = SUBM / MF;          // MFMA tiles per wave
    static_assert(TN >= 1 && TM >= 1, "wave tile smaller than one MFMA");
    constexpr int KSTEPS_TILE = (MF == 32) ? BK / 16 : BK / 32;   // MFMA steps per LDS tile
    static_assert(KSTEPS_TILE % WK == 0, "the wave groups split the MFMA steps evenly");
    constexpr int KSTEPS = KSTEPS_TILE / WK;               // MFMA issues per LDS tile and wave
    constexpr int KLANES = 64 / MF;                        // lane groups along the reduction index
    constexpr int ACC_REGS = (MF == 32) ? 16 : 4;
    constexpr int CH_ROW = BK / 8;                         // 16-byte chunks per tile row
    constexpr int ROW_STEP = NT / CH_ROW;                  // tile rows covered by one pass of the workgroup
    constexpr int W_CHUNKS = (BN + ROW_STEP - 1) / ROW_STEP;
    constexpr int X_CHUNKS = (BM + ROW_STEP - 1) / ROW_STEP;
    typedef typename Mma<T, MF>::Acc Acc;

    // One LDS block: two filter tile buffers, then two im2col tile buffers; reused for the accumulator exchange.
    constexpr int W_TILE = W_CHUNKS * ROW_STEP * LDK, X_TILE = X_CHUNKS * ROW_STEP * LDK;
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * (W_TILE + X_TILE)];
    uint16_t(*Ws)[W_TILE] = reinterpret_cast<uint16_t(*)[W_TILE]>(&smem[0]);
    uint16_t(*Xs)[X_TILE] = reinterpret_cast<uint16_t(*)[X_TILE]>(&smem[2 * W_TILE]);
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wk = wave / 4;                               // wave group along the reduction index
    const int wn = (wave % 4) % WN, wm = (wave % 4) / WN;

    // Workgroup ids are dealt round-robin to the 8 XCDs; remap so that each XCD (one L2) works on a
    // contiguous range of tiles and the tiles sharing an activation tile share an L2.
    const int M = a.N * a.P * a.Q;
    const int tiles_m = (M + BM - 1) / BM;
    const int tiles_n = a.n_pad / BN;
    const int total = tiles_m * tiles_n * a.split_k;
    const int per_xcd = (total + NXCD - 1) / NXCD;
    const int vid = (blockIdx.x % NXCD) * per_xcd + blockIdx.x / NXCD;
    if (vid >= total) return;
    const int z = vid % a.split_k;
    const int tile = vid / a.split_k;
    const int tn_idx = a.tile_order ? tile / tiles_m : tile % tiles_n;
    const int tm_idx = a.tile_order ? tile % tiles_m : tile / tiles_n;
    const int n0 = tn_idx * BN;
    const int m0 = tm_idx * BM;

    const int nkt = a.k_pad / BK;
    const int kt_per = (nkt + a.split_k - 1) / a.split_k;
    const int kt_begin = z * kt_per;
    const int nk = min(nkt, kt_begin + kt_per) - kt_begin;     // tiles of this workgroup (>= 1 by construction)

    const int XS = a.x_ct;                 // channels per pixel of the input buffer (> C for a grouped convolution)
    const T *x = (const T *)a.x + a.x_coff;
    const uint16_t *wp = (const uint16_t *)a.w;

    // ---- per-thread load coordinates -------------------------------------------------------
    const int kc = tid % CH_ROW;          // chunk column (same for every chunk of this thread)
    const int row0 = tid / CH_ROW;        // first tile row; further chunks are ROW_STEP rows apart

    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T *>(x), 0, (int)(((int64_t)a.N * a.H * a.W * XS - a.x_coff) * (int)sizeof(T)), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(wp), 0, (int)((int64_t)a.n_pad * a.k_pad * 2), 0x00027000);

    int img_off[X_CHUNKS];                // element offset of input pixel (n, 0, 0, 0) of the chunk's tile row
    int ih0[X_CHUNKS], iw0[X_CHUNKS];
    bool xrow_ok[X_CHUNKS];
#pragma unroll
    for (int i = 0; i < X_CHUNKS; ++i) {
        const int row = row0 + i * ROW_STEP;
        const int m = m0 + row;
        xrow_ok[i] = (row < BM) & (m < M);
        const uint32_t mm = xrow_ok[i] ? (uint32_t)m : 0u;
        // pixel index -> (image, row, column) by multiply-high divisions: a divide instruction sequence per row is a
        // large part of the prologue of a short, latency-bound launch
        // With the pooled epilogue the pixel index walks 2x2 quads (quad index * 4 + position inside the quad) and the
        // divisors are those of the pooled map, so four consecutive tile rows are one pooling window.
        const uint32_t mq = a.pool2 ? mm >> 2 : mm;
        const uint32_t pqd = a.pool2 ? (uint32_t)((a.P >> 1) * (a.Q >> 1)) : (uint32_t)(a.P * a.Q);
        const uint32_t qd = a.pool2 ? (uint32_t)(a.Q >> 1) : (uint32_t)a.Q;
        const uint32_t t1 = __umulhi(a.divpq_m, mq);
        const int n = (int)((t1 + ((mq - t1) >> a.divpq_s1)) >> a.divpq_s2);
        const uint32_t rem = mq - (uint32_t)n * pqd;
        const uint32_t t2 = __umulhi(a.divq_m, rem);
        int p = (int)((t2 + ((rem - t2) >> a.divq_s1)) >> a.divq_s2);
        int q = (int)(rem - (uint32_t)p * qd);
        if (a.pool2) {
            p = 2 * p + (int)((mm >> 1) & 1u);
            q = 2 * q + (int)(mm & 1u);
        }
        img_off[i] = n * a.H * a.W * XS;
        ih0[i] = p * a.sh - a.ph;
        iw0[i] = q * a.sw - a.pw;
    }
    uint32_t wvoff[W_CHUNKS];             // byte offset of the chunk inside the packed filter bank, tile 0
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) {
        const int row = min(row0 + i * ROW_STEP, BN - 1);
        wvoff[i] = (uint32_t)(((n0 + row) * a.k_pad + kc * 8) * 2);
    }
    uint32_t wsoff = (uint32_t)(kt_begin * BK * 2);     // scalar: byte offset of the current tile in a filter row

    // A_UNIFORM: the tap (r, s) and the channel base of the current tile are wave-uniform.
    int u_r = 0, u_s = 0, u_tap = 0, u_cb = 0;
    uint64_t tapmask[X_CHUNKS];           // bit r*S+s: the tap reads inside the image for this chunk's pixel
    int rowoff[X_CHUNKS];                 // byte offset of (n, ih0, iw0, kc*8)
    // A_VEC8 / A_SCALAR: position of this thread's chunk inside the (r, s, c) reduction index.
    const int adv_c = BK % a.C, adv_rs = BK / a.C;
    const uint32_t inv_s = (uint32_t)((0x100000000ull + (uint32_t)a.S - 1) / (uint32_t)a.S);   // wraps to 0 for S == 1
    auto tap_row = [&](int rs) { return a.S == 1 ? rs : (int)__umulhi((uint32_t)rs, inv_s); };
    int kcx = 0, krs = 0;
    int jbase = kt_begin * BK + kc * 8;
    if constexpr (AMODE == A_UNIFORM) {
        const int j0 = kt_begin * BK;
        u_cb = j0 % a.C;
        u_tap = j0 / a.C;
        u_r = u_tap / a.S;
        u_s = u_tap - u_r * a.S;
#pragma unroll
        for (int i = 0; i < X_CHUNKS; ++i) {
            uint64_t mask = 0;
            for (int r = 0; r < a.R; ++r)
                for (int sx = 0; sx < a.S; ++sx) {
                    const bool v = xrow_ok[i] & ((uint32_t)(ih0[i] + r) < (uint32_t)a.H) & ((uint32_t)(iw0[i] + sx) < (uint32_t)a.W);
                    mask |= (uint64_t)(v ? 1u : 0u) << (r * a.S + sx);
                }
            tapmask[i] = mask;
            rowoff[i] = (img_off[i] + (ih0[i] * a.W + iw0[i]) * XS + kc * 8) * 2;
        }
    } else {
        const int j0 = kt_begin * BK + kc * 8;
        kcx = j0 % a.C;
        krs = j0 / a.C;
    }

    u32x4 wreg[STAGES][W_CHUNKS], xreg[STAGES][X_CHUNKS];

    // A tile is fetched and copied to LDS chunk by chunk (filter chunks first, then im2col chunks), so that the main
    // loop can spread the chunks of the next tiles between the matrix instructions of the current one.  All loads are
    // straight-line code: the compiler counts them exactly and lets the newer register sets stay in flight while the
    // oldest one is consumed.
    constexpr int NCH = W_CHUNKS + X_CHUNKS;
    int t_tapoff = 0, t_sh = 0, t_kr = 0, t_ks = 0;      // per-tile values of the im2col gather, set by tile_begin
    bool t_tap_ok = false;
    auto tile_begin = [&]() {
        if constexpr (AMODE == A_UNIFORM) {
            t_tapoff = ((u_r * a.W + u_s) * XS + u_cb) * 2;                // scalar
            t_tap_ok = u_tap < a.R * a.S;
            t_sh = t_tap_ok ? u_tap : 0;
        } else if constexpr (AMODE == A_VEC8) {
            t_kr = tap_row(krs);
            t_ks = krs - t_kr * a.S;
        }
    };
    auto load_chunk = [&]<int I>(u32x4 (&wr)[W_CHUNKS], u32x4 (&xr)[X_CHUNKS]) {
        if constexpr (I < W_CHUNKS) {
            wr[I] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, wvoff[I], wsoff, 0);
        } else if constexpr (AMODE == A_UNIFORM) {
            constexpr int i = I - W_CHUNKS;
            const bool v = t_tap_ok & (((tapmask[i] >> t_sh) & 1ull) != 0);
            const uint32_t voff = v ? (uint32_t)(rowoff[i] + t_tapoff) : OOB_OFFSET;
            xr[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, voff, 0, 0);
        } else if constexpr (AMODE == A_VEC8) {
            constexpr int i = I - W_CHUNKS;
            const int ih = ih0[i] + t_kr, iw = iw0[i] + t_ks;
            const bool v = xrow_ok[i] & (t_kr < a.R) & ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
            const uint32_t voff = v ? (uint32_t)((img_off[i] + (ih * a.W + iw) * XS + kcx) * 2) : OOB_OFFSET;
            xr[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, voff, 0, 0);
        } else {
            // input channels not a multiple of 8 (first layers, C = 3): gather element by element
            constexpr int i = I - W_CHUNKS;
            const uint16_t *xs = reinterpret_cast<const uint16_t *>(x);
            uint32_t e[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int j = jbase + t;
                const int rs = j / a.C;
                const int c = j - rs * a.C;
                const int r = tap_row(rs);
                const int sx = rs - r * a.S;
                const int ih = ih0[i] + r, iw = iw0[i] + sx;
                const bool v = xrow_ok[i] & (j < a.gemm_k) & ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
                const int off = v ? img_off[i] + (ih * a.W + iw) * XS + c : 0;
                const uint32_t h = xs[off];
                e[t] = v ? h : 0u;
            }
            xr[i] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
        }
    };
    auto tile_end = [&]() {
        wsoff += BK * 2;
        if constexpr (AMODE == A_UNIFORM) {
            u_cb += BK;
            if (u_cb >= a.C) {              // scalar branch-free updates (uniform values)
                u_cb = 0;
                ++u_tap;
                ++u_s;
                if (u_s == a.S) {
                    u_s = 0;
                    ++u_r;
                }
            }
        } else if constexpr (AMODE == A_VEC8) {
            kcx += adv_c;
            krs += adv_rs;
            const bool carry = kcx >= a.C;
            kcx -= carry ? a.C : 0;
            krs += carry ? 1 : 0;
        } else {
            jbase += BK;
        }
    };
    // Every thread writes its chunks: tile rows beyond BN / BM land in spare LDS rows that nobody reads.
    auto store_chunk = [&]<int I>(int buf, const u32x4 (&wr)[W_CHUNKS], const u32x4 (&xr)[X_CHUNKS]) {
        if constexpr (I < W_CHUNKS) {
            *reinterpret_cast<u32x4 *>(&Ws[buf][(row0 + I * ROW_STEP) * LDK + kc * 8]) = wr[I];
        } else {
            constexpr int i = I - W_CHUNKS;
            *reinterpret_cast<u32x4 *>(&Xs[buf][(row0 + i * ROW_STEP) * LDK + kc * 8]) = xr[i];
        }
    };
    auto load_tiles = [&](u32x4 (&wr)[W_CHUNKS], u32x4 (&xr)[X_CHUNKS]) {
        tile_begin();
        [&]<int... I>(std::integer_sequence<int, I...>) {
            (load_chunk.template operator()<I>(wr, xr), ...);
        }(std::make_integer_sequence<int, NCH>{});
        tile_end();
    };
    auto store_tiles = [&](int buf, const u32x4 (&wr)[W_CHUNKS], const u32x4 (&xr)[X_CHUNKS]) {
        [&]<int... I>(std::integer_sequence<int, I...>) {
            (store_chunk.template operator()<I>(buf, wr, xr), ...);
        }(std::make_integer_sequence<int, NCH>{});
    };

    Acc acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < ACC_REGS; ++v) acc[i][j][v] = 0.f;

    const int frag_row = lane % MF;
    const int frag_k = (lane / MF) * 8;

    // Bias of this lane's output channels, fetched before the main loop so that the epilogue of a short,
    // latency-bound workgroup does not start with another round trip to memory (the bank is padded to n_pad).
    constexpr int GROUPS = ACC_REGS / 4;
    constexpr bool BIAS_EARLY = TN * GROUPS <= 4;
    float4 bias_pre[BIAS_EARLY ? TN * GROUPS : 1];
    if constexpr (BIAS_EARLY) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const int k = n0 + wn * SUBN + i * MF + ((MF == 32) ? (8 * g + 4 * (lane / 32)) : (4 * (lane / 16)));
                bias_pre[i * GROUPS + g] = *reinterpret_cast<const float4 *>(a.bias + k);
            }
    }

    // MFMA operand fragments of one reduction step (16 or 32 elements deep) of an LDS tile.  The fragments of step
    // kk + 1 are requested before the matrix instructions of step kk are issued, so that a wave's LDS reads run under
    // its own MFMA work instead of in front of it; the accumulation order (kk, then channel tile, then pixel tile) is
    // that of a plain loop.
    struct Frag {
        u32x4 a[TN], b[TM];
    };
    auto load_frag = [&](int buf, int kk, Frag &f) {
        const int koff = (wk * KSTEPS + kk) * (KLANES * 8) + frag_k;
#pragma unroll
        for (int i = 0; i < TN; ++i)
            f.a[i] = *reinterpret_cast<const u32x4 *>(&Ws[buf][(wn * SUBN + i * MF + frag_row) * LDK + koff]);
#pragma unroll
        for (int j = 0; j < TM; ++j)
            f.b[j] = *reinterpret_cast<const u32x4 *>(&Xs[buf][(wm * SUBM + j * MF + frag_row) * LDK + koff]);
    };
    auto mma = [&](const Frag &f) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) acc[i][j] = Mma<T, MF>::run(f.a[i], f.b[j], acc[i][j]);
    };

    auto prologue_load = [&]<int S>() {
        if (S < nk) load_tiles(wreg[S], xreg[S]);
    };
    [&]<int... S>(std::integer_sequence<int, S...>) {
        (prologue_load.template operator()<S>(), ...);
    }(std::make_integer_sequence<int, STAGES>{});

    // Tile t waits in register set t % STAGES until it is copied to LDS buffer t % 2.  FULL steps are the
    // steady state (every tile they touch exists) and contain no branch.
    {
        Frag fr[2];
        // One reduction tile: the chunks of tile t + 1 go from registers to the other LDS buffer and the chunks of tile
        // t + 1 + STAGES are requested from memory, a few after each reduction step of tile t, whose fragments are read
        // one step ahead of the matrix instructions that use them.
        // Spreading pays on the wide tiles (measured on MI355X: a 3x3 layer of 256 channels on a 56x56 map at batch 8,
        // 128x128 tile, 49.8 -> 44.8 us); tiles of few chunks per thread move them all before the first step.
        constexpr int PER = NCH >= 8 ? (NCH + KSTEPS - 1) / KSTEPS : NCH;   // chunks moved per reduction step
        auto step = [&]<int S, bool FULL>(int t) {
            constexpr int nxt = (S + 1) % STAGES;
            if (FULL || t < nk) {
                const bool more = FULL || t + 1 < nk;
                const bool fetch = FULL || t + 1 + STAGES < nk;
                constexpr bool SPREAD = PER < NCH;
                if constexpr (!SPREAD) {
                    if (more) {
                        store_tiles((S + 1) & 1, wreg[nxt], xreg[nxt]);
                        if (fetch) load_tiles(wreg[nxt], xreg[nxt]);
                    }
                } else {
                    if (fetch) tile_begin();
                }
                auto move_chunk = [&]<int C>() {
                    if constexpr (C < NCH) {
                        if (more) store_chunk.template operator()<C>((S + 1) & 1, wreg[nxt], xreg[nxt]);
                        if (fetch) load_chunk.template operator()<C>(wreg[nxt], xreg[nxt]);
                    }
                };
                auto kstep = [&]<int KK>() {
                    if constexpr (KK + 1 < KSTEPS) load_frag(S & 1, KK + 1, fr[(KK + 1) & 1]);
                    if constexpr (SPREAD) {
                        [&]<int... CI>(std::integer_sequence<int, CI...>) {
                            (move_chunk.template operator()<KK * PER + CI>(), ...);
                        }(std::make_integer_sequence<int, PER>{});
                    }
                    mma(fr[KK & 1]);
                };
                [&]<int... KK>(std::integer_sequence<int, KK...>) {
                    (kstep.template operator()<KK>(), ...);
                }(std::make_integer_sequence<int, KSTEPS>{});
                if constexpr (SPREAD) {
                    if (fetch) tile_end();
                }
                __syncthreads();
                if (more) load_frag((S + 1) & 1, 0, fr[0]);
            }
        };
        store_tiles(0, wreg[0], xreg[0]);
        if (STAGES < nk) load_tiles(wreg[0], xreg[0]);
        __syncthreads();
        load_frag(0, 0, fr[0]);
        auto round = [&]<bool FULL, int... S>(int t0, std::integer_sequence<int, S...>) {
            (step.template operator()<S, FULL>(t0 + S), ...);
        };
        int t0 = 0;
        for (; t0 + 2 * STAGES < nk; t0 += STAGES) round.template operator()<true>(t0, std::make_integer_sequence<int, STAGES>{});
        for (; t0 < nk; t0 += STAGES) round.template operator()<false>(t0, std::make_integer_sequence<int, STAGES>{});
    }
    // ---- wave groups: groups 1 .. WK-1 hand their accumulators to group 0 through LDS (the tile buffers are free:
    // the main loop ends with a barrier), which adds them in group order and alone runs the rest of the kernel.
    const bool owner = wk == 0;
    if constexpr (WK > 1) {
        constexpr int NACC_W = TN * TM * ACC_REGS;
        static_assert((size_t)(WK - 1) * NACC_W * 256 * sizeof(float) <= sizeof(smem), "accumulator exchange must fit the tile buffers");
        float *red = reinterpret_cast<float *>(&smem[0]);
        if (!owner) {
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
#pragma unroll
                    for (int v = 0; v < ACC_REGS; ++v)
                        red[(((wk - 1) * NACC_W) + (i * TM + j) * ACC_REGS + v) * 256 + (tid & 255)] = acc[i][j][v];
        }
        __syncthreads();
        if (owner) {
            for (int g = 1; g < WK; ++g)
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int j = 0; j < TM; ++j)
#pragma unroll
                        for (int v = 0; v < ACC_REGS; ++v)
                            acc[i][j][v] += red[(((g - 1) * NACC_W) + (i * TM + j) * ACC_REGS + v) * 256 + tid];
        }
    }

    // ---- split-K: publish partial sums; the last workgroup of the tile reduces in split order ----
    if (a.split_k > 1) {
        constexpr int NACC = TN * TM * ACC_REGS;
        float *wsp = a.ws + ((int64_t)tile * a.split_k + z) * NACC * 256;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int v = 0; v < ACC_REGS; ++v)
                    if (owner)
                        __hip_atomic_store(&wsp[((i * TM + j) * ACC_REGS + v) * 256 + tid], acc[i][j][v], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
        // Hand-off without a device-wide fence (a release at agent scope writes the whole L2 of the XCD back, about 80 us
        // per launch when tried).  What orders it instead:
        //  * the partial sums are relaxed ATOMIC stores at agent scope, i.e. written through to memory that every XCD
        //    reads coherently; they are complete when the wave's vector-memory counter has drained, which the
        //    s_waitcnt below waits for.  Its "memory" clobber keeps the compiler from moving any access across it, and
        //    the workgroup barrier after it (a workgroup-scope fence for the compiler, an s_barrier for the hardware)
        //    makes thread 0 bump the counter only after every wave of the workgroup has drained;
        //  * the counter is bumped by an atomic read-modify-write at agent scope, performed at the memory side, so the
        //    arrivals of one tile are totally ordered and exactly one workgroup sees split_k - 1;
        //  * that workgroup reads the partial sums with relaxed ATOMIC loads at agent scope (served by coherent
        //    memory, never by a stale line of its own L1 or L2) after the second barrier; atomics are not moved across
        //    the barrier's fence by the compiler, and the loads depend on s_last through the branch below.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(&a.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (old == (unsigned)a.split_k - 1u);
        }
        __syncthreads();
        if (!s_last) return;                // the whole workgroup
        const float *wsr = a.ws + (int64_t)tile * a.split_k * NACC * 256;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int v = 0; v < ACC_REGS; ++v) acc[i][j][v] = 0.f;
        // Loads of RB splits are issued together (they are independent), then added in split order.
        constexpr int RB = (NACC <= 16) ? 4 : 1;
        for (int zz0 = 0; owner && zz0 < a.split_k; zz0 += RB) {
            float part[RB][NACC];
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                const float *p = wsr + (int64_t)min(zz0 + b, a.split_k - 1) * NACC * 256;
#pragma unroll
                for (int e = 0; e < NACC; ++e)
                    part[b][e] = __hip_atomic_load(&p[e * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                if (zz0 + b < a.split_k) {
#pragma unroll
                    for (int i = 0; i < TN; ++i)
#pragma unroll
                        for (int j = 0; j < TM; ++j)
#pragma unroll
                            for (int v = 0; v < ACC_REGS; ++v) acc[i][j][v] += part[b][(i * TM + j) * ACC_REGS + v];
                }
            }
        }
        if (tid == 0) __hip_atomic_store(&a.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- epilogue: bias, residual, activation, one rounding, NHWC store -------------------------
    T *y = (T *)a.y;
    const T *res = (const T *)a.res;
    // Coalesced form (channel counts and offsets multiples of 8): the accumulators plus bias go through LDS as an
    // fp32 [pixel][channel] tile, then every thread finishes 8 consecutive channels of one pixel: one 16-byte residual
    // load and one 16-byte store, a pixel's channels forming whole cache lines.  Same operations in the same order
    // as the direct form below, so the results are identical.
    const bool vec8_ok = (a.K % 8 == 0) && (a.y_ct % 8 == 0) && (a.y_coff % 8 == 0) && (a.res_ct % 8 == 0);
    if (vec8_ok) {
        constexpr int ELD = BN + 4;                       // row stride in floats: 4 lanes apart land 16 banks apart
        static_assert((size_t)BM * ELD * sizeof(float) <= sizeof(smem), "epilogue tile must fit the tile buffers");
        float *et = reinterpret_cast<float *>(&smem[0]);
        constexpr int CPR = BN / 8;                       // 8-channel chunks per pixel row of the tile
        // The residual chunks this thread will add are requested now, all of them, so that their trip to memory runs
        // under the accumulator exchange below.  (Inside the store loop every load would have to wait behind the store
        // of the chunk before it, which may alias it for all the compiler knows: one memory latency per chunk.)
        constexpr int EP_IT = (BM * CPR + NT - 1) / NT;
        u32x4 res_raw[EP_IT];
        const bool add_res = res != nullptr && !a.pool2;
        if (add_res) {
#pragma unroll
            for (int it = 0; it < EP_IT; ++it) {
                const int c = tid + it * NT;
                const int m = m0 + c / CPR, k = n0 + (c % CPR) * 8;
                const bool live = (c < BM * CPR) & (m < M) & (k < a.K);
                res_raw[it] = live ? *reinterpret_cast<const u32x4 *>(res + (int64_t)m * a.res_ct + k) : u32x4{0u, 0u, 0u, 0u};
            }
        }
        __syncthreads();                                  // the accumulator exchange above may still be read
        if (owner) {
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
#pragma unroll
                    for (int g = 0; g < GROUPS; ++g) {
                        const int ml = wm * SUBM + j * MF + frag_row;
                        const int kl = wn * SUBN + i * MF + ((MF == 32) ? (8 * g + 4 * (lane / 32)) : (4 * (lane / 16)));
                        float4 b;
                        if constexpr (BIAS_EARLY) b = bias_pre[i * GROUPS + g];
                        else b = *reinterpret_cast<const float4 *>(a.bias + n0 + kl);
                        float4 v;
                        v.x = acc[i][j][g * 4 + 0] + b.x;
                        v.y = acc[i][j][g * 4 + 1] + b.y;
                        v.z = acc[i][j][g * 4 + 2] + b.z;
                        v.w = acc[i][j][g * 4 + 3] + b.w;
                        *reinterpret_cast<float4 *>(&et[ml * ELD + kl]) = v;
                    }
        }
        __syncthreads();
        if (a.pool2) {
            // Four consecutive tile rows are one 2x2 window (see the pixel walk above) and the pooled pixel index is the
            // quad index.  Activation and rounding are monotonic, so the maximum is taken before them on fp32 values.
            for (int c = tid; c < (BM / 4) * CPR; c += NT) {
                const int r4 = c / CPR, col = (c % CPR) * 8;
                const int m = m0 + r4 * 4, k = n0 + col;
                if (m >= M || k >= a.K) continue;
                float v[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) v[t] = -INFINITY;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const float4 lo = *reinterpret_cast<const float4 *>(&et[(r4 * 4 + rr) * ELD + col]);
                    const float4 hi = *reinterpret_cast<const float4 *>(&et[(r4 * 4 + rr) * ELD + col + 4]);
                    v[0] = fmaxf(v[0], lo.x); v[1] = fmaxf(v[1], lo.y); v[2] = fmaxf(v[2], lo.z); v[3] = fmaxf(v[3], lo.w);
                    v[4] = fmaxf(v[4], hi.x); v[5] = fmaxf(v[5], hi.y); v[6] = fmaxf(v[6], hi.z); v[7] = fmaxf(v[7], hi.w);
                }
#pragma unroll
                for (int t = 0; t < 8; ++t) v[t] = apply_act(v[t], a.act);
                store_pack<T, 8>(y + (int64_t)(m >> 2) * a.y_ct + a.y_coff + k, v);
            }
            return;
        }
#pragma unroll
        for (int it = 0; it < EP_IT; ++it) {
            const int c = tid + it * NT;
            const int row = c / CPR, col = (c % CPR) * 8;
            const int m = m0 + row, k = n0 + col;
            if (c >= BM * CPR || m >= M || k >= a.K) continue;
            float v[8];
            const float4 lo = *reinterpret_cast<const float4 *>(&et[row * ELD + col]);
            const float4 hi = *reinterpret_cast<const float4 *>(&et[row * ELD + col + 4]);
            v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
            if (add_res) {
                const Pack<T, 8> rp = __builtin_bit_cast(Pack<T, 8>, res_raw[it]);
#pragma unroll
                for (int t = 0; t < 8; ++t) v[t] += to_f32(rp.e[t]);
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = apply_act(v[t], a.act);
            store_pack<T, 8>(y + (int64_t)m * a.y_ct + a.y_coff + k, v);
        }
        return;
    }
    if (!owner) return;
    const bool vec_ok = (a.y_ct % 4 == 0) && (a.y_coff % 4 == 0) && (a.res_ct % 4 == 0);
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m0 + wm * SUBM + j * MF + frag_row;
            if (m >= M) continue;
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const int k = n0 + wn * SUBN + i * MF + ((MF == 32) ? (8 * g + 4 * (lane / 32)) : (4 * (lane / 16)));
                if (k >= a.K) continue;
                float v[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) v[t] = acc[i][j][g * 4 + t];
                float4 b;
                if constexpr (BIAS_EARLY) b = bias_pre[i * GROUPS + g];
                else b = *reinterpret_cast<const float4 *>(a.bias + k);    // bias is padded to n_pad
                v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
                if (vec_ok && k + 4 <= a.K) {
                    if (res) {
                        float rv[4];
                        load_pack<T, 4>(res + (int64_t)m * a.res_ct + k, rv);
#pragma unroll
                        for (int t = 0; t < 4; ++t) v[t] += rv[t];
                    }
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[t] = apply_act(v[t], a.act);
                    store_pack<T, 4>(y + (int64_t)m * a.y_ct + a.y_coff + k, v);
                } else {
                    for (int t = 0; t < 4 && k + t < a.K; ++t) {
                        float f = v[t];
                        if (res) f += to_f32(res[(int64_t)m * a.res_ct + k + t]);
                        f = apply_act(f, a.act);
                        T o;
                        from_f32(f, o);
                        y[(int64_t)m * a.y_ct + a.y_coff + k + t] = o;
                    }
                }
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Matrix-vector form for 1x1 / fully connected layers with at most 8 output pixels (batch <= 8): the filter
// bank is streamed once with 16-byte loads, ROWS output channels per wavefront, the lanes stride along the
// reduction index and combine through a fixed butterfly of wavefront shuffles.  Bandwidth bound.
template <typename T>
__device__ __forceinline__ void unpack8(u32x4 v, float (&f)[8]) {
    const T *e = reinterpret_cast<const T *>(&v);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = to_f32(e[i]);
}

template <typename T, int MB, int ROWS, bool STREAM_W>
__device__ __forceinline__ void gemv_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int wave = (int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    const int lane = threadIdx.x & 63;
    const int k0 = wave * ROWS;
    if (k0 >= a.K) return;                           // whole wave
    const int J = a.gemm_k;                          // multiple of 8
    const T *x = (const T *)a.x;
    const uint16_t *wp = (const uint16_t *)a.w;
    float acc[ROWS][MB];
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int m = 0; m < MB; ++m) acc[r][m] = 0.f;
    float bias_k[ROWS];                              // fetched before the dot product, not after it (the bank is padded)
#pragma unroll
    for (int r = 0; r < ROWS; ++r) bias_k[r] = a.bias[k0 + r];
    constexpr int UNROLL = 4;
    for (int j0 = lane * 8; j0 < J; j0 += 64 * 8 * UNROLL) {
        u32x4 wv[UNROLL][ROWS], xv[UNROLL][MB];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int j = j0 + u * 64 * 8;
            const bool ok = j < J;
#pragma unroll
            for (int r = 0; r < ROWS; ++r)      // rows beyond K exist in the padded bank (zeros)
                // STREAM_W: a bank of 16 MB or more is read with non-temporal loads, so that it (VGG-16 FC1: 205 MB) does
                // not evict every other tenant's weights from the memory-side cache on its way through
                if (STREAM_W)
                    wv[u][r] = ok ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (int64_t)(k0 + r) * a.k_pad + j))
                                  : u32x4{0u, 0u, 0u, 0u};
                else
                    wv[u][r] = ok ? *reinterpret_cast<const u32x4 *>(wp + (int64_t)(k0 + r) * a.k_pad + j) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int m = 0; m < MB; ++m)
                xv[u][m] = (ok && m < a.N) ? *reinterpret_cast<const u32x4 *>(x + (int64_t)m * J + j) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float xf[MB][8];
#pragma unroll
            for (int m = 0; m < MB; ++m) unpack8<T>(xv[u][m], xf[m]);
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                float wf[8];
                unpack8<T>(wv[u][r], wf);
#pragma unroll
                for (int m = 0; m < MB; ++m)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][m] = fmaf(wf[e], xf[m][e], acc[r][m]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            float v = acc[r][m];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
            acc[r][m] = v;
        }
    if (lane == 0) {
        T *y = (T *)a.y;
        const T *res = (const T *)a.res;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int k = k0 + r;
            if (k >= a.K) continue;
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                if (m >= a.N) continue;
                float f = acc[r][m] + bias_k[r];
                if (res) f += to_f32(res[(int64_t)m * a.res_ct + k]);
                f = apply_act(f, a.act);
                T o;
                from_f32(f, o);
                y[(int64_t)m * a.y_ct + a.y_coff + k] = o;
            }
        }
    }
}
template <typename T, int MB, int ROWS, bool STREAM_W>
__global__ void __launch_bounds__(256) gemv_kernel(OpArgs a) {
    gemv_kernel_body<T, MB, ROWS, STREAM_W>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int MB, int ROWS, bool STREAM_W>
__global__ void __launch_bounds__(256) gemv_pair_kernel(OpArgsPair p) {
    gemv_kernel_body<T, MB, ROWS, STREAM_W>(p.a[blockIdx.y]);
}

// ---------------------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------------------
// 1x1 convolution on a small map (a few hundred pixels): latency bound, so no LDS tiles and no workgroup barrier in the
// reduction.  A wave owns 16 output channels x 16 pixels; filter rows and pixel rows are contiguous along the
// reduction index, so the 16x16x32 MFMA operands are 16-byte loads straight from memory, issued eight reduction steps
// at a time.  SLICES = 1: the four waves of a workgroup take four channel tiles of one pixel tile and each walks the
// whole reduction in ascending order into one accumulator (the arithmetic of the 64x16 tile kernel, bit for bit).
// SLICES = 4 (long reductions): the four waves split the reduction of one tile into four contiguous ranges and wave 0
// adds the partial sums in range order through LDS.
template <typename T, int SLICES>
__device__ __forceinline__ void pw_direct_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    typedef typename Mma<T, 16>::Acc Acc;
    constexpr int CH = 8;                                // reduction steps whose loads are in flight together
    __shared__ float red[SLICES > 1 ? (SLICES - 1) * 256 : 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int M = a.N * a.P * a.Q;
    const int tiles_m = (M + 15) / 16, tiles_n = (a.K + 15) / 16;
    const int tile = SLICES == 1 ? (int)blockIdx.x * 4 + wave : (int)blockIdx.x;
    if (tile >= tiles_m * tiles_n) return;               // SLICES = 1: a whole wave, and no barrier follows; SLICES = 4: the whole workgroup
    const int tn = tile % tiles_n, tm = tile / tiles_n;  // neighbouring waves share the pixel tile
    const int nsteps = a.k_pad / 32;
    const int per = (nsteps + SLICES - 1) / SLICES;
    const int s_begin = SLICES == 1 ? 0 : wave * per, s_end = SLICES == 1 ? nsteps : min(nsteps, s_begin + per);
    const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;

    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((int64_t)a.N * a.H * a.W * a.x_ct * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.w), 0, (int)((int64_t)a.n_pad * a.k_pad * 2), 0x00027000);

    // this lane's pixel row (operand B) and filter row (operand A)
    const int m = tm * 16 + frag_row;
    const uint32_t mm = m < M ? (uint32_t)m : 0u;
    const uint32_t t1 = __umulhi(a.divpq_m, mm);
    const int img = (int)((t1 + ((mm - t1) >> a.divpq_s1)) >> a.divpq_s2);
    const uint32_t rem = mm - (uint32_t)img * (uint32_t)(a.P * a.Q);
    const uint32_t t2 = __umulhi(a.divq_m, rem);
    const int pp = (int)((t2 + ((rem - t2) >> a.divq_s1)) >> a.divq_s2);
    const int qq = (int)(rem - (uint32_t)pp * (uint32_t)a.Q);
    const uint32_t xrow = (uint32_t)(((((img * a.H + pp * a.sh) * a.W) + qq * a.sw) * a.x_ct + a.x_coff + frag_k) * 2);
    const uint32_t wrow = (uint32_t)(((tn * 16 + frag_row) * a.k_pad + frag_k) * 2);
    const float4 bias4 = *reinterpret_cast<const float4 *>(a.bias + tn * 16 + 4 * (lane >> 4));       // padded to n_pad

    Acc acc;
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = 0.f;
    for (int s0 = s_begin; s0 < s_end; s0 += CH) {
        u32x4 wf[CH], xf[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int s = s0 + i;
            const bool live = s < s_end;
            wf[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, live ? wrow + (uint32_t)(s * 64) : OOB_OFFSET, 0, 0);
            const bool xv = live & (m < M) & (s * 32 + frag_k < a.C);
            xf[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, xv ? xrow + (uint32_t)(s * 64) : OOB_OFFSET, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (s0 + i < s_end) acc = Mma<T, 16>::run(wf[i], xf[i], acc);
    }
    if constexpr (SLICES > 1) {
        if (wave > 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((wave - 1) * 4 + v) * 64 + lane] = acc[v];
        }
        __syncthreads();
        if (wave > 0) return;
        for (int w = 1; w < SLICES; ++w)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] += red[((w - 1) * 4 + v) * 64 + lane];
    }

    // epilogue: bias, residual, activation, one rounding
    T *y = (T *)a.y;
    const T *res = (const T *)a.res;
    const int k = tn * 16 + 4 * (lane >> 4);
    if (m >= M || k >= a.K) return;
    float v[4] = {acc[0] + bias4.x, acc[1] + bias4.y, acc[2] + bias4.z, acc[3] + bias4.w};
    const bool vec_ok = (a.y_ct % 4 == 0) && (a.y_coff % 4 == 0) && (a.res_ct % 4 == 0);
    if (vec_ok && k + 4 <= a.K) {
        if (res) {
            float rv[4];
            load_pack<T, 4>(res + (int64_t)m * a.res_ct + k, rv);
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] += rv[t];
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = apply_act(v[t], a.act);
        store_pack<T, 4>(y + (int64_t)m * a.y_ct + a.y_coff + k, v);
    } else {
        for (int t = 0; t < 4 && k + t < a.K; ++t) {
            float f = v[t];
            if (res) f += to_f32(res[(int64_t)m * a.res_ct + k + t]);
            f = apply_act(f, a.act);
            T o;
            from_f32(f, o);
            y[(int64_t)m * a.y_ct + a.y_coff + k + t] = o;
        }
    }
}
template <typename T, int SLICES>
__global__ void __launch_bounds__(256) pw_direct_kernel(OpArgs a) {
    pw_direct_kernel_body<T, SLICES>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int SLICES>
__global__ void __launch_bounds__(256) pw_direct_pair_kernel(OpArgsPair p) {
    pw_direct_kernel_body<T, SLICES>(p.a[blockIdx.y]);
}

template <typename T, int BN, int BM, int WN, int WM, int MF, int STAGES, int AMODE, int WK = 1>
__global__ void __launch_bounds__(256 * WK) igemm_kernel(OpArgs a) {
    igemm_body<T, BN, BM, WN, WM, MF, STAGES, AMODE, WK>(a);
}
// Co-issue: the same tile program for two operators of equal launch shape, one per value of blockIdx.y.
template <typename T, int BN, int BM, int WN, int WM, int MF, int STAGES, int AMODE, int WK = 1>
__global__ void __launch_bounds__(256 * WK) igemm_pair_kernel(OpArgsPair p) {
    igemm_body<T, BN, BM, WN, WM, MF, STAGES, AMODE, WK>(p.a[blockIdx.y]);
}

template <typename T, int BN, int BM, int WN, int WM, int MF, int STAGES, int WK = 1>
static void launch_cfg(const OpArgs &a, hipStream_t st, const OpArgs *mate, int n_mates) {
    const dim3 grid(a.grid_x, mate ? 1 + n_mates : 1);
    OpArgsPair p;
    if (mate) {
        p.a[0] = a;
        for (int i = 0; i < n_mates; ++i) p.a[1 + i] = mate[i];
    }
    if (a.vec_a == A_UNIFORM) {
        if (mate) hipLaunchKernelGGL((igemm_pair_kernel<T, BN, BM, WN, WM, MF, STAGES, A_UNIFORM, WK>), grid, dim3(256 * WK), 0, st, p);
        else hipLaunchKernelGGL((igemm_kernel<T, BN, BM, WN, WM, MF, STAGES, A_UNIFORM, WK>), grid, dim3(256 * WK), 0, st, a);
    } else if (a.vec_a == A_VEC8) {
        if (mate) hipLaunchKernelGGL((igemm_pair_kernel<T, BN, BM, WN, WM, MF, STAGES, A_VEC8, WK>), grid, dim3(256 * WK), 0, st, p);
        else hipLaunchKernelGGL((igemm_kernel<T, BN, BM, WN, WM, MF, STAGES, A_VEC8, WK>), grid, dim3(256 * WK), 0, st, a);
    } else {
        hipLaunchKernelGGL((igemm_kernel<T, BN, BM, WN, WM, MF, 2, A_SCALAR>), grid, dim3(256), 0, st, a);
    }
}

template <typename T>
static int launch_igemm_typed(const OpArgs &a, hipStream_t st, const OpArgs *mate, int n_mates) {
    switch (a.kernel_id) {
        case K_IGEMM_128x128: launch_cfg<T, 128, 128, 2, 2, 32, 2>(a, st, mate, n_mates); break;
        case K_IGEMM_128x64:
            if (a.wk == 2) launch_cfg<T, 128, 64, 2, 2, 32, 2, 2>(a, st, mate, n_mates);
            else launch_cfg<T, 128, 64, 2, 2, 32, 2>(a, st, mate, n_mates);
            break;
        case K_IGEMM_64x64:
            if (a.wk == 2) launch_cfg<T, 64, 64, 2, 2, 32, 4, 2>(a, st, mate, n_mates);
            else launch_cfg<T, 64, 64, 2, 2, 32, 4, 1>(a, st, mate, n_mates);
            break;
        case K_IGEMM_64x16: launch_cfg<T, 64, 16, 4, 1, 16, 4>(a, st, mate, n_mates); break;
        case K_IGEMM_PW: {
            const dim3 grid(a.grid_x), block(256);
            if (a.split_k > 1) MT_LAUNCH((pw_direct_kernel<T, 4>), (pw_direct_pair_kernel<T, 4>), grid, block, st, a, mate);
            else MT_LAUNCH((pw_direct_kernel<T, 1>), (pw_direct_pair_kernel<T, 1>), grid, block, st, a, mate);
            break;
        }
        case K_GEMV: {
            const dim3 grid(a.grid_x), block(256);
            const bool stream_w = (int64_t)a.n_pad * a.k_pad * 2 >= (16ll << 20);
            auto go = [&]<int MB>() {
                if (stream_w) MT_LAUNCH((gemv_kernel<T, MB, 2, true>), (gemv_pair_kernel<T, MB, 2, true>), grid, block, st, a, mate);
                else MT_LAUNCH((gemv_kernel<T, MB, 2, false>), (gemv_pair_kernel<T, MB, 2, false>), grid, block, st, a, mate);
            };
            if (a.N <= 1) go.template operator()<1>();
            else if (a.N <= 2) go.template operator()<2>();
            else if (a.N <= 4) go.template operator()<4>();
            else go.template operator()<8>();
            break;
        }
        default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Depthwise 3x3 convolution fused into the 1x1 convolution that consumes it (the second half of an inverted
// residual block), for the case where the 1x1 layer runs on the 64x16 tile without a split: one launch instead of
// two on a latency-bound chain.  The im2col tile of the 1x1 layer is not read from memory but computed: for its
// (pixel, 8 channels) chunk a thread loads the nine taps, multiplies them with the depthwise filters (kept in LDS),
// adds bias, applies the activation and rounds to the storage type, exactly the operation sequence of the stand-alone
// depthwise kernel, and writes the chunk to the LDS tile (and, from the first channel tile, to the intermediate
// tensor, which stays valid).  The MFMA sequence, tile and reduction order are those of the 64x16 implicit-GEMM
// instantiation, so the output bits equal those of the two separate launches.
template <typename T>
__global__ void __launch_bounds__(256) dwpw_kernel(OpArgs a, OpArgs d) {
    set_wave_priority(a.prio);
    constexpr int BN = 64, BM = 16;
    constexpr int G = 3;                                 // channel chunks of a thread whose tap loads are in flight together
    typedef typename Mma<T, 16>::Acc Acc;
    __shared__ __attribute__((aligned(16))) uint16_t Ws[2][BN * LDK];
    // depthwise filters [9][k_pad] of T, bias [k_pad] floats, depthwise output of the 16 pixels [16][k_pad + 8] of T
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    const int M = a.N * a.P * a.Q;
    const int tiles_n = a.n_pad / BN;
    const int tn = blockIdx.x % tiles_n, tm = blockIdx.x / tiles_n;
    const int n0 = tn * BN, m0 = tm * BM;
    const int nk = a.k_pad / BK;
    const int C = d.C;                                   // channels of the depthwise layer = reduction length of the 1x1 layer
    const int CP8 = a.k_pad / 8;                         // 8-channel chunks per padded row
    const int XLD = a.k_pad + 8;                         // row stride of the depthwise output tile (16-byte reads fall in distinct banks)
    u32x4 *dww = reinterpret_cast<u32x4 *>(dyn);
    float *dwb = reinterpret_cast<float *>(dyn + (size_t)9 * a.k_pad * 2);
    uint16_t *Xf = reinterpret_cast<uint16_t *>(dyn + (size_t)9 * a.k_pad * 2 + (size_t)a.k_pad * 4);

    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.w), 0, (int)((int64_t)a.n_pad * a.k_pad * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(d.x), 0, (int)((int64_t)d.N * d.H * d.W * C * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_dw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(d.w), 0, (int)((int64_t)9 * C * 2), 0x00027000);

    // filter tile of the 1x1 layer: 512 chunks, two per thread; tile 0 is requested before anything else
    uint32_t wvoff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + i * 256;
        wvoff[i] = (uint32_t)(((n0 + c / 8) * a.k_pad + (c % 8) * 8) * 2);
    }
    u32x4 wr[2][2];
    auto load_w = [&](int t, u32x4 (&r)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i) r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, wvoff[i], (uint32_t)(t * BK * 2), 0);
    };
    auto store_w = [&](int buf, const u32x4 (&r)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = tid + i * 256;
            *reinterpret_cast<u32x4 *>(&Ws[buf][(c / 8) * LDK + (c % 8) * 8]) = r[i];
        }
    };
    load_w(0, wr[0]);
    if (1 < nk) load_w(1, wr[1]);

    // depthwise filters and bias of every channel into LDS (zeros beyond C)
    for (int i = tid; i < 9 * CP8; i += 256) {
        const int tap = i / CP8, c8 = i - tap * CP8;
        const uint32_t off = c8 * 8 < C ? (uint32_t)((tap * C + c8 * 8) * 2) : OOB_OFFSET;
        dww[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_dw, off, 0, 0);
    }
    for (int i = tid; i < a.k_pad; i += 256) dwb[i] = i < C ? d.bias[i] : 0.f;

    // ---- phase 1: the depthwise output of this tile's 16 pixels, every channel, into LDS -----------------------
    // 16 threads per pixel; a thread walks the 8-channel chunks (tid % 16) + 16 j of its pixel.
    const int px = tid >> 4, cl = tid & 15;
    const int m = m0 + px;
    const bool row_ok = m < M;
    const uint32_t mm = row_ok ? (uint32_t)m : 0u;
    const uint32_t t1 = __umulhi(a.divpq_m, mm);
    const int img = (int)((t1 + ((mm - t1) >> a.divpq_s1)) >> a.divpq_s2);
    const uint32_t rem = mm - (uint32_t)img * (uint32_t)(a.P * a.Q);
    const uint32_t t2 = __umulhi(a.divq_m, rem);
    const int pp = (int)((t2 + ((rem - t2) >> a.divq_s1)) >> a.divq_s2);
    const int qq = (int)(rem - (uint32_t)pp * (uint32_t)a.Q);
    const int ih0 = pp * d.sh - d.ph, iw0 = qq * d.sw - d.pw;
    bool tap_ok[9];
    uint32_t tapoff[9];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) {
            const int ih = ih0 + r, iw = iw0 + sx;
            tap_ok[r * 3 + sx] = row_ok & ((uint32_t)ih < (uint32_t)d.H) & ((uint32_t)iw < (uint32_t)d.W);
            tapoff[r * 3 + sx] = (uint32_t)((((img * d.H + ih) * d.W + iw) * C) * 2);
        }
    __syncthreads();                                     // depthwise filters and bias are in LDS
    for (int c8b = cl; c8b < CP8; c8b += 16 * G) {
        u32x4 xt[G][9];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int c0 = (c8b + 16 * g) * 8;
            const bool ch_ok = c0 < C;
#pragma unroll
            for (int k = 0; k < 9; ++k) {
                const uint32_t off = (tap_ok[k] & ch_ok) ? tapoff[k] + (uint32_t)(c0 * 2) : OOB_OFFSET;
                xt[g][k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0);
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int c8 = c8b + 16 * g;
            if (c8 >= CP8) continue;
            const int c0 = c8 * 8;
            const bool ch_ok = row_ok && c0 < C;
            float acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
            for (int k = 0; k < 9; ++k) {
                const Pack<T, 8> xv = __builtin_bit_cast(Pack<T, 8>, xt[g][k]);
                const Pack<T, 8> wv = __builtin_bit_cast(Pack<T, 8>, dww[k * CP8 + c8]);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = tap_ok[k] ? fmaf(to_f32(xv.e[i]), to_f32(wv.e[i]), acc[i]) : acc[i];
            }
            Pack<T, 8> o;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float v = apply_act(acc[i] + dwb[c0 + i], d.act);
                from_f32(ch_ok ? v : 0.f, o.e[i]);
            }
            *reinterpret_cast<Pack<T, 8> *>(&Xf[px * XLD + c0]) = o;
            if (tn == 0 && ch_ok) *reinterpret_cast<Pack<T, 8> *>((T *)d.y + (int64_t)m * d.y_ct + d.y_coff + c0) = o;
        }
    }

    // ---- phase 2: the 1x1 layer, im2col rows read from the LDS tile above --------------------------------------
    Acc acc;
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = 0.f;
    const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;
    const float4 bias4 = *reinterpret_cast<const float4 *>(a.bias + n0 + wn * 16 + 4 * (lane >> 4));   // padded to n_pad
    auto step = [&](int t, u32x4 (&r)[2]) {
        const int buf = t & 1;
        store_w(buf, r);
        if (t + 2 < nk) load_w(t + 2, r);
        __syncthreads();                   // filter tile t (and, at t = 0, the depthwise tile) complete; tile t - 1 was consumed
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int koff = kk * 32 + frag_k;
            const u32x4 fa = *reinterpret_cast<const u32x4 *>(&Ws[buf][(wn * 16 + frag_row) * LDK + koff]);
            const u32x4 fb = *reinterpret_cast<const u32x4 *>(&Xf[frag_row * XLD + t * BK + koff]);
            acc = Mma<T, 16>::run(fa, fb, acc);
        }
    };
    for (int t = 0; t < nk; t += 2) {
        step(t, wr[0]);
        if (t + 1 < nk) step(t + 1, wr[1]);
    }

    // epilogue of the 1x1 layer: bias, residual, activation, one rounding
    T *y = (T *)a.y;
    const T *res = (const T *)a.res;
    const int mo = m0 + frag_row, k = n0 + wn * 16 + 4 * (lane >> 4);
    if (mo >= M || k >= a.K) return;
    float v[4] = {acc[0] + bias4.x, acc[1] + bias4.y, acc[2] + bias4.z, acc[3] + bias4.w};
    const bool vec_ok = (a.y_ct % 4 == 0) && (a.y_coff % 4 == 0) && (a.res_ct % 4 == 0);
    if (vec_ok && k + 4 <= a.K) {
        if (res) {
            float rv[4];
            load_pack<T, 4>(res + (int64_t)mo * a.res_ct + k, rv);
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] += rv[t];
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = apply_act(v[t], a.act);
        store_pack<T, 4>(y + (int64_t)mo * a.y_ct + a.y_coff + k, v);
    } else {
        for (int t = 0; t < 4 && k + t < a.K; ++t) {
            float f = v[t];
            if (res) f += to_f32(res[(int64_t)mo * a.res_ct + k + t]);
            f = apply_act(f, a.act);
            T o;
            from_f32(f, o);
            y[(int64_t)mo * a.y_ct + a.y_coff + k + t] = o;
        }
    }
}

static size_t dwpw_lds_bytes(int k_pad) { return (size_t)k_pad * (18 + 4) + (size_t)16 * (k_pad + 8) * 2; }

// Host check of what the fused kernel assumes; the runtime pairs two operators only when this holds.
bool dwpw_fusable(const OpArgs &dw, const OpArgs &pw) {
    // the 1x1 layer must be one whose stand-alone kernel walks the reduction in one ascending pass, as the fused kernel does
    if (dw.kernel_id != K_DWCONV || !(pw.kernel_id == K_IGEMM_64x16 || pw.kernel_id == K_IGEMM_PW)) return false;
    if (dw.dtype != pw.dtype || (dw.dtype != MT_F16 && dw.dtype != MT_BF16)) return false;
    if (dw.R != 3 || dw.S != 3 || dw.vec != 8 || dw.C % 8 != 0 || dw.y_coff != 0 || dw.y_ct != dw.C) return false;
    if (pw.R != 1 || pw.S != 1 || pw.sh != 1 || pw.sw != 1 || pw.ph != 0 || pw.pw != 0 || pw.groups > 1) return false;
    if (pw.split_k != 1 || pw.vec_a == 0 || pw.C != dw.C || pw.x_ct != dw.C || pw.x_coff != 0) return false;
    if (pw.N != dw.N || pw.H != dw.P || pw.W != dw.Q || pw.P != dw.P || pw.Q != dw.Q) return false;
    if (dwpw_lds_bytes(pw.k_pad) > 44 * 1024) return false;          // filters, bias and the depthwise tile must fit beside the filter tiles in 64 KB of LDS
    return true;
}

int launch_dwpw(const OpArgs &dw, const OpArgs &pw, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (!dwpw_fusable(dw, pw)) return (int)hipErrorInvalidValue;
    const int M = pw.N * pw.P * pw.Q;
    const dim3 grid(((M + 15) / 16) * (pw.n_pad / 64)), block(256);
    const size_t dyn = dwpw_lds_bytes(pw.k_pad);
    if (pw.dtype == MT_F16) hipLaunchKernelGGL(dwpw_kernel<f16>, grid, block, dyn, st, pw, dw);
    else hipLaunchKernelGGL(dwpw_kernel<bf16>, grid, block, dyn, st, pw, dw);
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// 1x1 convolution fused with the depthwise 3x3 convolution that consumes it (the first two operators of an inverted
// residual block): one launch instead of two on a latency-bound chain.  A workgroup owns HC channels of the widened
// tensor and a band of output rows of one image.  It computes the widened tensor on the input rows the band needs
// (one row of overlap on each side) with the MFMA sequence of the 64x16 implicit-GEMM instantiation (operands straight
// from memory into registers: filter rows and pixel rows are contiguous along the reduction index), rounds it to the
// storage type into LDS (and, for the rows the band owns, to the intermediate tensor, which stays valid), and then
// runs the depthwise filter over the LDS copy with the operation sequence of the stand-alone depthwise kernel.  Both
// halves therefore produce the bits of the two separate launches.
// MT: 16-pixel tiles per wave (a band reads at most 64 * MT pixels), KS: 32-deep reduction steps (k_pad <= 32 * KS).
template <typename T, int MT, int KS, int HC>
__global__ void __launch_bounds__(256) pwdw_kernel(OpArgs e, OpArgs d, int bands) {
    set_wave_priority(d.prio);
    constexpr int NI = HC / 16;                          // MFMA tiles along the channels
    constexpr int CPP = HC / 8;                          // 8-channel chunks per pixel
    constexpr int ELD = HC + 8;                          // LDS row stride
    typedef typename Mma<T, 16>::Acc Acc;
    __shared__ __attribute__((aligned(16))) uint16_t Es[MT * 64 * ELD];
    __shared__ __attribute__((aligned(16))) uint16_t Wd[9 * HC];
    __shared__ float Bd[HC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunks = (e.K + HC - 1) / HC;
    const int c0 = (blockIdx.x % chunks) * HC;
    const int band = (blockIdx.x / chunks) % bands;
    const int img = blockIdx.x / (chunks * bands);
    const int W = d.W, Min = d.H * d.W;                  // the widened map has the pixels of the input map (1x1, stride 1)
    const int PB = (d.P + bands - 1) / bands;
    const int p_lo = band * PB, p_hi = min(d.P, p_lo + PB);               // output rows of this band
    const int r_lo = max(0, p_lo * d.sh - 1), r_hi = min(d.H - 1, (p_hi - 1) * d.sh + 1);   // widened rows it reads
    const int px0 = r_lo * W, Mb = (r_hi - r_lo + 1) * W;
    const int own_lo = p_lo * d.sh, own_hi = band == bands - 1 ? d.H : min(d.H, p_hi * d.sh);   // widened rows it stores
    const int nsteps = e.k_pad / 32;
    const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;

    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(e.x), 0, (int)((int64_t)e.N * Min * e.C * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(e.w), 0, (int)((int64_t)e.n_pad * e.k_pad * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_dw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(d.w), 0, (int)((int64_t)9 * d.C * 2), 0x00027000);

    u32x4 wf[NI][KS], xf[MT][KS];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint32_t off = s < nsteps ? (uint32_t)(((c0 + i * 16 + frag_row) * e.k_pad + s * 32 + frag_k) * 2) : OOB_OFFSET;
            wf[i][s] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, off, 0, 0);
        }
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        const int px = (wave + 4 * j) * 16 + frag_row;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int k = s * 32 + frag_k;
            const bool v = (px < Mb) & (k < e.C);
            const uint32_t off = v ? (uint32_t)((((img * Min + px0 + px) * e.C) + k) * 2) : OOB_OFFSET;
            xf[j][s] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, off, 0, 0);
        }
    }
    float4 bias4[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) bias4[i] = *reinterpret_cast<const float4 *>(e.bias + c0 + i * 16 + 4 * (lane >> 4));   // padded to n_pad
    // depthwise filters [9][HC] and bias of this workgroup's channels (zeros beyond the last channel)
    if (tid < 9 * CPP) {
        const int tap = tid / CPP, c8 = tid - tap * CPP;
        const int c = c0 + c8 * 8;
        const uint32_t off = c < d.C ? (uint32_t)((tap * d.C + c) * 2) : OOB_OFFSET;
        *reinterpret_cast<u32x4 *>(&Wd[tap * HC + c8 * 8]) = __builtin_amdgcn_raw_buffer_load_b128(rsrc_dw, off, 0, 0);
    }
    if (tid < HC) Bd[tid] = c0 + tid < d.C ? d.bias[c0 + tid] : 0.f;

    // ---- the 1x1 layer: reduction steps in ascending order into one accumulator per tile ---------------------
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        if ((wave + 4 * j) * 16 >= Mb) continue;         // wave-uniform
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            Acc acc;
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                if (s < nsteps) acc = Mma<T, 16>::run(wf[i][s], xf[j][s], acc);
            float v[4] = {acc[0] + bias4[i].x, acc[1] + bias4[i].y, acc[2] + bias4[i].z, acc[3] + bias4[i].w};
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = apply_act(v[t], e.act);
            Pack<T, 4> o;
#pragma unroll
            for (int t = 0; t < 4; ++t) from_f32(v[t], o.e[t]);
            *reinterpret_cast<Pack<T, 4> *>(&Es[((wave + 4 * j) * 16 + frag_row) * ELD + i * 16 + 4 * (lane >> 4)]) = o;
        }
    }
    __syncthreads();

    // ---- the rows of the widened tensor this band owns, to memory, 16 bytes per thread ------------------------
    T *ey = (T *)e.y;
    for (int it = (own_lo - r_lo) * W * CPP + tid; it < (own_hi - r_lo) * W * CPP; it += 256) {
        const int px = it / CPP, c8 = it - px * CPP;
        const int c = c0 + c8 * 8;
        if (c < e.K)
            *reinterpret_cast<u32x4 *>(ey + (int64_t)(img * Min + px0 + px) * e.y_ct + e.y_coff + c) = *reinterpret_cast<const u32x4 *>(&Es[px * ELD + c8 * 8]);
    }
    // ---- the depthwise layer over the LDS copy ---------------------------------------------------------------
    T *dy = (T *)d.y;
    const int Mout = d.P * d.Q;
    for (int it = tid; it < (p_hi - p_lo) * d.Q * CPP; it += 256) {
        const int ol = it / CPP, c8 = it - ol * CPP;
        const int c = c0 + c8 * 8;
        const int pl = ol / d.Q;
        const int p = p_lo + pl, q = ol - pl * d.Q;
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) {
                const int ih = p * d.sh - 1 + r, iw = q * d.sw - 1 + sx;
                const bool ok = ((uint32_t)ih < (uint32_t)d.H) & ((uint32_t)iw < (uint32_t)W);
                const int ihc = min(max(ih, r_lo), r_hi), iwc = min(max(iw, 0), W - 1);
                const Pack<T, 8> xv = *reinterpret_cast<const Pack<T, 8> *>(&Es[((ihc - r_lo) * W + iwc) * ELD + c8 * 8]);
                const Pack<T, 8> wv = *reinterpret_cast<const Pack<T, 8> *>(&Wd[(r * 3 + sx) * HC + c8 * 8]);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = ok ? fmaf(to_f32(xv.e[i]), to_f32(wv.e[i]), acc[i]) : acc[i];
            }
        if (c < d.C) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = apply_act(acc[i] + Bd[c8 * 8 + i], d.act);
            store_pack<T, 8>(dy + (int64_t)(img * Mout + p * d.Q + q) * d.y_ct + d.y_coff + c, acc);
        }
    }
}

// Launch shape of the fused pair: the kernel variant (pixels a band may read, by reduction depth) and the number of
// row bands, chosen so that enough workgroups exist and a band's input rows fit the variant.  False: not fusable.
static bool pwdw_plan(const OpArgs &pw, const OpArgs &dw, int *variant, int *bands) {
    // the 1x1 layer must be one whose stand-alone kernel walks the reduction in one ascending pass, as the fused kernel does
    if (!(pw.kernel_id == K_IGEMM_64x16 || pw.kernel_id == K_IGEMM_PW) || dw.kernel_id != K_DWCONV) return false;
    if (dw.dtype != pw.dtype || (dw.dtype != MT_F16 && dw.dtype != MT_BF16)) return false;
    if (pw.R != 1 || pw.S != 1 || pw.sh != 1 || pw.sw != 1 || pw.ph != 0 || pw.pw != 0 || pw.groups > 1) return false;
    if (pw.split_k != 1 || pw.vec_a == 0 || pw.C % 8 != 0 || pw.x_ct != pw.C || pw.x_coff != 0 || pw.res_ct != 0) return false;
    if (pw.K % 8 != 0 || pw.y_coff != 0 || pw.y_ct != pw.K) return false;
    if (dw.R != 3 || dw.S != 3 || dw.ph != 1 || dw.pw != 1 || dw.sh < 1 || dw.sh > 2 || dw.vec != 8 || dw.C != pw.K) return false;
    if (dw.N != pw.N || dw.H != pw.P || dw.W != pw.Q) return false;
    const int steps = pw.k_pad / 32;
    const int limit = steps <= 2 ? 512 : steps <= 4 ? 256 : steps <= 8 ? 64 : 0;     // pixels a band may read
    *variant = steps <= 2 ? 0 : steps <= 4 ? 1 : 2;
    if (limit == 0 || 3 * dw.W > limit) return false;
    const int chunks = (pw.K + PWDW_HC - 1) / PWDW_HC;
    const int by_count = (PWDW_WGS + pw.N * chunks - 1) / (pw.N * chunks);
    const int by_work = (dw.P * dw.Q * (PWDW_HC / 8) + PWDW_ITEMS - 1) / PWDW_ITEMS;
    int b = std::max(1, std::min(dw.P, std::max(by_count, by_work)));
    for (;; ++b) {
        const int PB = (dw.P + b - 1) / b;
        if (std::min(dw.H, (PB - 1) * dw.sh + 3) * dw.W <= limit) {        // b <= P here: one output row per band always fits
            *bands = (dw.P + PB - 1) / PB;                                  // no empty band
            return true;
        }
    }
}

bool pwdw_fusable(const OpArgs &pw, const OpArgs &dw) {
    int variant = 0, bands = 0;
    return pwdw_plan(pw, dw, &variant, &bands);
}

int launch_pwdw(const OpArgs &pw, const OpArgs &dw, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    int variant = 0, bands = 0;
    if (!pwdw_plan(pw, dw, &variant, &bands)) return (int)hipErrorInvalidValue;
    constexpr int HC = PWDW_HC;
    const dim3 grid(pw.N * bands * ((pw.K + HC - 1) / HC)), block(256);
    auto go = [&]<typename T>() {
        if (variant == 0) hipLaunchKernelGGL((pwdw_kernel<T, 8, 2, HC>), grid, block, 0, st, pw, dw, bands);
        else if (variant == 1) hipLaunchKernelGGL((pwdw_kernel<T, 4, 4, HC>), grid, block, 0, st, pw, dw, bands);
        else hipLaunchKernelGGL((pwdw_kernel<T, 1, 8, HC>), grid, block, 0, st, pw, dw, bands);
    };
    if (pw.dtype == MT_F16) go.template operator()<f16>();
    else go.template operator()<bf16>();
    return (int)hipGetLastError();
}

// ---- what the chip sustains (diagnostics) -----------------------------------------------------------------------
// A loop of 32x32x16 matrix instructions on registers alone: four independent accumulators per wave, so that the
// issue of one never waits for the result of the one before.  Operands are small non-trivial values (all-zero inputs
// would draw less power than real work and let the clock run higher); every lane folds its accumulators into one
// word at the end, which keeps the loop alive.
template <typename T>
__global__ void __launch_bounds__(256) peak_mfma_kernel(float *sink, int iters) {
    const uint32_t lane = threadIdx.x;
    u32x4 a, b;
    const uint32_t expo = std::is_same<T, f16>::value ? 0x2000u : 0x3c00u;    // 2^-7 in either format, mantissa below
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t h0 = ((lane * 2654435761u + i * 40503u) >> 20) & 0x7fu, h1 = ((lane * 2246822519u + i * 9973u) >> 21) & 0x7fu;
        a[i] = (expo | h0) | ((expo | h1) << 16);
        b[i] = (expo | h1) | ((expo | h0) << 16);
    }
    typename Mma<T, 32>::Acc acc0 = {}, acc1 = {}, acc2 = {}, acc3 = {};
    for (int it = 0; it < iters; ++it) {
        acc0 = Mma<T, 32>::run(a, b, acc0);
        acc1 = Mma<T, 32>::run(b, a, acc1);
        acc2 = Mma<T, 32>::run(a, a, acc2);
        acc3 = Mma<T, 32>::run(b, b, acc3);
    }
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) v += acc0[i] + acc1[i] + acc2[i] + acc3[i];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = v;
}

// mode 0: dst[i] = src[i] in 16-byte pieces, grid-stride, eight pieces in flight per thread; mode 1: reads only and
// folds what it read into one word per thread (written to dst, which then needs gridDim.x * 256 words).
template <int MODE>
__global__ void __launch_bounds__(256) peak_stream_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n16) {
    constexpr int U = 8;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4 s = {0u, 0u, 0u, 0u};
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (MODE == 0) __builtin_nontemporal_store(v[u], dst + i + u * stride);
            else s ^= v[u];
        }
    }
    for (; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        if (MODE == 0) __builtin_nontemporal_store(v, dst + i);
        else s ^= v;
    }
    if (MODE == 1) ((uint32_t *)dst)[(size_t)blockIdx.x * 256 + threadIdx.x] = s[0] ^ s[1] ^ s[2] ^ s[3];
}

int launch_peak_mfma(int dtype, float *sink, int n_groups, int iters, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MT_F16) hipLaunchKernelGGL(peak_mfma_kernel<f16>, dim3((unsigned)n_groups), dim3(256), 0, st, sink, iters);
    else if (dtype == MT_BF16) hipLaunchKernelGGL(peak_mfma_kernel<bf16>, dim3((unsigned)n_groups), dim3(256), 0, st, sink, iters);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

int launch_peak_stream(int mode, const void *src, void *dst, size_t bytes, int n_groups, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (bytes % 16 != 0 || n_groups < 1) return (int)hipErrorInvalidValue;
    if (mode == 0) hipLaunchKernelGGL(peak_stream_kernel<0>, dim3((unsigned)n_groups), dim3(256), 0, st, (const u32x4 *)src, (u32x4 *)dst, bytes / 16);
    else hipLaunchKernelGGL(peak_stream_kernel<1>, dim3((unsigned)n_groups), dim3(256), 0, st, (const u32x4 *)src, (u32x4 *)dst, bytes / 16);
    return (int)hipGetLastError();
}

// ---- fixed scratch for callers that cannot allocate ---------------------------------------------------------------
// Split-K workspaces and arrival counters of mt_run_static_scratch live here.  In host code the array's name is only a
// handle for the symbol lookup below: every use of the memory (kernel arguments, fills) goes through the address that
// hipGetSymbolAddress returned for the device in question, because each GPU holds its own copy at its own address.
static __device__ __align__(256) unsigned char scratch[MT_STATIC_SCRATCH_BYTES];

int static_scratch_address(int device, void **ptr) {
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void *addr[MAX_DEV] = {};
    if (!ptr || device < 0 || device >= MAX_DEV) return (int)hipErrorInvalidValue;
    std::lock_guard<std::mutex> lk(mu);
    if (!addr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return (int)e;
        if (cur != device) return (int)hipErrorInvalidDevice;      // the lookup answers for the current device
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        addr[device] = p;
    }
    *ptr = addr[device];
    return 0;
}

int launch_igemm(const OpArgs &a, void *stream, const OpArgs *mate, int n_mates) {
    if (mate && (n_mates < 1 || n_mates >= COISSUE_MAX)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (mate && !coissue_supported(a)) return (int)hipErrorInvalidValue;
    if (a.dtype == MT_F16) return launch_igemm_typed<f16>(a, st, mate, n_mates);
    if (a.dtype == MT_BF16) return launch_igemm_typed<bf16>(a, st, mate, n_mates);
    return (int)hipErrorInvalidValue;
}

// Kernels that exist in a two-operator form: every kernel of the 16-bit storage types that works on 16-byte vectors
// (the tile kernels with 16-byte or tap-uniform gathers, the small-map 1x1 kernel, the weight-streaming kernel, the
// patch-staged, resident-filter and first-layer kernels, depthwise, pooling, normalisation and add).  Not: fp32 storage,
// grouped convolutions (several launches per operator), element-wise gathers and scalar channel counts.
bool coissue_supported(const OpArgs &a) {
    if (a.dtype != MT_F16 && a.dtype != MT_BF16) return false;
    if (a.groups > 1) return false;
    switch (a.kernel_id) {
        case K_IGEMM_128x128: case K_IGEMM_128x64: case K_IGEMM_64x64: case K_IGEMM_64x16:
            return a.vec_a == A_UNIFORM || a.vec_a == A_VEC8;
        case K_IGEMM_PW: case K_GEMV: case K_PCONV: case K_ROWB: case K_STEM: return true;
        case K_DWCONV: case K_MAXPOOL: case K_AVGPOOL: case K_GAP: case K_LRN: case K_ADD: return a.vec == 8;
        default: return false;
    }
}

}  // namespace mt
