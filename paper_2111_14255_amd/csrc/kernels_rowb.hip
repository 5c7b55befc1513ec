// Convolutions whose whole filter bank fits in LDS (1x1 and 3x3 windows on 64 .. 256 input channels, up to 72 KB of
// filters), with the activations going from memory straight into the MFMA operand registers.
//
// The tile kernel stages both operands of every 64-deep reduction tile in LDS and synchronises the workgroup once per
// tile; on layers with few output channels (a 64 x 64 tile re-reads 16 KB per 0.5 MFLOP) it spends its time waiting.
// Here the filters are copied to LDS once per workgroup, packed on the host in the order the matrix instruction reads
// them (step, channel tile, lane), and a wave owns 32 output pixels on its own: in reduction step t lanes 0..31 load
// channels 16 * (t % SPT) + 0..7 of tap t / SPT of their pixel and lanes 32..63 the next 8, one 16-byte buffer load each
// (a tap outside the image gets an out-of-range offset and reads zeros).  No activation tile in LDS, no workgroup
// barrier after the prologue, waves progress independently.
//   * Short reductions (at most 16 steps: 1x1 windows) keep all operand registers of the pixel tile and walk the
//     output channels in groups of 64 (the activations are read once).
//   * Long reductions (3x3 on 64 channels: 36 steps, 64 output channels) keep a window of 12 loads in flight: the
//     register of step t is refilled with step t + 12 as soon as its matrix instructions are issued.
// Epilogue per group of 64 channels: the residual tile is fetched with 16-byte loads (whole cache lines per pixel),
// handed to the accumulator layout through a private LDS block of the wave, added in fp32 after the bias, then
// activation, one rounding, and the way back through the same block to 16-byte stores.  fp32 accumulation in step order.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "device_types.h"
#include "mfma.h"

namespace mt {

namespace {

constexpr uint32_t ROWB_OOB = 0x80000000u;   // beyond any tensor: buffer loads return zeros

template <typename T, int R, int S, int SPT, int NTA, int NW>
__device__ __forceinline__ void rowb_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    constexpr int TAPS = R * S;
    constexpr int KS = TAPS * SPT;            // MFMA steps (16 reduction elements each)
    constexpr int C = 16 * SPT;               // input channels
    constexpr int NGRP = NTA / 2;             // groups of 64 output channels
    constexpr bool STATIONARY = KS <= 16;
    constexpr int WIN = STATIONARY ? KS : 12;  // operand registers (steps in flight)
    constexpr int SLD = 64 + 8;               // staging row in elements
    static_assert(NTA % 2 == 0, "output channels come in groups of 64");
    static_assert(STATIONARY || NGRP == 1, "a long reduction is walked once");
    static_assert(TAPS <= 32, "one validity bit per tap");
    typedef typename Mma<T, 32>::Acc Acc;

    __shared__ __attribute__((aligned(16))) u32x4 Wf[KS * NTA * 64];
    __shared__ __attribute__((aligned(16))) uint16_t stage[NW][32 * SLD];
    __shared__ __attribute__((aligned(16))) float bias_s[NTA * 32];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, px = lane & 31;

    // A workgroup owns one slice of 32 * NTA output channels (its filters are one contiguous block of the packed bank)
    // and every n_slices-th chunk of NW pixel tiles.
    const int n_slices = a.n_pad / (32 * NTA);
    const int slice = blockIdx.x % n_slices;
    const int kslice = slice * 32 * NTA;
    {
        const u32x4 *wp = reinterpret_cast<const u32x4 *>(a.w) + (size_t)slice * KS * NTA * 64;
        for (int c = tid; c < KS * NTA * 64; c += 64 * NW) Wf[c] = wp[c];
        for (int c = tid; c < NTA * 32; c += 64 * NW) bias_s[c] = a.bias[kslice + c];
    }
    __syncthreads();

    const int M = a.N * a.P * a.Q;
    const int n_tiles = (M + 31) / 32;
    const int size = a.N * a.H * a.W * C * 2;       // < 2 GiB by construction of the model
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, size, 0x00027000);
    T *y = reinterpret_cast<T *>(a.y);
    const T *res = reinterpret_cast<const T *>(a.res);
    uint16_t *sg = stage[wave];
    // staging coordinates of this lane's four 16-byte pieces: pixel row and first channel
    const int srow = lane >> 3, scol = (lane & 7) * 8;

    for (int tile = (blockIdx.x / n_slices) * NW + wave; tile < n_tiles; tile += (gridDim.x / n_slices) * NW) {
        const int m = tile * 32 + px;
        const bool ok = m < M;
        const uint32_t mm = ok ? (uint32_t)m : 0u;
        const uint32_t t1 = __umulhi(a.divpq_m, mm);
        const int n = (int)((t1 + ((mm - t1) >> a.divpq_s1)) >> a.divpq_s2);
        const uint32_t rem = mm - (uint32_t)n * (uint32_t)(a.P * a.Q);
        const uint32_t t2 = __umulhi(a.divq_m, rem);
        const int p = (int)((t2 + ((rem - t2) >> a.divq_s1)) >> a.divq_s2);
        const int q = (int)(rem - (uint32_t)p * (uint32_t)a.Q);
        const int ih0 = p * a.sh - a.ph, iw0 = q * a.sw - a.pw;
        const int pix = (((n * a.H + ih0) * a.W + iw0) * C + 8 * h) * 2;    // byte offset of tap (0, 0), this lane's half
        uint32_t tapmask = 0;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const bool v = ok & ((uint32_t)(ih0 + r) < (uint32_t)a.H) & ((uint32_t)(iw0 + s) < (uint32_t)a.W);
                tapmask |= v ? (1u << (r * S + s)) : 0u;
            }
        auto load_step = [&](int t) {
            const int tap = t / SPT, r = tap / S, s = tap % S;
            const int o = pix + ((r * a.W + s) * C + (t % SPT) * 16) * 2;
            const uint32_t voff = ((tapmask >> tap) & 1u) ? (uint32_t)o : ROWB_OOB;
            return __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, 0, 0);
        };

        u32x4 b[WIN];
        if constexpr (STATIONARY) {
#pragma unroll
            for (int t = 0; t < KS; ++t) b[t] = load_step(t);
        }
#pragma unroll 1
        for (int grp = 0; grp < NGRP; ++grp) {
            const int kb = grp * 64;
            u32x4 rr[4];
            if (res) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int mr = tile * 32 + srow + 8 * j;
                    rr[j] = mr < M ? *reinterpret_cast<const u32x4 *>(res + (int64_t)mr * a.res_ct + kslice + kb + scol) : u32x4{0u, 0u, 0u, 0u};
                }
            }
            Acc acc[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
            if constexpr (!STATIONARY) {
#pragma unroll
                for (int t = 0; t < WIN; ++t) b[t] = load_step(t);
            }
#pragma unroll
            for (int t = 0; t < KS; ++t) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[i] = Mma<T, 32>::run(Wf[(t * NTA + grp * 2 + i) * 64 + lane], b[t % WIN], acc[i]);
                if constexpr (!STATIONARY) {
                    if (t + WIN < KS) b[t % WIN] = load_step(t + WIN);
                }
            }
            // ---- epilogue of the group; the staging block is private to the wave and LDS serves a wave's accesses in
            // order, so compiler fences are all the synchronisation it takes
            if (res) {
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(&sg[(srow + 8 * j) * SLD + scol]) = rr[j];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int kl = i * 32 + 8 * g + 4 * h;
                    const float4 bv = *reinterpret_cast<const float4 *>(&bias_s[kb + kl]);
                    float v[4] = {acc[i][g * 4 + 0] + bv.x, acc[i][g * 4 + 1] + bv.y, acc[i][g * 4 + 2] + bv.z, acc[i][g * 4 + 3] + bv.w};
                    Pack<T, 4> *slot = reinterpret_cast<Pack<T, 4> *>(&sg[px * SLD + kl]);
                    if (res) {
                        const Pack<T, 4> rp = *slot;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += to_f32(rp.e[e]);
                    }
                    Pack<T, 4> o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) from_f32(apply_act(v[e], a.act), o.e[e]);
                    *slot = o;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = srow + 8 * j;
                const int mr = tile * 32 + row;
                const u32x4 v = *reinterpret_cast<const u32x4 *>(&sg[row * SLD + scol]);
                if (mr < M) *reinterpret_cast<u32x4 *>(y + (int64_t)mr * a.y_ct + a.y_coff + kslice + kb + scol) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}
template <typename T, int R, int S, int SPT, int NTA, int NW>
__global__ void __launch_bounds__(64 * NW) rowb_kernel(OpArgs a) {
    rowb_kernel_body<T, R, S, SPT, NTA, NW>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int R, int S, int SPT, int NTA, int NW>
__global__ void __launch_bounds__(64 * NW) rowb_pair_kernel(OpArgsPair p) {
    rowb_kernel_body<T, R, S, SPT, NTA, NW>(p.a[blockIdx.y]);
}

// 3x3 window, stride 1, 64 -> 64 channels: the activations go through LDS once, as the input patch of the wave's pixel
// tile, instead of once per tap through the L1.  A wave owns 4 x 8 output pixels; their 6 x 10 input pixels (128 bytes
// each, padded to 144 so that the fragment reads of neighbouring pixels fall into different banks) are
// fetched with whole-cache-line 16-byte loads (pixels outside the image read zeros) into a private LDS block, and the
// operand fragment of tap (r, s), channels 16 u + 8 h .. + 7 is the 16-byte piece at patch pixel (dy + r, dx + s).  Every
// input line is read from memory once per tile instead of nine times; the patch of the next tile is in flight (in
// registers) while the matrix instructions of the current one run.  Filters resident in LDS as above; the epilogue
// reuses the patch block as its staging block.  fp32 accumulation in step order (tap-major, 16 channels per step), the
// same order as the streaming form above.
template <typename T>
__device__ __forceinline__ void rowp_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    constexpr int KS = 36, NTA = 2, NW = 8, C = 64, SPT = 4;
    constexpr int TP = 4, TQ = 8;                 // output rows x columns of a wave tile
    constexpr int PR = TP + 2, PC = TQ + 2;       // its input patch
    constexpr int PIX = 72;                       // elements per patch pixel (128 + 16 bytes)
    // Elements per patch row: 10 pixels and 224 bytes, so that rows are 128 bytes apart modulo the 256 bytes of the LDS
    // banks.  The 16 lanes served together (8 pixels of two rows) then read 16 different 16-byte bank groups: pixels 144
    // bytes apart fall on groups 0, 9, 2, 11, 4, 13, 6, 15, the next row on the other eight.
    constexpr int PROW = PC * PIX + 112;
    constexpr int NCHUNK = PR * PC * 8;           // 16-byte pieces of a patch
    constexpr int NLD = (NCHUNK + 63) / 64;
    constexpr int SLD = PIX;                      // staging rows of the epilogue live in the same block
    typedef typename Mma<T, 32>::Acc Acc;

    __shared__ __attribute__((aligned(16))) u32x4 Wf[KS * NTA * 64];
    __shared__ __attribute__((aligned(16))) uint16_t patch[NW][PR * PROW];
    __shared__ __attribute__((aligned(16))) float bias_s[64];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, px = lane & 31;
    const int dy = px >> 3, dx = px & 7;
    {
        const u32x4 *wp = reinterpret_cast<const u32x4 *>(a.w);
        for (int c = tid; c < KS * NTA * 64; c += 64 * NW) Wf[c] = wp[c];
        if (tid < 64) bias_s[tid] = a.bias[tid];
    }
    __syncthreads();

    const int tiles_q = (a.Q + TQ - 1) / TQ, tiles_p = (a.P + TP - 1) / TP;
    const int per_img = tiles_p * tiles_q;
    const int n_tiles = a.N * per_img;
    const int size = a.N * a.H * a.W * C * 2;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, size, 0x00027000);
    T *y = reinterpret_cast<T *>(a.y);
    const T *res = reinterpret_cast<const T *>(a.res);
    uint16_t *pt = patch[wave];
    const int srow = lane >> 3, scol = (lane & 7) * 8;

    struct Where {
        int n, p0, q0;
    };
    auto where = [&](int tile) {
        Where w;
        w.n = tile / per_img;
        const int rem = tile - w.n * per_img;
        const int tp = rem / tiles_q;
        w.p0 = tp * TP;
        w.q0 = (rem - tp * tiles_q) * TQ;
        return w;
    };
    // piece c = lane + 64 k of the patch: pixel j = c / 8 = lane / 8 + 8 k, channels 8 * (lane % 8) ..
    auto fetch = [&](const Where &w, u32x4 (&g)[NLD]) {
#pragma unroll
        for (int k = 0; k < NLD; ++k) {
            const int j = (lane >> 3) + 8 * k;
            const int pr = (j * 205) >> 11, pc = j - pr * PC;      // j / 10 for j < 64
            const int ih = w.p0 - a.ph + pr, iw = w.q0 - a.pw + pc;
            const bool v = (j < PR * PC) & ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
            const uint32_t voff = v ? (uint32_t)((((w.n * a.H + ih) * a.W + iw) * C + (lane & 7) * 8) * 2) : ROWB_OOB;
            g[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, 0, 0);
        }
    };
    auto wave_fence = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    const int stride = gridDim.x * NW;
    int tile = blockIdx.x * NW + wave;
    u32x4 g[NLD];
    if (tile < n_tiles) fetch(where(tile), g);
    for (; tile < n_tiles; tile += stride) {
        const Where w = where(tile);
        // the patch block is private to the wave and LDS serves a wave's accesses in order: compiler fences suffice
        wave_fence();
#pragma unroll
        for (int k = 0; k < NLD; ++k) {
            const int j = (lane >> 3) + 8 * k;
            const int pr = (j * 205) >> 11, pc = j - pr * PC;
            if (j < PR * PC) *reinterpret_cast<u32x4 *>(&pt[pr * PROW + pc * PIX + (lane & 7) * 8]) = g[k];
        }
        wave_fence();
        if (tile + stride < n_tiles) fetch(where(tile + stride), g);

        // rows of the staging block = pixels of the tile in (dy, dx) order
        u32x4 rr[4];
        int mrow[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = srow + 8 * j;
            const int p = w.p0 + (row >> 3), q = w.q0 + (row & 7);
            mrow[j] = (p < a.P && q < a.Q) ? (w.n * a.P + p) * a.Q + q : -1;
            if (res) rr[j] = mrow[j] >= 0 ? *reinterpret_cast<const u32x4 *>(res + (int64_t)mrow[j] * a.res_ct + scol) : u32x4{0u, 0u, 0u, 0u};
        }
        Acc acc[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const int tap = t / SPT, r = tap / 3, sx = tap % 3, u = t % SPT;
            const u32x4 b = *reinterpret_cast<const u32x4 *>(&pt[(dy + r) * PROW + (dx + sx) * PIX + u * 16 + h * 8]);
#pragma unroll
            for (int i = 0; i < 2; ++i) acc[i] = Mma<T, 32>::run(Wf[(t * NTA + i) * 64 + lane], b, acc[i]);
        }
        wave_fence();                                   // every fragment is read before the block becomes the staging block
        if (res) {
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(&pt[(srow + 8 * j) * SLD + scol]) = rr[j];
            wave_fence();
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int kl = i * 32 + 8 * gq + 4 * h;
                const float4 bv = *reinterpret_cast<const float4 *>(&bias_s[kl]);
                float v[4] = {acc[i][gq * 4 + 0] + bv.x, acc[i][gq * 4 + 1] + bv.y, acc[i][gq * 4 + 2] + bv.z, acc[i][gq * 4 + 3] + bv.w};
                Pack<T, 4> *slot = reinterpret_cast<Pack<T, 4> *>(&pt[px * SLD + kl]);
                if (res) {
                    const Pack<T, 4> rp = *slot;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += to_f32(rp.e[e]);
                }
                Pack<T, 4> o;
#pragma unroll
                for (int e = 0; e < 4; ++e) from_f32(apply_act(v[e], a.act), o.e[e]);
                *slot = o;
            }
        wave_fence();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(&pt[(srow + 8 * j) * SLD + scol]);
            if (mrow[j] >= 0) *reinterpret_cast<u32x4 *>(y + (int64_t)mrow[j] * a.y_ct + a.y_coff + scol) = v;
        }
    }
}
template <typename T>
__global__ void __launch_bounds__(512) rowp_kernel(OpArgs a) {
    rowp_kernel_body<T>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T>
__global__ void __launch_bounds__(512) rowp_pair_kernel(OpArgsPair p) {
    rowp_kernel_body<T>(p.a[blockIdx.y]);
}

}  // namespace

// Channel tiles (of 32) per slice and waves per workgroup for a window / channel combination, 0 if there is no
// instantiation.  A slice's filters (32 * tiles * R * S * C elements) stay at or below 72 KB.
int rowb_tiles(int R, int S, int C, int channels) {
    if (R != S) return 0;
    if (R == 3) return (C == 64 && channels == 64) ? 2 : 0;
    if (R != 1) return 0;
    if (C == 64) return channels % 256 == 0 ? 8 : channels % 64 == 0 ? 2 : 0;
    if (C == 128) return channels % 128 == 0 ? 4 : 0;
    if (C == 256) return channels % 128 == 0 ? 4 : channels % 64 == 0 ? 2 : 0;
    return 0;
}

// The 3x3 layers of stride 1 take the patch form (rowp_kernel); its grid walks 4 x 8 pixel tiles, not runs of 32 pixels.
bool rowb_patch_form(const OpArgs &a) { return a.R == 3 && a.S == 3 && a.sh == 1 && a.sw == 1 && a.C == 64 && a.n_pad == 64; }

int rowb_waves(int R, int S, int C, int channels) { return rowb_tiles(R, S, C, channels) ? 8 : 0; }

int launch_rowb(const OpArgs &a, void *stream, const OpArgs *mate, int n_mates) {
    if (mate && (n_mates < 1 || n_mates >= COISSUE_MAX)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(a.grid_x), block(a.block);
    const int nta = rowb_tiles(a.R, a.S, a.C, a.n_pad);
    if (nta == 0 || (int)block.x != 64 * rowb_waves(a.R, a.S, a.C, a.n_pad)) return (int)hipErrorInvalidValue;
    auto go = [&]<typename T>() {
        if (a.R == 3 && rowb_patch_form(a)) MT_LAUNCH((rowp_kernel<T>), (rowp_pair_kernel<T>), grid, block, st, a, mate);
        else if (a.R == 3) MT_LAUNCH((rowb_kernel<T, 3, 3, 4, 2, 8>), (rowb_pair_kernel<T, 3, 3, 4, 2, 8>), grid, block, st, a, mate);
        else if (a.C == 64 && nta == 2) MT_LAUNCH((rowb_kernel<T, 1, 1, 4, 2, 8>), (rowb_pair_kernel<T, 1, 1, 4, 2, 8>), grid, block, st, a, mate);
        else if (a.C == 64) MT_LAUNCH((rowb_kernel<T, 1, 1, 4, 8, 8>), (rowb_pair_kernel<T, 1, 1, 4, 8, 8>), grid, block, st, a, mate);
        else if (a.C == 128) MT_LAUNCH((rowb_kernel<T, 1, 1, 8, 4, 8>), (rowb_pair_kernel<T, 1, 1, 8, 4, 8>), grid, block, st, a, mate);
        else if (nta == 2) MT_LAUNCH((rowb_kernel<T, 1, 1, 16, 2, 8>), (rowb_pair_kernel<T, 1, 1, 16, 2, 8>), grid, block, st, a, mate);
        else MT_LAUNCH((rowb_kernel<T, 1, 1, 16, 4, 8>), (rowb_pair_kernel<T, 1, 1, 16, 4, 8>), grid, block, st, a, mate);
    };
    if (a.dtype == MT_F16) go.template operator()<f16>();
    else go.template operator()<bf16>();
    return (int)hipGetLastError();
}

}  // namespace mt
