// 3x3 convolutions of stride 1 and padding 1 on 64 k input channels as an implicit GEMM whose activation operand is
// staged in LDS as an input PATCH, once per 64 input channels, instead of as one im2col tile per filter tap.
//
// With stride 1 and padding 1 the input map has the shape of the output map, so for output pixel m (flattened over
// image, row, column) tap (r, s) reads input pixel m + (r - 1) W + (s - 1), provided the row and the column stay
// inside the image.  A workgroup owns 64 output channels x 64 consecutive output pixels; the input pixels
// m0 - W - 1 .. m0 + 64 + W of one 64-channel chunk form its patch (64 + 2 W + 2 pixels of 128 bytes, LDS rows padded
// to 144), and the operand fragment of pixel i for tap (r, s) is patch row i + r W + s.  Where the tap leaves the
// image the fragment is replaced by zeros in registers (one validity bit per pixel and tap).  The reduction index
// runs (channel chunk, tap, channel), so one patch serves nine reduction tiles and the activations cross the path
// memory -> registers -> LDS once instead of nine times; the filter tiles (64 channels x 64 deep, the host packs the
// bank in this order) are streamed three at a time (one filter row), three rows ahead in registers, double buffered
// in LDS: one workgroup barrier per filter row plus one per channel chunk (the patch is replaced in place; the next
// one waits in registers meanwhile).
//
// Eight waves: two groups of four split the four MFMA steps of every tile and add their accumulators through LDS at
// the end (group order); each wave holds a 32 x 32 piece of the tile.  Epilogue as in the tile kernel: fp32 tile in
// LDS, every thread finishes 8 consecutive channels of one pixel (bias, residual, activation, one rounding).
#include <hip/hip_runtime.h>

#include <utility>

#include "internal.h"
#include "device_types.h"
#include "mfma.h"

namespace mt {

namespace {

constexpr uint32_t PC_OOB = 0x80000000u;
constexpr int PC_LDK = IGEMM_BK + 8;     // LDS row: 64 elements + 16 bytes

// PPX: patch pixels the LDS block holds (>= 64 + 2 W + 2)
template <typename T, int PPX>
__device__ __forceinline__ void pconv_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    constexpr int BN = 64, BM = 64, NT = 512, LDK = PC_LDK;
    constexpr int A_TILE = BN * LDK;
    constexpr int PCH = (PPX * 8 + NT - 1) / NT;      // 16-byte patch pieces per thread
    typedef typename Mma<T, 32>::Acc Acc;
    __shared__ __attribute__((aligned(16))) uint16_t smem[6 * A_TILE + PPX * LDK];     // two sets of three filter tiles, the patch
    uint16_t *Ws = smem;
    uint16_t *Ps = smem + 6 * A_TILE;
    static_assert(sizeof(smem) >= (size_t)BM * (BN + 4) * sizeof(float), "epilogue tile must fit");
    static_assert(sizeof(smem) >= (size_t)16 * 256 * sizeof(float), "accumulator exchange must fit");

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wk = wave >> 2, wn = wave & 1, wm = (wave >> 1) & 1;
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;

    const int M = a.N * a.P * a.Q;
    const int W = a.W;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = a.n_pad / BN;
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int vid = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;     // each XCD's L2 serves a contiguous tile range
    if (vid >= total) return;
    const int n0 = (vid % tiles_n) * BN, m0 = (vid / tiles_n) * BM;
    const int ncc = a.C / 64;
    const int npx = BM + 2 * W + 2;                  // patch pixels in use (<= PPX, checked by the planner)
    const int f0 = m0 - W - 1;                        // flattened input pixel of patch row 0

    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((int64_t)M * a.C * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.w), 0, (int)((int64_t)a.n_pad * a.k_pad * 2), 0x00027000);

    // this lane's pixel for the activation fragments, and which taps stay inside the image
    uint32_t tapmask = 0;
    {
        const int m = m0 + wm * 32 + frag_row;
        const bool ok = m < M;
        const uint32_t mm = ok ? (uint32_t)m : 0u;
        const uint32_t t1 = __umulhi(a.divpq_m, mm);
        const int n = (int)((t1 + ((mm - t1) >> a.divpq_s1)) >> a.divpq_s2);
        const uint32_t rem = mm - (uint32_t)n * (uint32_t)(a.P * a.Q);
        const uint32_t t2 = __umulhi(a.divq_m, rem);
        const int p = (int)((t2 + ((rem - t2) >> a.divq_s1)) >> a.divq_s2);
        const int q = (int)(rem - (uint32_t)p * (uint32_t)a.Q);
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const bool v = ok & ((uint32_t)(p + r - 1) < (uint32_t)a.H) & ((uint32_t)(q + s - 1) < (uint32_t)a.W);
                tapmask |= v ? (1u << (r * 3 + s)) : 0u;
            }
    }

    // ---- loaders -----------------------------------------------------------------------------------------------
    const int arow = tid >> 3, akc = tid & 7;        // this thread's 16-byte piece of a filter tile / first patch piece
    const uint32_t a_voff = (uint32_t)(((n0 + arow) * a.k_pad + akc * 8) * 2);
    auto load_a = [&](int t) { return __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, a_voff, (uint32_t)(t * 64 * 2), 0); };
    auto store_a = [&](int slot, u32x4 v) { *reinterpret_cast<u32x4 *>(&Ws[slot * A_TILE + arow * LDK + akc * 8]) = v; };
    auto load_patch = [&](int cc, u32x4 (&pr)[PCH]) {
#pragma unroll
        for (int k = 0; k < PCH; ++k) {
            const int j = arow + 64 * k;
            const int f = f0 + j;
            const bool v = (j < npx) & (f >= 0) & (f < M);
            const uint32_t voff = v ? (uint32_t)((f * a.C + cc * 64 + akc * 8) * 2) : PC_OOB;
            pr[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, voff, 0, 0);
        }
    };
    auto store_patch = [&](const u32x4 (&pr)[PCH]) {
#pragma unroll
        for (int k = 0; k < PCH; ++k) {
            const int j = arow + 64 * k;
            if (j < PPX) *reinterpret_cast<u32x4 *>(&Ps[j * LDK + akc * 8]) = pr[k];
        }
    };

    // Two accumulators per wave, one per MFMA step of its half of a tile, so that consecutive matrix instructions do
    // not wait for each other; they are added (step 0 + step 1) before the groups meet.
    Acc acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;

    // A step of the main loop is one filter row of one channel chunk: three reduction tiles (s = 0, 1, 2) between two
    // workgroup barriers.  (One tile per barrier leaves a wave two dependent matrix instructions per barrier, and the
    // chain barrier -> fragment reads -> MFMA -> LDS store -> barrier, about 600 cycles, is paid 9 C / 64 times.)
    // Filter tiles wait in registers three steps ahead; the unroll of three makes both the register set and the
    // filter row static.
    const int nsteps = ncc * 3;
    u32x4 ar[3][3], pr[PCH];
    load_patch(0, pr);
    {
        u32x4 a0[3];
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) a0[sx] = load_a(sx);
#pragma unroll
        for (int d = 1; d <= 3; ++d)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) ar[d % 3][sx] = (d < nsteps) ? load_a(d * 3 + sx) : u32x4{0u, 0u, 0u, 0u};
        store_patch(pr);
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) store_a(sx, a0[sx]);
    }
    __syncthreads();

    int cc = 0;
    auto step = [&]<int S>(int u) {                      // S = u % 3 = filter row
        constexpr int S1 = (S + 1) % 3;
        if (u + 1 < nsteps) {
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) store_a(((u + 1) & 1) * 3 + sx, ar[S1][sx]);     // requested three steps ago
        }
        if (u + 4 < nsteps) {
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) ar[S1][sx] = load_a((u + 4) * 3 + sx);
        }
        if (S == 0 && cc + 1 < ncc) load_patch(cc + 1, pr);                                // three steps to arrive
        const uint16_t *wsb = Ws + (u & 1) * 3 * A_TILE + (wn * 32 + frag_row) * LDK + frag_k + wk * 32;
        const uint16_t *psb = Ps + (wm * 32 + frag_row + S * W) * LDK + frag_k + wk * 32;
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) {
            const bool tv = (tapmask >> (S * 3 + sx)) & 1u;
            const u32x4 fa0 = *reinterpret_cast<const u32x4 *>(wsb + sx * A_TILE);
            const u32x4 fa1 = *reinterpret_cast<const u32x4 *>(wsb + sx * A_TILE + 16);
            u32x4 fb0 = *reinterpret_cast<const u32x4 *>(psb + sx * LDK);
            u32x4 fb1 = *reinterpret_cast<const u32x4 *>(psb + sx * LDK + 16);
            fb0 = tv ? fb0 : u32x4{0u, 0u, 0u, 0u};
            fb1 = tv ? fb1 : u32x4{0u, 0u, 0u, 0u};
            acc0 = Mma<T, 32>::run(fa0, fb0, acc0);
            acc1 = Mma<T, 32>::run(fa1, fb1, acc1);
        }
        if (S == 2) {
            ++cc;
            if (cc < ncc) {
                __syncthreads();                       // every wave has read the old patch
                store_patch(pr);
            }
        }
        __syncthreads();
    };
    for (int u0 = 0; u0 < nsteps; u0 += 3) {
        step.template operator()<0>(u0);
        step.template operator()<1>(u0 + 1);
        step.template operator()<2>(u0 + 2);
    }
    Acc acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = acc0[v] + acc1[v];

    // ---- wave group 1 hands its accumulators to group 0 (the tile buffers are free: the loop ends with a barrier)
    {
        float *red = reinterpret_cast<float *>(smem);
        if (wk == 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) red[v * 256 + (tid & 255)] = acc[v];
        }
        __syncthreads();
        if (wk == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] += red[v * 256 + tid];
        }
    }

    // ---- epilogue: fp32 tile through LDS, then 8 channels of one pixel per thread ---------------------------------
    T *y = reinterpret_cast<T *>(a.y);
    const T *res = reinterpret_cast<const T *>(a.res);
    constexpr int ELD = BN + 4;
    float *et = reinterpret_cast<float *>(smem);
    const int erow = tid >> 3, ecol = (tid & 7) * 8;      // 64 pixels x 8 pieces = 512 threads
    const int em = m0 + erow, ek = n0 + ecol;
    const bool live = (em < M) & (ek < a.K);
    u32x4 res_raw = u32x4{0u, 0u, 0u, 0u};
    if (res && live) res_raw = *reinterpret_cast<const u32x4 *>(res + (int64_t)em * a.res_ct + ek);
    __syncthreads();                                      // the accumulator exchange has been read
    if (wk == 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int ml = wm * 32 + frag_row;
            const int kl = wn * 32 + 8 * g + 4 * (lane >> 5);
            const float4 b = *reinterpret_cast<const float4 *>(a.bias + n0 + kl);     // the bias is padded to n_pad
            float4 v;
            v.x = acc[g * 4 + 0] + b.x;
            v.y = acc[g * 4 + 1] + b.y;
            v.z = acc[g * 4 + 2] + b.z;
            v.w = acc[g * 4 + 3] + b.w;
            *reinterpret_cast<float4 *>(&et[ml * ELD + kl]) = v;
        }
    }
    __syncthreads();
    if (!live) return;
    float v[8];
    const float4 lo = *reinterpret_cast<const float4 *>(&et[erow * ELD + ecol]);
    const float4 hi = *reinterpret_cast<const float4 *>(&et[erow * ELD + ecol + 4]);
    v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    if (res) {
        const Pack<T, 8> rp = __builtin_bit_cast(Pack<T, 8>, res_raw);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] += to_f32(rp.e[t]);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = apply_act(v[t], a.act);
    store_pack<T, 8>(y + (int64_t)em * a.y_ct + a.y_coff + ek, v);
}
template <typename T, int PPX>
__global__ void __launch_bounds__(512) pconv_kernel(OpArgs a) {
    pconv_kernel_body<T, PPX>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int PPX>
__global__ void __launch_bounds__(512) pconv_pair_kernel(OpArgsPair p) {
    pconv_kernel_body<T, PPX>(p.a[blockIdx.y]);
}

}  // namespace

// Patch pixels of the smallest instantiation that holds a map of this width, 0 if there is none.
int pconv_patch_pixels(int W) {
    const int need = 64 + 2 * W + 2;
    return need <= 128 ? 128 : need <= 192 ? 192 : need <= 320 ? 320 : 0;
}

int launch_pconv(const OpArgs &a, void *stream, const OpArgs *mate, int n_mates) {
    if (mate && (n_mates < 1 || n_mates >= COISSUE_MAX)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(a.grid_x), block(512);
    const int ppx = pconv_patch_pixels(a.W);
    if (ppx == 0 || a.R != 3 || a.S != 3 || a.sh != 1 || a.sw != 1 || a.ph != 1 || a.pw != 1 || a.C % 64 != 0) return (int)hipErrorInvalidValue;
    auto go = [&]<typename T>() {
        if (ppx == 128) MT_LAUNCH((pconv_kernel<T, 128>), (pconv_pair_kernel<T, 128>), grid, block, st, a, mate);
        else if (ppx == 192) MT_LAUNCH((pconv_kernel<T, 192>), (pconv_pair_kernel<T, 192>), grid, block, st, a, mate);
        else MT_LAUNCH((pconv_kernel<T, 320>), (pconv_pair_kernel<T, 320>), grid, block, st, a, mate);
    };
    if (a.dtype == MT_F16) go.template operator()<f16>();
    else go.template operator()<bf16>();
    return (int)hipGetLastError();
}

}  // namespace mt
