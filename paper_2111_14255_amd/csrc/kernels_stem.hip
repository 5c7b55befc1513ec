// First convolution of a network (three input channels, 2-byte storage, 3x3 or 7x7 window) on the gfx950 matrix
// cores, with the activations going from memory straight into the MFMA operand registers.
//
// With C = 3 the reduction index (r, s, c) of one output pixel is, for every filter row r, one contiguous run of
// 3 * S elements of an NHWC input row.  In the aligned form (even horizontal stride, even width) the run is widened by
// DUMMY leading elements so that it starts at a 4-byte address (the start element 3 * (q * sw - pw) - DUMMY is even
// with DUMMY = (3 * pw) % 2); in the general form a run may start on an odd element, and a group is then loaded from
// one element earlier with a fifth dword and shifted down 16 bits in registers.  Runs are padded to whole 16-byte
// groups of 8 elements; GR groups per filter row, R * GR groups per pixel.  The filter bank is packed on the host in the same index, with zeros at the dummy and padding positions.
// An MFMA step of v_mfma_f32_32x32x16 takes two groups: lanes 0..31 feed group 2t of their pixel, lanes 32..63 group
// 2t + 1, each with ONE 16-byte buffer load.  Neighbouring pixels read overlapping addresses, so a wave's load
// touches a handful of cache lines; there is no im2col tile in LDS and no workgroup barrier in the loop.
// What a load cannot know is masked in registers: elements of columns outside the image (left / right border), the
// dummy and the padding (their weights are zero, but the data must not be NaN or infinity).  Rows outside the image
// get an out-of-range offset, for which buffer loads return zeros.  A group that straddles the first or the last byte
// of the tensor is fetched dword by dword instead (wave-uniform branch, taken by the first and last rows only), so the
// result does not depend on how the hardware range-checks a partly out-of-range 16-byte access.
//
// The packed filters (KS steps x TN channel tiles x 64 lanes x 16 bytes, already in fragment order) are copied to LDS
// once per workgroup; a wave then walks 32-pixel tiles with a grid stride.  Epilogue: bias, activation, one rounding, then the wave's
// 32 x (32 * TN) tile goes through a private LDS block so that every store instruction writes whole 16-byte pieces of
// consecutive channels (full cache lines per pixel).  fp32 accumulation in step order t = 0 .. KS-1.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "device_types.h"
#include "mfma.h"

namespace mt {

namespace {

constexpr uint32_t STEM_OOB = 0x80000000u;   // beyond any tensor: buffer loads return zeros

template <typename T, int R, int S, int DUMMY, int TN, bool ALIGNED>
__device__ __forceinline__ void stem_kernel_body(const OpArgs &a) {
    static_assert(ALIGNED || DUMMY == 0, "the general form has no dummy element");
    set_wave_priority(a.prio);
    constexpr int SEG = DUMMY + 3 * S;        // elements of one filter row's run
    constexpr int GR = (SEG + 7) / 8;         // 16-byte groups per filter row
    constexpr int NG = R * GR;                // groups per pixel
    constexpr int KS = (NG + 1) / 2;          // MFMA steps
    constexpr int KC = 32 * TN;               // output channels
    constexpr int SLD = KC + 8;               // staging row in elements (16-byte aligned rows, 2-way conflicts at most)
    constexpr int CPR = KC / 8;               // 16-byte pieces per pixel
    static_assert(GR * 8 <= 32, "the validity mask of a run is one 32-bit word");
    typedef typename Mma<T, 32>::Acc Acc;

    __shared__ __attribute__((aligned(16))) u32x4 Wf[KS * TN * 64];
    __shared__ __attribute__((aligned(16))) uint16_t stage[4][32 * SLD];
    __shared__ __attribute__((aligned(16))) float bias_s[KC];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, px = lane & 31;

    const int M = a.N * a.P * a.Q;
    const int n_tiles = (M + 31) / 32;
    const int rowbytes = a.W * 3 * 2;
    const int size = a.N * a.H * rowbytes;    // < 2 GiB by construction of the model
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, size, 0x00027000);
    T *y = reinterpret_cast<T *>(a.y);

    // Requests the KS groups of this lane for its pixel of `tile`; vm = bit e set when element e of a run is a real
    // element of a column inside the image (the same for every filter row of the pixel).
    auto fetch = [&](int tile, u32x4 (&b)[KS], uint32_t &vm) {
        const int m = tile * 32 + px;
        const bool ok = m < M;
        const uint32_t mm = ok ? (uint32_t)m : 0u;
        const uint32_t t1 = __umulhi(a.divpq_m, mm);
        const int n = (int)((t1 + ((mm - t1) >> a.divpq_s1)) >> a.divpq_s2);
        const uint32_t rem = mm - (uint32_t)n * (uint32_t)(a.P * a.Q);
        const uint32_t t2 = __umulhi(a.divq_m, rem);
        const int p = (int)((t2 + ((rem - t2) >> a.divq_s1)) >> a.divq_s2);
        const int q = (int)(rem - (uint32_t)p * (uint32_t)a.Q);
        const int ih0 = p * a.sh - a.ph, col0 = q * a.sw - a.pw;
        const int base_e = ((n * a.H + ih0) * a.W + col0) * 3 - DUMMY;      // first element of the run of filter row 0
        const int s_lo = max(0, -col0), s_hi = min(S - 1, a.W - 1 - col0);
        const int e_lo = DUMMY + 3 * s_lo, e_hi = DUMMY + 3 * s_hi + 2;       // inclusive, e_hi <= 31
        const uint32_t upto = e_hi >= 31 ? 0xFFFFFFFFu : ((1u << (e_hi + 1)) - 1u);
        vm = (ok && s_hi >= s_lo) ? (upto & ~((1u << e_lo) - 1u)) : 0u;
        // ALIGNED: every run starts on an even element, a group is one 16-byte load.  Otherwise a run may start on an odd
        // element (odd stride, odd width, ...): the load starts one element earlier, takes a fifth dword, and the five
        // dwords are shifted down by 16 bits in registers.
        constexpr int SPAN = ALIGNED ? 16 : 20;                               // bytes a group's loads cover
        int off[KS];
        uint32_t live = 0;                    // bit t: the group lies in a row of the image
        uint32_t oddbits = 0;                 // bit t: the run of that group starts on an odd element
        bool straddles = false;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const int G0 = 2 * t, G1 = 2 * t + 1;
            const int r = h ? (G1 < NG ? G1 / GR : 0) : G0 / GR;
            const int g = h ? (G1 < NG ? G1 % GR : 0) : G0 % GR;
            const bool gok = h ? (G1 < NG) : true;
            const bool v = ok & gok & ((uint32_t)(ih0 + r) < (uint32_t)a.H);
            const int e0 = base_e + r * a.W * 3;
            const int odd = ALIGNED ? 0 : (e0 & 1);
            const int o = (e0 - odd) * 2 + g * 16;
            off[t] = o;
            live |= v ? (1u << t) : 0u;
            oddbits |= odd ? (1u << t) : 0u;
            straddles |= v & (((o < 0) & (o > -SPAN)) | ((o < size) & (o > size - SPAN)));
        }
        if (__builtin_amdgcn_ballot_w64(straddles) == 0) {
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                // a group wholly in front of the tensor holds only columns left of the image: zeros are its value
                const uint32_t voff = (((live >> t) & 1u) && off[t] >= 0) ? (uint32_t)off[t] : STEM_OOB;
                const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, 0, 0);
                if constexpr (ALIGNED) {
                    b[t] = w;
                } else {
                    const uint32_t w4 = __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff + 16u, 0, 0);
                    const uint32_t sh = ((oddbits >> t) & 1u) * 16u;
                    b[t] = u32x4{__builtin_amdgcn_alignbit(w[1], w[0], sh), __builtin_amdgcn_alignbit(w[2], w[1], sh),
                                 __builtin_amdgcn_alignbit(w[3], w[2], sh), __builtin_amdgcn_alignbit(w4, w[3], sh)};
                }
            }
        } else {
            // first / last rows of the tensor: dword by dword, and a last element that fills half a dword on its own
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                uint32_t w[5];
#pragma unroll
                for (int d = 0; d < (ALIGNED ? 4 : 5); ++d) {
                    const int od = off[t] + 4 * d;
                    const bool in = ((live >> t) & 1u) && od >= 0;
                    const uint32_t voff = in ? (uint32_t)od : STEM_OOB;
                    if (!ALIGNED && in && od + 2 == size) w[d] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rsrc, voff, 0, 0);
                    else w[d] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, 0, 0);
                }
                if constexpr (ALIGNED) {
                    b[t] = u32x4{w[0], w[1], w[2], w[3]};
                } else {
                    const uint32_t sh = ((oddbits >> t) & 1u) * 16u;
                    b[t] = u32x4{__builtin_amdgcn_alignbit(w[1], w[0], sh), __builtin_amdgcn_alignbit(w[2], w[1], sh),
                                 __builtin_amdgcn_alignbit(w[3], w[2], sh), __builtin_amdgcn_alignbit(w[4], w[3], sh)};
                }
            }
        }
    };

    auto finish = [&](int tile, const u32x4 (&b)[KS], uint32_t vm) {
        Acc acc[TN];
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
        // Interior tiles (every pixel's window inside the image: all lanes hold VM_FULL) only clear the dummy and the
        // padding, with masks known at compile time; border tiles expand each lane's own mask.
        constexpr uint32_t VM_FULL = (SEG >= 32 ? 0xFFFFFFFFu : ((1u << SEG) - 1u)) & ~((1u << DUMMY) - 1u);
        auto dmask = [](uint32_t two) { return ((two & 1u) ? 0x0000FFFFu : 0u) | ((two & 2u) ? 0xFFFF0000u : 0u); };
        auto steps = [&]<bool INTERIOR>() {
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                const int G0 = 2 * t, G1 = 2 * t + 1;
                const int g0 = G0 % GR, g1 = G1 < NG ? G1 % GR : 0;
                u32x4 bm = b[t];
                if constexpr (INTERIOR) {
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t m0 = dmask(VM_FULL >> (8 * g0 + 2 * d)), m1 = dmask(VM_FULL >> (8 * g1 + 2 * d));
                        if (m0 != 0xFFFFFFFFu || m1 != 0xFFFFFFFFu) bm[d] &= h ? m1 : m0;
                    }
                } else {
                    const uint32_t bits = vm >> (8 * (h ? g1 : g0));
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t lo = (uint32_t)((int32_t)(bits << (31 - 2 * d)) >> 31);
                        const uint32_t hi = (uint32_t)((int32_t)(bits << (30 - 2 * d)) >> 31);
                        bm[d] &= (lo & 0x0000FFFFu) | (hi & 0xFFFF0000u);
                    }
                }
#pragma unroll
                for (int i = 0; i < TN; ++i) acc[i] = Mma<T, 32>::run(Wf[(t * TN + i) * 64 + lane], bm, acc[i]);
            }
        };
        // lanes past the last pixel hold zeros and an empty mask; they do not force the slow form
        if (__builtin_amdgcn_ballot_w64(vm != VM_FULL && tile * 32 + px < M) == 0) steps.template operator()<true>();
        else steps.template operator()<false>();
        uint16_t *sg = stage[wave];
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int kl = i * 32 + 8 * g + 4 * h;
                const float4 bv = *reinterpret_cast<const float4 *>(&bias_s[kl]);
                Pack<T, 4> o;
                from_f32(apply_act(acc[i][g * 4 + 0] + bv.x, a.act), o.e[0]);
                from_f32(apply_act(acc[i][g * 4 + 1] + bv.y, a.act), o.e[1]);
                from_f32(apply_act(acc[i][g * 4 + 2] + bv.z, a.act), o.e[2]);
                from_f32(apply_act(acc[i][g * 4 + 3] + bv.w, a.act), o.e[3]);
                *reinterpret_cast<Pack<T, 4> *>(&sg[px * SLD + kl]) = o;
            }
        // the block is private to the wave and LDS serves a wave's accesses in order: a compiler fence is all it takes
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int c = lane; c < 32 * CPR; c += 64) {
            const int row = c / CPR, col = (c % CPR) * 8;
            const int m = tile * 32 + row;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(&sg[row * SLD + col]);
            if (m < M && col < a.K) *reinterpret_cast<u32x4 *>(y + (int64_t)m * a.y_ct + a.y_coff + col) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    const int stride = gridDim.x * 4;
    int tile = blockIdx.x * 4 + wave;
    u32x4 b[KS];
    uint32_t vm = 0;
    // the first tile's activations are requested before the filters, so that both trips to memory overlap
    if (tile < n_tiles) fetch(tile, b, vm);
    {
        const u32x4 *wp = reinterpret_cast<const u32x4 *>(a.w);
        for (int c = tid; c < KS * TN * 64; c += 256) Wf[c] = wp[c];
        if (tid < KC) bias_s[tid] = a.bias[tid];
    }
    __syncthreads();
    // One tile in flight per wave: the other waves of the SIMD cover its trips to memory.  (Requesting the next tile
    // before finishing the current one doubles the operand registers and leaves two waves per SIMD instead of three:
    // measured on MI355X, ResNet stem at batch 16 / 128, 15.1 / 67.8 us against 12.6 / 58.1 us.)
    while (tile < n_tiles) {
        finish(tile, b, vm);
        tile += stride;
        if (tile < n_tiles) fetch(tile, b, vm);
    }
}
template <typename T, int R, int S, int DUMMY, int TN, bool ALIGNED>
__global__ void __launch_bounds__(256) stem_kernel(OpArgs a) {
    stem_kernel_body<T, R, S, DUMMY, TN, ALIGNED>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int R, int S, int DUMMY, int TN, bool ALIGNED>
__global__ void __launch_bounds__(256) stem_pair_kernel(OpArgsPair p) {
    stem_kernel_body<T, R, S, DUMMY, TN, ALIGNED>(p.a[blockIdx.y]);
}

}  // namespace

// 0: no instantiation; 1: aligned form (even horizontal stride, even width, odd 3 * pad: with one dummy element every run
// starts on a 4-byte address); 2: general form (runs may start on an odd element).
int stem_form(int R, int S, int sw, int W, int pw, int channels) {
    if (!((R == 7 && S == 7) || (R == 3 && S == 3)) || !(channels == 32 || channels == 64)) return 0;
    return (sw % 2 == 0 && W % 2 == 0 && ((3 * pw) & 1)) ? 1 : 2;
}

int launch_stem(const OpArgs &a, void *stream, const OpArgs *mate, int n_mates) {
    if (mate && (n_mates < 1 || n_mates >= COISSUE_MAX)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(a.grid_x), block(256);
    const int tn = a.n_pad / 32;
    const int form = stem_form(a.R, a.S, a.sw, a.W, a.pw, a.n_pad);
    if (form == 0) return (int)hipErrorInvalidValue;
    auto go = [&]<typename T>() {
        if (form == 1) {
            if (a.R == 7 && tn == 2) MT_LAUNCH((stem_kernel<T, 7, 7, 1, 2, true>), (stem_pair_kernel<T, 7, 7, 1, 2, true>), grid, block, st, a, mate);
            else if (a.R == 7) MT_LAUNCH((stem_kernel<T, 7, 7, 1, 1, true>), (stem_pair_kernel<T, 7, 7, 1, 1, true>), grid, block, st, a, mate);
            else if (tn == 2) MT_LAUNCH((stem_kernel<T, 3, 3, 1, 2, true>), (stem_pair_kernel<T, 3, 3, 1, 2, true>), grid, block, st, a, mate);
            else MT_LAUNCH((stem_kernel<T, 3, 3, 1, 1, true>), (stem_pair_kernel<T, 3, 3, 1, 1, true>), grid, block, st, a, mate);
        } else {
            if (a.R == 7 && tn == 2) MT_LAUNCH((stem_kernel<T, 7, 7, 0, 2, false>), (stem_pair_kernel<T, 7, 7, 0, 2, false>), grid, block, st, a, mate);
            else if (a.R == 7) MT_LAUNCH((stem_kernel<T, 7, 7, 0, 1, false>), (stem_pair_kernel<T, 7, 7, 0, 1, false>), grid, block, st, a, mate);
            else if (tn == 2) MT_LAUNCH((stem_kernel<T, 3, 3, 0, 2, false>), (stem_pair_kernel<T, 3, 3, 0, 2, false>), grid, block, st, a, mate);
            else MT_LAUNCH((stem_kernel<T, 3, 3, 0, 1, false>), (stem_pair_kernel<T, 3, 3, 0, 1, false>), grid, block, st, a, mate);
        }
    };
    if (a.dtype == MT_F16) go.template operator()<f16>();
    else go.template operator()<bf16>();
    return (int)hipGetLastError();
}

}  // namespace mt
