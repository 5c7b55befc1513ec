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
// fp16 / bf16 inputs, fp32 accumulation; bias, residual, activation in fp32; one rounding on store.
// Tiny-M layers are split along j across workgroups; partial sums go to a workspace and the workgroup that
// arrives last adds them in split order, so the result does not depend on arrival order.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "device_types.h"

namespace mt {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 32;           // reduction elements per LDS tile
constexpr int LDK = BK + 8;      // padded LDS row (80 bytes: 16-byte reads of a wave fall in distinct banks)
constexpr int NXCD = 8;

template <typename T, int MF>
struct Mma;
template <>
struct Mma<f16, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<bf16, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<f16, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<bf16, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(uint4 a, uint4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

// BN: output channels per workgroup, BM: pixels per workgroup, WN x WM: wave grid (4 waves), MF: MFMA edge.
template <typename T, int BN, int BM, int WN, int WM, int MF, bool VEC_A>
__global__ void __launch_bounds__(256) igemm_kernel(OpArgs a) {
    static_assert(WN * WM == 4, "four waves per workgroup");
    constexpr int SUBN = BN / WN, SUBM = BM / WM;          // wave tile
    constexpr int TN = SUBN / MF, TM = SUBM / MF;          // MFMA tiles per wave
    static_assert(TN >= 1 && TM >= 1, "wave tile smaller than one MFMA");
    constexpr int KSTEPS = (MF == 32) ? BK / 16 : BK / 32; // MFMA issues per LDS tile
    constexpr int KLANES = 64 / MF;                        // lane groups along the reduction index
    constexpr int ACC_REGS = (MF == 32) ? 16 : 4;
    constexpr int CH_ROW = BK / 8;                         // 16-byte chunks per tile row
    constexpr int W_CHUNKS = (BN * CH_ROW + 255) / 256;    // chunks per thread, filter tile
    constexpr int X_CHUNKS = (BM * CH_ROW + 255) / 256;    // chunks per thread, pixel tile
    typedef typename Mma<T, MF>::Acc Acc;

    __shared__ __attribute__((aligned(16))) uint16_t Ws[BN * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Xs[BM * LDK];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wn = wave % WN, wm = wave / WN;

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
    const int tn_idx = tile % tiles_n;
    const int tm_idx = tile / tiles_n;
    const int n0 = tn_idx * BN;
    const int m0 = tm_idx * BM;

    const int nkt = a.k_pad / BK;
    const int kt_per = (nkt + a.split_k - 1) / a.split_k;
    const int kt_begin = z * kt_per;
    const int kt_end = min(nkt, kt_begin + kt_per);

    const T *x = (const T *)a.x;
    const uint16_t *wp = (const uint16_t *)a.w;

    // ---- per-thread load coordinates -------------------------------------------------------
    const int kc = tid % CH_ROW;          // chunk column (same for every chunk of this thread)
    const int row0 = tid / CH_ROW;        // first tile row; further chunks are 256/CH_ROW rows apart
    constexpr int ROW_STEP = 256 / CH_ROW;

    int64_t xbase[X_CHUNKS];              // element offset of (n, 0, 0, 0)
    int ih0[X_CHUNKS], iw0[X_CHUNKS];
    bool xrow_ok[X_CHUNKS];
#pragma unroll
    for (int i = 0; i < X_CHUNKS; ++i) {
        const int row = row0 + i * ROW_STEP;
        const int m = m0 + row;
        xrow_ok[i] = row < BM && m < M;
        const int mm = xrow_ok[i] ? m : 0;
        const int q = mm % a.Q;
        const int p = (mm / a.Q) % a.P;
        const int n = mm / (a.Q * a.P);
        xbase[i] = (int64_t)n * a.H * a.W * a.C;
        ih0[i] = p * a.sh - a.ph;
        iw0[i] = q * a.sw - a.pw;
    }
    // position of this thread's chunk inside the (r, s, c) reduction index
    int kr, ks, kcx;
    {
        const int j0 = kt_begin * BK + kc * 8;
        kcx = j0 % a.C;
        const int rs = j0 / a.C;
        ks = rs % a.S;
        kr = rs / a.S;
    }

    uint4 wreg[W_CHUNKS], xreg[X_CHUNKS];

    auto load_tiles = [&](int kt) {
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) {
            const int row = row0 + i * ROW_STEP;
            if (row < BN)
                wreg[i] = *reinterpret_cast<const uint4 *>(wp + (int64_t)(n0 + row) * a.k_pad + kt * BK + kc * 8);
        }
        if constexpr (VEC_A) {
#pragma unroll
            for (int i = 0; i < X_CHUNKS; ++i) {
                const int ih = ih0[i] + kr, iw = iw0[i] + ks;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (xrow_ok[i] && kr < a.R && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W)
                    v = *reinterpret_cast<const uint4 *>(x + xbase[i] + ((int64_t)ih * a.W + iw) * a.C + kcx);
                xreg[i] = v;
            }
            // advance the chunk by one tile along the reduction index
            kcx += BK;
            while (kcx >= a.C) {
                kcx -= a.C;
                if (++ks == a.S) {
                    ks = 0;
                    ++kr;
                }
            }
        } else {
            // input channels not a multiple of 8 (first layers, C = 3): gather element by element
            const int jbase = kt * BK + kc * 8;
#pragma unroll
            for (int i = 0; i < X_CHUNKS; ++i) {
                uint16_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int j = jbase + t;
                    const int c = j % a.C;
                    const int rs = j / a.C;
                    const int s = rs % a.S;
                    const int r = rs / a.S;
                    const int ih = ih0[i] + r, iw = iw0[i] + s;
                    uint16_t v = 0;
                    if (xrow_ok[i] && j < a.gemm_k && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W)
                        v = reinterpret_cast<const uint16_t *>(x)[xbase[i] + ((int64_t)ih * a.W + iw) * a.C + c];
                    e[t] = v;
                }
                xreg[i] = make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16),
                                     e[4] | ((uint32_t)e[5] << 16), e[6] | ((uint32_t)e[7] << 16));
            }
        }
    };

    auto store_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) {
            const int row = row0 + i * ROW_STEP;
            if (row < BN) *reinterpret_cast<uint4 *>(&Ws[row * LDK + kc * 8]) = wreg[i];
        }
#pragma unroll
        for (int i = 0; i < X_CHUNKS; ++i) {
            const int row = row0 + i * ROW_STEP;
            if (row < BM) *reinterpret_cast<uint4 *>(&Xs[row * LDK + kc * 8]) = xreg[i];
        }
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

    if (kt_begin < kt_end) load_tiles(kt_begin);
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        store_tiles();
        __syncthreads();
        if (kt + 1 < kt_end) load_tiles(kt + 1);     // next tile's global loads overlap the MFMAs below
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int koff = kk * (KLANES * 8) + frag_k;
            uint4 af[TN], bf[TM];
#pragma unroll
            for (int i = 0; i < TN; ++i)
                af[i] = *reinterpret_cast<const uint4 *>(&Ws[(wn * SUBN + i * MF + frag_row) * LDK + koff]);
#pragma unroll
            for (int j = 0; j < TM; ++j)
                bf[j] = *reinterpret_cast<const uint4 *>(&Xs[(wm * SUBM + j * MF + frag_row) * LDK + koff]);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) acc[i][j] = Mma<T, MF>::run(af[i], bf[j], acc[i][j]);
        }
        __syncthreads();
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
                for (int v = 0; v < ACC_REGS; ++v) wsp[((i * TM + j) * ACC_REGS + v) * 256 + tid] = acc[i][j][v];
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const unsigned old = atomicAdd(&a.counters[tile], 1u);
            s_last = (old == (unsigned)a.split_k - 1u);
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();
        const float *wsr = a.ws + (int64_t)tile * a.split_k * NACC * 256;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int v = 0; v < ACC_REGS; ++v) acc[i][j][v] = 0.f;
        for (int zz = 0; zz < a.split_k; ++zz) {
            const float *p = wsr + (int64_t)zz * NACC * 256;
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
#pragma unroll
                    for (int v = 0; v < ACC_REGS; ++v)
                        acc[i][j][v] += __builtin_nontemporal_load(&p[((i * TM + j) * ACC_REGS + v) * 256 + tid]);
        }
        if (tid == 0) a.counters[tile] = 0;      // ready for the next launch of this operator
    }

    // ---- epilogue: bias, residual, activation, one rounding, NHWC store -------------------------
    T *y = (T *)a.y;
    const T *res = (const T *)a.res;
    const bool vec_ok = (a.y_ct % 4 == 0) && (a.y_coff % 4 == 0) && (a.res_ct % 4 == 0);
    constexpr int GROUPS = ACC_REGS / 4;
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
                const float4 b = *reinterpret_cast<const float4 *>(a.bias + k);    // bias is padded to n_pad
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

template <typename T, int BN, int BM, int WN, int WM, int MF>
static void launch_cfg(const OpArgs &a, hipStream_t st) {
    const dim3 grid(a.grid_x), block(256);
    if (a.vec_a)
        hipLaunchKernelGGL((igemm_kernel<T, BN, BM, WN, WM, MF, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((igemm_kernel<T, BN, BM, WN, WM, MF, false>), grid, block, 0, st, a);
}

template <typename T>
static int launch_igemm_typed(const OpArgs &a, hipStream_t st) {
    switch (a.kernel_id) {
        case K_IGEMM_128x128: launch_cfg<T, 128, 128, 2, 2, 32>(a, st); break;
        case K_IGEMM_128x64: launch_cfg<T, 128, 64, 2, 2, 32>(a, st); break;
        case K_IGEMM_64x64: launch_cfg<T, 64, 64, 2, 2, 32>(a, st); break;
        case K_IGEMM_64x16: launch_cfg<T, 64, 16, 4, 1, 16>(a, st); break;
        default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

int launch_igemm(const OpArgs &a, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (a.dtype == MT_F16) return launch_igemm_typed<f16>(a, st);
    if (a.dtype == MT_BF16) return launch_igemm_typed<bf16>(a, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace mt
