// Channel-wise, bandwidth-bound operators (depthwise conv, pooling, global average pooling) and the
// generic direct convolution used for fp32 storage.  Activations are NHWC, so consecutive lanes of a
// wavefront touch consecutive channel vectors: every global access of a wave is one contiguous run.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "device_types.h"

namespace mt {

// Linear element index -> (channel vector, column, row, image).  Tensors stay below 2^31 elements (checked when a
// model is finalised), so the index arithmetic is 32-bit: a 64-bit division costs several hundred instructions,
// which is a large part of a kernel that otherwise makes one memory round trip.
struct ElemIdx {
    int cv, q, p, n;
    uint32_t m;       // pixel index (n * P + p) * Q + q
};
__device__ inline ElemIdx split_index(uint32_t g, int CV, int Q, int P) {
    ElemIdx e;
    e.m = g / (uint32_t)CV;
    e.cv = (int)(g - e.m * (uint32_t)CV);
    const uint32_t t = e.m / (uint32_t)Q;
    e.q = (int)(e.m - t * (uint32_t)Q);
    const uint32_t n = t / (uint32_t)P;
    e.p = (int)(t - n * (uint32_t)P);
    e.n = (int)n;
    return e;
}

// ---------------------------------------------------------------------------------------------
// Direct convolution / fully connected: one thread per output element, output channel fastest.
// Sum order is fixed (r, s, c), so the result does not depend on the launch environment.
template <typename T>
__global__ void __launch_bounds__(256) conv_direct_kernel(OpArgs a) {
    set_wave_priority(a.prio);
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * a.K;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const ElemIdx e = split_index(gid, a.K, a.Q, a.P);
    const int k = e.cv, q = e.q, p = e.p, n = e.n;
    const int64_t m = e.m;
    const T *x = (const T *)a.x;
    const T *w = (const T *)a.w + (int64_t)k * a.R * a.S * a.C;
    const bool vec4 = (a.C % 4 == 0) && (a.x_ct % 4 == 0) && (a.x_coff % 4 == 0) && (((uintptr_t)a.x | (uintptr_t)a.w) % 16 == 0);
    float acc = 0.f;
    for (int r = 0; r < a.R; ++r) {
        const int ih = p * a.sh - a.ph + r;
        if (ih < 0 || ih >= a.H) continue;
        for (int s = 0; s < a.S; ++s) {
            const int iw = q * a.sw - a.pw + s;
            if (iw < 0 || iw >= a.W) continue;
            const T *xp = x + (((int64_t)n * a.H + ih) * a.W + iw) * a.x_ct + a.x_coff;
            const T *wp = w + ((int64_t)r * a.S + s) * a.C;
            int c = 0;
            if constexpr (sizeof(T) == 4) {
                // four channels per step when both rows are 16-byte aligned: the same products added in the same
                // order, with a quarter of the loads
                if (vec4) {
                    for (; c + 4 <= a.C; c += 4) {
                        const float4 xv = *reinterpret_cast<const float4 *>(xp + c);
                        const float4 wv = *reinterpret_cast<const float4 *>(wp + c);
                        acc = fmaf(xv.x, wv.x, acc);
                        acc = fmaf(xv.y, wv.y, acc);
                        acc = fmaf(xv.z, wv.z, acc);
                        acc = fmaf(xv.w, wv.w, acc);
                    }
                }
            }
            for (; c < a.C; ++c) acc = fmaf(to_f32(xp[c]), to_f32(wp[c]), acc);
        }
    }
    if (a.bias) acc += a.bias[k];
    if (a.res) acc += to_f32(((const T *)a.res)[m * a.res_ct + k]);
    acc = apply_act(acc, a.act);
    T o;
    from_f32(acc, o);
    ((T *)a.y)[m * a.y_ct + a.y_coff + k] = o;
}

// ---------------------------------------------------------------------------------------------
// Depthwise convolution, any window.  One thread per (pixel, V-channel vector); weights repacked as [R][S][C] so
// that the weight vector of a tap is one contiguous load, shared by every pixel through the caches.
template <typename T, int V>
__device__ __forceinline__ void dwconv_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * CV;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const ElemIdx e = split_index(gid, CV, a.Q, a.P);
    const int cv = e.cv, q = e.q, p = e.p, n = e.n;
    const int64_t m = e.m;
    const int c0 = cv * V;
    const T *x = (const T *)a.x;
    const T *w = (const T *)a.w;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;

    for (int r = 0; r < a.R; ++r) {
        const int ih = p * a.sh - a.ph + r;
        if (ih < 0 || ih >= a.H) continue;
        for (int s = 0; s < a.S; ++s) {
            const int iw = q * a.sw - a.pw + s;
            if (iw < 0 || iw >= a.W) continue;
            float xv[V], wv[V];
            load_pack<T, V>(x + (((int64_t)n * a.H + ih) * a.W + iw) * a.C + c0, xv);
            load_pack<T, V>(w + ((int64_t)r * a.S + s) * a.C + c0, wv);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = fmaf(xv[i], wv[i], acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) {
        if (a.bias) acc[i] += a.bias[c0 + i];
        acc[i] = apply_act(acc[i], a.act);
    }
    store_pack<T, V>((T *)a.y + m * a.y_ct + a.y_coff + c0, acc);
}
template <typename T, int V>
__global__ void __launch_bounds__(256) dwconv_kernel(OpArgs a) {
    dwconv_kernel_body<T, V>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V>
__global__ void __launch_bounds__(256) dwconv_pair_kernel(OpArgsPair p) {
    dwconv_kernel_body<T, V>(p.a[blockIdx.y]);
}

// ---------------------------------------------------------------------------------------------
// Fixed-window variants (KS x KS known at compile time, 16-byte channel vectors).  All taps are loaded first,
// from clamped addresses and without branches, so the loads of a thread overlap instead of each waiting for the
// one before it; taps in the padding halo are masked afterwards.  Tap order of the sums is the same (r, s).
template <typename T, int V, int KS>
__device__ __forceinline__ void dwconv_fixed_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * CV;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const ElemIdx e = split_index(gid, CV, a.Q, a.P);
    const int cv = e.cv, q = e.q, p = e.p, n = e.n;
    const int64_t m = e.m;
    const int c0 = cv * V;
    const T *x = (const T *)a.x + (int64_t)n * a.H * a.W * a.C + c0;
    const T *w = (const T *)a.w + c0;
    float xv[KS * KS][V], wv[KS * KS][V], bv[V];
    bool ok[KS * KS];
#pragma unroll
    for (int r = 0; r < KS; ++r)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int ih = p * a.sh - a.ph + r, iw = q * a.sw - a.pw + s;
            ok[r * KS + s] = ((unsigned)ih < (unsigned)a.H) & ((unsigned)iw < (unsigned)a.W);
            const int ihc = min(max(ih, 0), a.H - 1), iwc = min(max(iw, 0), a.W - 1);
            load_pack<T, V>(x + ((int64_t)ihc * a.W + iwc) * a.C, xv[r * KS + s]);
            load_pack<T, V>(w + (int64_t)(r * KS + s) * a.C, wv[r * KS + s]);
        }
    // the bias vector always exists (zeros when the layer has none): loaded with the taps, not after the sum
#pragma unroll
    for (int i = 0; i < V; i += 4) {
        const float4 b4 = *reinterpret_cast<const float4 *>(a.bias + c0 + i);
        bv[i] = b4.x; bv[i + 1] = b4.y; bv[i + 2] = b4.z; bv[i + 3] = b4.w;
    }
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
#pragma unroll
    for (int t = 0; t < KS * KS; ++t)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = ok[t] ? fmaf(xv[t][i], wv[t][i], acc[i]) : acc[i];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = apply_act(acc[i] + bv[i], a.act);
    store_pack<T, V>((T *)a.y + m * a.y_ct + a.y_coff + c0, acc);
}
template <typename T, int V, int KS>
__global__ void __launch_bounds__(256) dwconv_fixed_kernel(OpArgs a) {
    dwconv_fixed_kernel_body<T, V, KS>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V, int KS>
__global__ void __launch_bounds__(256) dwconv_fixed_pair_kernel(OpArgsPair p) {
    dwconv_fixed_kernel_body<T, V, KS>(p.a[blockIdx.y]);
}

// 3x3 depthwise convolution with padding 1 on a large map: a thread owns one (column, channel vector) of a band of
// `rows` output rows and keeps the three input rows of the window in registers, so that an output row costs one new
// input row (stride 1) or two (stride 2) instead of three.  Along a row the neighbouring columns are the own columns of
// the threads CV lanes to either side (channel vector is the fastest thread index), so at stride 1 a thread loads only
// its own column of a new row and takes the left and right taps from those lanes with wavefront shuffles; lanes whose
// neighbour lies in another wavefront load it themselves.  At stride 2 the left tap is the neighbour's right column.
// Taps are multiplied in the order (r, s) of the other depthwise kernels and every value has the bits a load would give,
// so the result is bit-identical to theirs.  Lanes beyond the last thread mirror it (they take part in the shuffles)
// and store nothing.
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));

template <typename T, int ST>
__device__ __forceinline__ void dwconv3_rows_kernel_body(const OpArgs &a, int rows, int bands) {
    static_assert(sizeof(T) == 2, "16-byte vectors of 8 channels");
    constexpr int V = 8;
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * bands * a.Q * CV;
    const uint32_t gid0 = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = gid0 < total;
    const ElemIdx e = split_index(live ? gid0 : total - 1, CV, a.Q, bands);
    const int cv = e.cv, q = e.q, band = e.p, n = e.n;
    const int lane = threadIdx.x & 63;
    const int c0 = cv * V;
    const T *x = (const T *)a.x + (int64_t)n * a.H * a.W * a.C + c0;
    const T *w = (const T *)a.w + c0;
    u32x4v wv[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) wv[t] = *reinterpret_cast<const u32x4v *>(w + (int64_t)t * a.C);
    float bv[V];
#pragma unroll
    for (int i = 0; i < V; i += 4) {
        const float4 b4 = *reinterpret_cast<const float4 *>(a.bias + c0 + i);
        bv[i] = b4.x; bv[i + 1] = b4.y; bv[i + 2] = b4.z; bv[i + 3] = b4.w;
    }
    const bool l_lane = lane >= CV, r_lane = lane + CV < 64;      // the neighbouring column's thread is in this wavefront
    const int iw1 = q * ST - 1 + 1;                               // the centre tap's column: always inside the map
    const bool ok_s[3] = {q * ST - 1 >= 0, true, q * ST + 1 < a.W};
    auto shuffle = [&](u32x4v v, int src) {
        u32x4v o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (uint32_t)__shfl((int)v[k], src, 64);
        return o;
    };
    auto at = [&](const T *row, int iw) { return *reinterpret_cast<const u32x4v *>(row + (int64_t)iw * a.C); };
    // one input row: the three taps of this thread's window (values of taps in the padding are never used)
    auto load_row = [&](int ih, u32x4v (&taps)[3], bool &ok) {
        ok = (unsigned)ih < (unsigned)a.H;
        const T *row = x + (int64_t)min(max(ih, 0), a.H - 1) * a.W * a.C;
        const u32x4v c = at(row, iw1);
        taps[1] = c;
        if constexpr (ST == 1) {
            u32x4v l = shuffle(c, lane - CV), r = shuffle(c, lane + CV);
            if (!l_lane && ok_s[0]) l = at(row, iw1 - 1);
            if (!r_lane && ok_s[2]) r = at(row, iw1 + 1);
            taps[0] = l;
            taps[2] = r;
        } else {
            const u32x4v r = at(row, ok_s[2] ? iw1 + 1 : iw1);
            u32x4v l = shuffle(r, lane - CV);                     // the left neighbour's right column is this thread's left one
            if (!l_lane && ok_s[0]) l = at(row, iw1 - 1);
            taps[0] = l;
            taps[2] = r;
        }
    };
    const int p0 = band * rows, p1 = min(a.P, p0 + rows);
    u32x4v win[3][3];
    bool rok[3];
    load_row(p0 * ST - 1, win[0], rok[0]);
    load_row(p0 * ST, win[1], rok[1]);
    for (int p = p0; p < p1; ++p) {                               // uniform trip count within a wavefront's band... per thread the same p range
        load_row(p * ST + 1, win[2], rok[2]);
        float acc[V];
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = 0.f;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) {
                const Pack<T, V> xv = __builtin_bit_cast(Pack<T, V>, win[r][sx]);
                const Pack<T, V> wt = __builtin_bit_cast(Pack<T, V>, wv[r * 3 + sx]);
                const bool ok = rok[r] & ok_s[sx];
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = ok ? fmaf(to_f32(xv.e[i]), to_f32(wt.e[i]), acc[i]) : acc[i];
            }
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = apply_act(acc[i] + bv[i], a.act);
        if (live) store_pack<T, V>((T *)a.y + ((int64_t)(n * a.P + p) * a.Q + q) * a.y_ct + a.y_coff + c0, acc);
        if constexpr (ST == 1) {
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) { win[0][sx] = win[1][sx]; win[1][sx] = win[2][sx]; }
            rok[0] = rok[1]; rok[1] = rok[2];
        } else {
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) win[0][sx] = win[2][sx];
            rok[0] = rok[2];
            if (p + 1 < p1) load_row((p + 1) * ST, win[1], rok[1]);
        }
    }
}
template <typename T, int ST>
__global__ void __launch_bounds__(256) dwconv3_rows_kernel(OpArgs a, int rows, int bands) {
    dwconv3_rows_kernel_body<T, ST>(a, rows, bands);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int ST>
__global__ void __launch_bounds__(256) dwconv3_rows_pair_kernel(OpArgsPair p, int rows, int bands) {
    dwconv3_rows_kernel_body<T, ST>(p.a[blockIdx.y], rows, bands);
}

// Output rows per thread of the banded 3x3 depthwise kernel: 1 (the one-pixel kernel) unless the map is large enough
// to leave at least 65536 threads with 2 or 4 rows each.  A pure function of the operator's shape.
static int dwconv_band_rows(const OpArgs &a) {
    if (a.dtype == MT_F32 || a.R != 3 || a.S != 3 || a.ph != 1 || a.pw != 1 || a.sh != a.sw || a.sh < 1 || a.sh > 2 || a.vec != 8) return 1;
    const int64_t th = (int64_t)a.N * a.P * a.Q * (a.C / 8);
    return th >= 4 * 65536 ? 4 : th >= 2 * 65536 ? 2 : 1;
}

template <typename T, int V, bool IS_MAX, int KS>
__device__ __forceinline__ void pool_fixed_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * CV;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const ElemIdx e = split_index(gid, CV, a.Q, a.P);
    const int cv = e.cv, q = e.q, p = e.p, n = e.n;
    const int64_t m = e.m;
    const int c0 = cv * V;
    const T *x = (const T *)a.x + (int64_t)n * a.H * a.W * a.C + c0;
    float xv[KS * KS][V];
    bool ok[KS * KS];
#pragma unroll
    for (int r = 0; r < KS; ++r)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int ih = p * a.sh - a.ph + r, iw = q * a.sw - a.pw + s;
            ok[r * KS + s] = ((unsigned)ih < (unsigned)a.H) & ((unsigned)iw < (unsigned)a.W);
            const int ihc = min(max(ih, 0), a.H - 1), iwc = min(max(iw, 0), a.W - 1);
            load_pack<T, V>(x + ((int64_t)ihc * a.W + iwc) * a.C, xv[r * KS + s]);
        }
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = IS_MAX ? -INFINITY : 0.f;
    int cnt = 0;
#pragma unroll
    for (int t = 0; t < KS * KS; ++t) {
        cnt += ok[t] ? 1 : 0;
#pragma unroll
        for (int i = 0; i < V; ++i)
            acc[i] = ok[t] ? (IS_MAX ? fmaxf(acc[i], xv[t][i]) : acc[i] + xv[t][i]) : acc[i];
    }
    if (!IS_MAX) {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = acc[i] / (float)cnt;
    }
    store_pack<T, V>((T *)a.y + m * a.y_ct + a.y_coff + c0, acc);
}
template <typename T, int V, bool IS_MAX, int KS>
__global__ void __launch_bounds__(256) pool_fixed_kernel(OpArgs a) {
    pool_fixed_kernel_body<T, V, IS_MAX, KS>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V, bool IS_MAX, int KS>
__global__ void __launch_bounds__(256) pool_fixed_pair_kernel(OpArgsPair p) {
    pool_fixed_kernel_body<T, V, IS_MAX, KS>(p.a[blockIdx.y]);
}

// ---------------------------------------------------------------------------------------------
// Window pooling: one thread per (output pixel, V-channel vector).
template <typename T, int V, bool IS_MAX>
__device__ __forceinline__ void pool_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * CV;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const ElemIdx e = split_index(gid, CV, a.Q, a.P);
    const int cv = e.cv, q = e.q, p = e.p, n = e.n;
    const int64_t m = e.m;
    const int c0 = cv * V;
    const T *x = (const T *)a.x;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = IS_MAX ? -INFINITY : 0.f;
    int cnt = 0;
    for (int r = 0; r < a.R; ++r) {
        const int ih = p * a.sh - a.ph + r;
        if (ih < 0 || ih >= a.H) continue;
        for (int s = 0; s < a.S; ++s) {
            const int iw = q * a.sw - a.pw + s;
            if (iw < 0 || iw >= a.W) continue;
            float xv[V];
            load_pack<T, V>(x + (((int64_t)n * a.H + ih) * a.W + iw) * a.C + c0, xv);
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] = IS_MAX ? fmaxf(acc[i], xv[i]) : acc[i] + xv[i];
            ++cnt;
        }
    }
    if (!IS_MAX) {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = acc[i] / (float)cnt;
    }
    store_pack<T, V>((T *)a.y + m * a.y_ct + a.y_coff + c0, acc);
}
template <typename T, int V, bool IS_MAX>
__global__ void __launch_bounds__(256) pool_kernel(OpArgs a) {
    pool_kernel_body<T, V, IS_MAX>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V, bool IS_MAX>
__global__ void __launch_bounds__(256) pool_pair_kernel(OpArgsPair p) {
    pool_kernel_body<T, V, IS_MAX>(p.a[blockIdx.y]);
}

// ---------------------------------------------------------------------------------------------
// Global average pooling.  A wavefront owns one (image, group of channel vectors): its 64 lanes are
// arranged as LANES_HW spatial slices x LANES_C channel vectors; each lane sums its slice in order and
// the slices are combined by a fixed butterfly of wavefront shuffles, so the sum order is fixed.
template <typename T, int V>
__device__ __forceinline__ void gap_kernel_body(const OpArgs &a, int lanes_c) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const int lanes_hw = 64 / lanes_c;
    const int groups = (CV + lanes_c - 1) / lanes_c;            // wave tasks per image
    const int wave = (int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    const int lane = threadIdx.x & 63;
    if (wave >= a.N * groups) return;                            // whole wave exits together
    const int n = wave / groups;
    const int cv = (wave % groups) * lanes_c + (lane % lanes_c);
    const int slice = lane / lanes_c;
    const int HW = a.H * a.W;
    const bool cv_ok = cv < CV;
    const T *x = (const T *)a.x + (int64_t)n * HW * a.C + (cv_ok ? cv : 0) * V;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    // four pixels of the slice per round, loaded before any is added (clamped address + select, no branch)
    for (int base = slice; base < HW; base += 4 * lanes_hw) {
        float xv[4][V];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * lanes_hw;
            ok[u] = i < HW;
            load_pack<T, V>(x + (int64_t)(ok[u] ? i : slice) * a.C, xv[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] = ok[u] ? acc[j] + xv[u][j] : acc[j];
    }
    for (int off = 32; off >= lanes_c; off >>= 1) {
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] += __shfl_xor(acc[j], off);
    }
    if (slice == 0 && cv_ok) {
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] = acc[j] / (float)HW;
        store_pack<T, V>((T *)a.y + (int64_t)n * a.y_ct + a.y_coff + cv * V, acc);
    }
}
template <typename T, int V>
__global__ void __launch_bounds__(256) gap_kernel(OpArgs a, int lanes_c) {
    gap_kernel_body<T, V>(a, lanes_c);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V>
__global__ void __launch_bounds__(256) gap_pair_kernel(OpArgsPair p, int lanes_c) {
    gap_kernel_body<T, V>(p.a[blockIdx.y], lanes_c);
}

// ---------------------------------------------------------------------------------------------
// Local response normalisation across channels: out[c] = in[c] / (k + alpha * sum_{|j-c| <= size/2} in[j]^2)^beta.
// One thread per (pixel, V-channel vector); it loads its own vector and the two neighbouring vectors (the window
// reaches at most 7 channels to either side, V >= 8 for the vector form), all before any arithmetic.
template <typename T, int V>
__device__ __forceinline__ void lrn_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * CV;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const uint32_t m = gid / (uint32_t)CV;
    const int cv = (int)(gid - m * (uint32_t)CV);
    const int c0 = cv * V;
    const int half = a.R / 2;
    const T *x = (const T *)a.x + (int64_t)m * a.C;
    float win[3 * V];                        // channels c0 - V .. c0 + 2V - 1, zero outside the tensor
    if constexpr (V > 1) {
        float lo[V], mid[V], hi[V];
        const bool has_lo = cv > 0, has_hi = cv + 1 < CV;
        load_pack<T, V>(x + (has_lo ? c0 - V : c0), lo);
        load_pack<T, V>(x + c0, mid);
        load_pack<T, V>(x + (has_hi ? c0 + V : c0), hi);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            win[i] = has_lo ? lo[i] : 0.f;
            win[V + i] = mid[i];
            win[2 * V + i] = has_hi ? hi[i] : 0.f;
        }
    } else {
        for (int i = 0; i < 3; ++i) win[i] = 0.f;
        win[1] = to_f32(x[c0]);
    }
    float out[V];
    if constexpr (V > 1) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            float ssq = 0.f;
#pragma unroll
            for (int d = -7; d <= 7; ++d) {
                const float v = win[V + i + d];
                ssq = (d >= -half && d <= half) ? fmaf(v, v, ssq) : ssq;
            }
            out[i] = win[V + i] / powf(a.lrn_k + a.lrn_alpha * ssq, a.lrn_beta);
        }
    } else {
        float ssq = 0.f;
        for (int d = -half; d <= half; ++d) {
            const int c = c0 + d;
            if (c >= 0 && c < a.C) {
                const float v = to_f32(x[c]);
                ssq = fmaf(v, v, ssq);
            }
        }
        out[0] = win[1] / powf(a.lrn_k + a.lrn_alpha * ssq, a.lrn_beta);
    }
    store_pack<T, V>((T *)a.y + (int64_t)m * a.y_ct + a.y_coff + c0, out);
}
template <typename T, int V>
__global__ void __launch_bounds__(256) lrn_kernel(OpArgs a) {
    lrn_kernel_body<T, V>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V>
__global__ void __launch_bounds__(256) lrn_pair_kernel(OpArgsPair p) {
    lrn_kernel_body<T, V>(p.a[blockIdx.y]);
}

// Element-wise sum of two tensors of the same shape, activation, one rounding.
template <typename T, int V>
__device__ __forceinline__ void add_kernel_body(const OpArgs &a) {
    set_wave_priority(a.prio);
    const int CV = a.C / V;
    const uint32_t total = (uint32_t)a.N * a.P * a.Q * CV;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const uint32_t m = gid / (uint32_t)CV;
    const int c0 = (int)(gid - m * (uint32_t)CV) * V;
    float u[V], v[V];
    load_pack<T, V>((const T *)a.x + (int64_t)m * a.C + c0, u);
    load_pack<T, V>((const T *)a.res + (int64_t)m * a.res_ct + c0, v);
#pragma unroll
    for (int i = 0; i < V; ++i) u[i] = apply_act(u[i] + v[i], a.act);
    store_pack<T, V>((T *)a.y + (int64_t)m * a.y_ct + a.y_coff + c0, u);
}
template <typename T, int V>
__global__ void __launch_bounds__(256) add_kernel(OpArgs a) {
    add_kernel_body<T, V>(a);
}
// two operators of equal launch shape in one launch, one per value of blockIdx.y
template <typename T, int V>
__global__ void __launch_bounds__(256) add_pair_kernel(OpArgsPair p) {
    add_kernel_body<T, V>(p.a[blockIdx.y]);
}

// Records the hardware id registers of the compute unit each one-wavefront workgroup runs on, then keeps the unit
// busy for a few microseconds so that later workgroups spread over every unit the queue may use.
__global__ void __launch_bounds__(64) probe_kernel(uint32_t *out) {
    const uint32_t hw_id = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);     // HW_REG_HW_ID, 32 bits
    const uint32_t xcc_id = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 20);   // HW_REG_XCC_ID, 32 bits
    float v = (float)threadIdx.x;
    for (int i = 0; i < 4000; ++i) v = fmaf(v, 1.0000001f, 1e-7f);
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x + 0] = hw_id;
        out[2 * blockIdx.x + 1] = xcc_id | (v == 12345.f ? 0x80000000u : 0u);   // keeps the loop alive
    }
}

// Arrival at a stage barrier taken with a counter: one thread bumps the word that the queues of the next stage poll.
// System scope, release: the word lives in host-visible signal memory and the increment must not pass the stage's stores.
__global__ void __launch_bounds__(64) arrive_kernel(uint32_t *counter) {
    if (threadIdx.x == 0) __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void fill_u32_kernel(uint32_t *p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---------------------------------------------------------------------------------------------
template <typename T>
static int launch_typed(const OpArgs &a, hipStream_t st, const OpArgs *mate, int n_mates) {
    const dim3 block(256);
    auto blocks = [](int64_t threads) { return dim3((unsigned)((threads + 255) / 256)); };
    constexpr int VMAX = 16 / sizeof(T);          // 16-byte accesses
    switch (a.kernel_id) {
        case K_CONV_DIRECT:
            hipLaunchKernelGGL(conv_direct_kernel<T>, blocks((int64_t)a.N * a.P * a.Q * a.K), block, 0, st, a);
            break;
        case K_DWCONV: {
            if (a.vec == VMAX) {
                const int64_t th = (int64_t)a.N * a.P * a.Q * (a.C / VMAX);
                const int rows = dwconv_band_rows(a);
                if constexpr (sizeof(T) == 2) {
                    if (rows > 1) {
                        const int bands = (a.P + rows - 1) / rows;
                        const int64_t tb = (int64_t)a.N * bands * a.Q * (a.C / VMAX);
                        if (a.sh == 1) MT_LAUNCH((dwconv3_rows_kernel<T, 1>), (dwconv3_rows_pair_kernel<T, 1>), blocks(tb), block, st, a, mate, rows, bands);
                        else MT_LAUNCH((dwconv3_rows_kernel<T, 2>), (dwconv3_rows_pair_kernel<T, 2>), blocks(tb), block, st, a, mate, rows, bands);
                        break;
                    }
                }
                if (a.R == 3 && a.S == 3)
                    MT_LAUNCH((dwconv_fixed_kernel<T, VMAX, 3>), (dwconv_fixed_pair_kernel<T, VMAX, 3>), blocks(th), block, st, a, mate);
                else
                    MT_LAUNCH((dwconv_kernel<T, VMAX>), (dwconv_pair_kernel<T, VMAX>), blocks(th), block, st, a, mate);
            } else {
                hipLaunchKernelGGL((dwconv_kernel<T, 1>), blocks((int64_t)a.N * a.P * a.Q * a.C), block, 0, st, a);
            }
            break;
        }
        case K_MAXPOOL:
        case K_AVGPOOL: {
            const bool mx = a.kernel_id == K_MAXPOOL;
            if (a.vec == VMAX) {
                const int64_t th = (int64_t)a.N * a.P * a.Q * (a.C / VMAX);
                if (mx && a.R == 2 && a.S == 2)
                    MT_LAUNCH((pool_fixed_kernel<T, VMAX, true, 2>), (pool_fixed_pair_kernel<T, VMAX, true, 2>), blocks(th), block, st, a, mate);
                else if (mx && a.R == 3 && a.S == 3)
                    MT_LAUNCH((pool_fixed_kernel<T, VMAX, true, 3>), (pool_fixed_pair_kernel<T, VMAX, true, 3>), blocks(th), block, st, a, mate);
                else if (!mx && a.R == 3 && a.S == 3)
                    MT_LAUNCH((pool_fixed_kernel<T, VMAX, false, 3>), (pool_fixed_pair_kernel<T, VMAX, false, 3>), blocks(th), block, st, a, mate);
                else if (mx)
                    MT_LAUNCH((pool_kernel<T, VMAX, true>), (pool_pair_kernel<T, VMAX, true>), blocks(th), block, st, a, mate);
                else
                    MT_LAUNCH((pool_kernel<T, VMAX, false>), (pool_pair_kernel<T, VMAX, false>), blocks(th), block, st, a, mate);
            } else {
                const int64_t th = (int64_t)a.N * a.P * a.Q * a.C;
                if (mx)
                    hipLaunchKernelGGL((pool_kernel<T, 1, true>), blocks(th), block, 0, st, a);
                else
                    hipLaunchKernelGGL((pool_kernel<T, 1, false>), blocks(th), block, 0, st, a);
            }
            break;
        }
        case K_GAP: {
            const int V = a.vec == VMAX ? VMAX : 1;
            const int CV = a.C / V;
            int lanes_c = 1;
            while (lanes_c < 4 && lanes_c < CV) lanes_c <<= 1;     // at least 16 spatial slices per wave
            const int groups = (CV + lanes_c - 1) / lanes_c;
            const int64_t th = (int64_t)a.N * groups * 64;
            if (V == VMAX)
                MT_LAUNCH((gap_kernel<T, VMAX>), (gap_pair_kernel<T, VMAX>), blocks(th), block, st, a, mate, lanes_c);
            else
                hipLaunchKernelGGL((gap_kernel<T, 1>), blocks(th), block, 0, st, a, lanes_c);
            break;
        }
        case K_LRN:
        case K_ADD: {
            const bool lrn = a.kernel_id == K_LRN;
            bool done = false;
            if constexpr (VMAX >= 8) {          // the vector form of the normalisation needs the window inside one neighbour vector
                if (a.vec == VMAX) {
                    const int64_t th = (int64_t)a.N * a.P * a.Q * (a.C / VMAX);
                    if (lrn) MT_LAUNCH((lrn_kernel<T, VMAX>), (lrn_pair_kernel<T, VMAX>), blocks(th), block, st, a, mate);
                    else MT_LAUNCH((add_kernel<T, VMAX>), (add_pair_kernel<T, VMAX>), blocks(th), block, st, a, mate);
                    done = true;
                }
            }
            if (!done) {
                const int64_t th = (int64_t)a.N * a.P * a.Q * a.C;
                if (lrn) hipLaunchKernelGGL((lrn_kernel<T, 1>), blocks(th), block, 0, st, a);
                else hipLaunchKernelGGL((add_kernel<T, 1>), blocks(th), block, 0, st, a);
            }
            break;
        }
        default:
            return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

int launch_direct(const OpArgs &a, void *stream, const OpArgs *mate, int n_mates) {
    if (mate && (n_mates < 1 || n_mates >= COISSUE_MAX)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (mate && !coissue_supported(a)) return (int)hipErrorInvalidValue;
    switch (a.dtype) {
        case MT_F32: return launch_typed<float>(a, st, mate, n_mates);
        case MT_F16: return launch_typed<f16>(a, st, mate, n_mates);
        case MT_BF16: return launch_typed<bf16>(a, st, mate, n_mates);
    }
    return (int)hipErrorInvalidValue;
}

int launch_probe(uint32_t *out, int n_groups, void *stream) {
    hipLaunchKernelGGL(probe_kernel, dim3((unsigned)n_groups), dim3(64), 0, (hipStream_t)stream, out);
    return (int)hipGetLastError();
}

int launch_arrive(uint32_t *counter, void *stream) {
    hipLaunchKernelGGL(arrive_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, counter);
    return (int)hipGetLastError();
}

int launch_fill_u32(uint32_t *p, size_t n, uint32_t v, void *stream) {
    if (n == 0) return 0;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, p, n, v);
    return (int)hipGetLastError();
}

}  // namespace mt
