// Storage types and conversions used by every kernel (device side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mt {

typedef _Float16 f16;
struct bf16 {
    uint16_t v;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16 v) { return (float)v; }
__device__ __forceinline__ float to_f32(bf16 v) { return __uint_as_float(((uint32_t)v.v) << 16); }

__device__ __forceinline__ void from_f32(float f, float &o) { o = f; }
__device__ __forceinline__ void from_f32(float f, f16 &o) { o = (f16)f; }   // v_cvt_f16_f32: nearest even
__device__ __forceinline__ void from_f32(float f, bf16 &o) {
    o.v = __builtin_bit_cast(uint16_t, (__bf16)f);      // v_cvt_pk_bf16_f32: nearest even, NaN stays NaN
}

// Activation as a clamp to [lo, hi]: none = [-inf, inf], ReLU = [0, inf], ReLU6 = [0, 6]; the bounds depend only on
// the kernel argument, so the per-value cost is one v_med3_f32.
__device__ __forceinline__ float apply_act(float v, int act) {
    const float lo = act == MT_ACT_NONE ? -__builtin_inff() : 0.f;
    const float hi = act == MT_ACT_RELU6 ? 6.f : __builtin_inff();
    return __builtin_amdgcn_fmed3f(v, lo, hi);
}

// Issue priority of the calling wave among the waves of its SIMD (0 lowest, 3 highest); the instruction takes an
// immediate, hence the ladder.  Changes timing only, never results.
__device__ __forceinline__ void set_wave_priority(int p) {
    if (p == 1) __builtin_amdgcn_s_setprio(1);
    else if (p == 2) __builtin_amdgcn_s_setprio(2);
    else if (p == 3) __builtin_amdgcn_s_setprio(3);
}

// Launches K1 with the operator's arguments, or, when `mate` points to n_mates (1 .. 3) further operators of equal
// launch shape, K2 (the several-operator form of the same kernel) on a grid of 1 + n_mates times the workgroups,
// blockIdx.y naming the operator.
#define MT_LAUNCH(K1, K2, grid, block, st, a, mate, ...)                                    \
    do {                                                                                    \
        if (mate) {                                                                         \
            OpArgsPair pair_;                                                               \
            pair_.a[0] = (a);                                                               \
            for (int i_ = 0; i_ < n_mates; ++i_) pair_.a[1 + i_] = (mate)[i_];              \
            dim3 grid2_ = (grid);                                                           \
            grid2_.y = 1 + n_mates;                                                         \
            hipLaunchKernelGGL(K2, grid2_, block, 0, st, pair_ __VA_OPT__(, ) __VA_ARGS__); \
        } else {                                                                            \
            hipLaunchKernelGGL(K1, grid, block, 0, st, a __VA_OPT__(, ) __VA_ARGS__);       \
        }                                                                                   \
    } while (0)

// V consecutive elements of T moved as one access when V*sizeof(T) is 4, 8 or 16 bytes.
template <typename T, int V>
struct alignas(sizeof(T) * V) Pack {
    T e[V];
};

template <typename T, int V>
__device__ __forceinline__ void load_pack(const T *p, float (&out)[V]) {
    Pack<T, V> t = *reinterpret_cast<const Pack<T, V> *>(p);
#pragma unroll
    for (int i = 0; i < V; ++i) out[i] = to_f32(t.e[i]);
}

template <typename T, int V>
__device__ __forceinline__ void store_pack(T *p, const float (&in)[V]) {
    Pack<T, V> t;
#pragma unroll
    for (int i = 0; i < V; ++i) from_f32(in[i], t.e[i]);
    *reinterpret_cast<Pack<T, V> *>(p) = t;
}

}  // namespace mt
