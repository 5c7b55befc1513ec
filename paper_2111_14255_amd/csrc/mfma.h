// Matrix-core instruction wrappers shared by the convolution kernels (gfx950: v_mfma_f32_32x32x16 and 16x16x32 on
// fp16 / bf16 operands, fp32 accumulators).  A lane feeds 8 consecutive reduction elements of one operand row:
// row = lane % MF, elements 8 * (lane / MF) .. + 7.  With MF = 32 a lane's 16 accumulators are rows
// 8 * g + 4 * (lane / 32) + 0..3 (g = 0..3) of column lane % 32; with MF = 16 its 4 accumulators are rows
// 4 * (lane / 16) + 0..3 of column lane % 16.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_types.h"

namespace mt {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte register chunk

template <typename T, int MF>
struct Mma;
template <>
struct Mma<f16, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<bf16, 32> {
    typedef f32x16 Acc;
    static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<f16, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <>
struct Mma<bf16, 16> {
    typedef f32x4 Acc;
    static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

}  // namespace mt
