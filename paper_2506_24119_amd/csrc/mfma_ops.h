// MFMA operand helpers shared by the projection kernels.
#pragma once
#include "spiral_internal.h"

namespace spiral {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// bf16 pair -> half pair: widen each to fp32 (a shift), convert (exact for normal-range values)
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
    const float lo = __uint_as_float(w << 16);
    const float hi = __uint_as_float(w & 0xFFFF0000u);
    typedef __attribute__((ext_vector_type(2))) __fp16 f16x2;
    f16x2 h = __builtin_amdgcn_cvt_pkrtz(lo, hi);
    return __builtin_bit_cast(uint32_t, h);
}

// convert a weight fragment once, then reuse it for every batch tile
__device__ __forceinline__ u32x4 prep_w(const u32x4& w) {
    u32x4 wh;
    wh.x = bf16x2_to_f16x2(w.x); wh.y = bf16x2_to_f16x2(w.y);
    wh.z = bf16x2_to_f16x2(w.z); wh.w = bf16x2_to_f16x2(w.w);
    return wh;
}
__device__ __forceinline__ f32x4 mma_prepped(const u32x4& w, const u32x4& a, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, a), c, 0, 0, 0);
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

}  // namespace spiral
