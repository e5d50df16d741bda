// Storage types of node matrices: float32, or bfloat16 kept as its 16-bit pattern.  Arithmetic is always float32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gad {

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_float(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }

// round to nearest, ties to even; NaN stays a (quiet) NaN.  One instruction on gfx950 (v_cvt_pk_bf16_f32).
__device__ __forceinline__ bf16_t float_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_float(v); }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return float_to_bf16(v); }

// V consecutive elements starting at p (p aligned to 16 bytes when V * sizeof(T) == 16) -> float
template <int V, typename T>
__device__ __forceinline__ void load_row_piece(const T* p, float (&r)[V]) {
  if constexpr (sizeof(T) == 4 && V == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    r[0] = t.x; r[1] = t.y; r[2] = t.z; r[3] = t.w;
  } else if constexpr (sizeof(T) == 2 && V == 8) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    r[0] = __uint_as_float(t.x << 16); r[1] = __uint_as_float(t.x & 0xffff0000u);
    r[2] = __uint_as_float(t.y << 16); r[3] = __uint_as_float(t.y & 0xffff0000u);
    r[4] = __uint_as_float(t.z << 16); r[5] = __uint_as_float(t.z & 0xffff0000u);
    r[6] = __uint_as_float(t.w << 16); r[7] = __uint_as_float(t.w & 0xffff0000u);
  } else {
#pragma unroll
    for (int k = 0; k < V; ++k) r[k] = to_f32<T>(p[k]);
  }
}

// sigma(v) and sigma'(.) * v for sigma = ReLU (slope 0) or LeakyReLU (Eq. 7's activation); `on` = pre-activation > 0.
__device__ __forceinline__ float leaky(float v, bool on, float slope) {
  return on ? v : (slope == 0.f ? 0.f : slope * v);
}

}  // namespace gad
