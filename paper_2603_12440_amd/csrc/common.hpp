// Shared device-side helpers for the gfx950 GEMM kernels: storage types,
// conversions and the fused epilogue (bias + activation, computed in fp32 on
// the accumulators; Sec. 3.2 of the paper files this under "fused operations,
// single pass over data").
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mi355gemm {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// Epilogue codes: numerically equal to gemm_epilogue_t in the public header.
enum : int {
  kEpiNone = 0, kEpiBias = 1, kEpiBiasRelu = 2, kEpiBiasGeluErf = 3,
  kEpiBiasGeluTanh = 4, kEpiRelu = 5, kEpiGeluErf = 6
};

__host__ __device__ inline bool epilogue_has_bias(int e) {
  return e >= kEpiBias && e <= kEpiBiasGeluTanh;
}

// Activation kinds after the bias has been folded away.
enum : int { kActNone = 0, kActRelu = 1, kActGeluErf = 2, kActGeluTanh = 3 };

__host__ __device__ inline int epilogue_activation(int e) {
  switch (e) {
    case kEpiBiasRelu: case kEpiRelu: return kActRelu;
    case kEpiBiasGeluErf: case kEpiGeluErf: return kActGeluErf;
    case kEpiBiasGeluTanh: return kActGeluTanh;
    default: return kActNone;
  }
}

// act(t) in fp32.  `act` is uniform over the launch.
__device__ __forceinline__ float apply_activation(int act, float t) {
  switch (act) {
    case kActRelu:
      return fmaxf(t, 0.0f);
    case kActGeluErf:
      return 0.5f * t * (1.0f + erff(t * 0.70710678118654752440f));
    case kActGeluTanh: {
      float u = 0.79788456080286535588f * (t + 0.044715f * t * t * t);
      return 0.5f * t * (1.0f + tanhf(u));
    }
    default:
      return t;
  }
}

// Storage <-> fp32.  Narrowing is round-to-nearest-even (hardware converts).
template <typename T> __device__ __forceinline__ float to_float(T v);
template <> __device__ __forceinline__ float to_float<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_float<bf16_t>(bf16_t v) { return (float)v; }
template <> __device__ __forceinline__ float to_float<f16_t>(f16_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return (bf16_t)v; }
template <> __device__ __forceinline__ f16_t from_float<f16_t>(float v) { return (f16_t)v; }

// Two fp32 -> one packed 32-bit word of two 16-bit values (low half = a).
template <typename T> __device__ __forceinline__ uint32_t pack2(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2<bf16_t>(float a, float b) {
  f32x2_t v = {a, b};
  bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
  return __builtin_bit_cast(uint32_t, r);
}
template <> __device__ __forceinline__ uint32_t pack2<f16_t>(float a, float b) {
  f32x2_t v = {a, b};
  f16x2_t r = __builtin_convertvector(v, f16x2_t);
  return __builtin_bit_cast(uint32_t, r);
}

}  // namespace mi355gemm
