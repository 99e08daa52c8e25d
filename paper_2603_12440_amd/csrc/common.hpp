// Shared device-side helpers for the gfx950 GEMM kernels: storage types,
// conversions and the fused epilogue (bias + activation, computed in fp32 on
// the accumulators: in the taxonomy of Sec. 3.2 of the paper, operator fusion with one
// pass over the data).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mi355gemm {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;
// 8-bit floating point, OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 significand bits;
// no infinities, S.1111.111 is NaN, largest finite value 448): storage only, the matrix
// cores multiply it directly.
struct f8e4m3_t { unsigned char bits; };

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
  kEpiBiasGeluTanh = 4, kEpiRelu = 5, kEpiGeluErf = 6,
  kEpiBiasSwishScale = 7, kEpiBiasSigmoidScaleResidual = 8,
  kEpiSwishScale = 9, kEpiSigmoidScaleResidual = 10
};

__host__ __device__ inline bool epilogue_has_bias(int e) {
  return (e >= kEpiBias && e <= kEpiBiasGeluTanh) || e == kEpiBiasSwishScale ||
         e == kEpiBiasSigmoidScaleResidual;
}
__host__ __device__ inline bool epilogue_has_scale(int e) {
  return e >= kEpiBiasSwishScale && e <= kEpiSigmoidScaleResidual;
}

// Activation kinds after the bias has been folded away.
enum : int {
  kActNone = 0, kActRelu = 1, kActGeluErf = 2, kActGeluTanh = 3,
  kActSwishScale = 4, kActSigmoidScaleResidual = 5
};

__host__ __device__ inline int epilogue_activation(int e) {
  switch (e) {
    case kEpiBiasRelu: case kEpiRelu: return kActRelu;
    case kEpiBiasGeluErf: case kEpiGeluErf: return kActGeluErf;
    case kEpiBiasGeluTanh: return kActGeluTanh;
    case kEpiBiasSwishScale: case kEpiSwishScale: return kActSwishScale;
    case kEpiBiasSigmoidScaleResidual: case kEpiSigmoidScaleResidual: return kActSigmoidScaleResidual;
    default: return kActNone;
  }
}

// GELU in fp32 with a handful of instructions (the epilogue runs on every output
// element while the matrix cores idle, so it has to be short).
//
// erf form: erf(|x|) = 1 - (a1 s + ... + a5 s^5) exp(-x^2), s = 1/(1 + p|x|), the
// five-term rational approximation of Abramowitz & Stegun (7.1.26), |error| <= 1.5e-7,
// evaluated with the hardware reciprocal and exp2.  For negative arguments
// 1 + erf(x) is formed as the tail itself, so nothing cancels.
__device__ __forceinline__ float gelu_erf_f32(float t) {
  const float x = t * 0.70710678118654752440f;
  const float ax = fabsf(x);
  const float s = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float poly = fmaf(s, 1.061405429f, -1.453152027f);
  poly = fmaf(s, poly, 1.421413741f);
  poly = fmaf(s, poly, -0.284496736f);
  poly = fmaf(s, poly, 0.254829592f);
  poly *= s;
  const float tail = poly * __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);  // 1 - erf(|x|)
  const float one_plus_erf = x < 0.0f ? tail : 2.0f - tail;
  return 0.5f * t * one_plus_erf;
}
// tanh form: 1 + tanh(u) = 2 e / (e + 1) with e = exp(2u)  (no cancellation for u < 0).
__device__ __forceinline__ float gelu_tanh_f32(float t) {
  const float u = 0.79788456080286535588f * fmaf(0.044715f * t, t * t, t);
  const float e = __builtin_amdgcn_exp2f(fminf(2.0f * 1.4426950408889634f * u, 126.0f));
  const float one_plus_tanh = 2.0f * e * __builtin_amdgcn_rcpf(e + 1.0f);
  return 0.5f * t * one_plus_tanh;
}

// sigma(t) = 1 / (1 + exp(-t)) with the hardware exp2 and reciprocal.  exp2 overflows to
// +inf for t below about -88, whose reciprocal is the correct limit 0.
__device__ __forceinline__ float sigmoid_f32(float t) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * t));
}
// The post-ops of two of the paper's tasks: matmul followed by Swish and a scaling, GEMM followed by
// sigmoid, scaling and a residual add (App. "Per-task results"); c is the descriptor's scale.
__device__ __forceinline__ float swish_scale_f32(float t, float c) { return c * (t * sigmoid_f32(t)); }
__device__ __forceinline__ float sigmoid_scale_residual_f32(float t, float c) {
  return fmaf(c, sigmoid_f32(t), t);
}

// act(t) in fp32.  `act` and `scale` are uniform over the launch.
__device__ __forceinline__ float apply_activation(int act, float t, float scale) {
  switch (act) {
    case kActRelu: return fmaxf(t, 0.0f);
    case kActGeluErf: return gelu_erf_f32(t);
    case kActGeluTanh: return gelu_tanh_f32(t);
    case kActSwishScale: return swish_scale_f32(t, scale);
    case kActSigmoidScaleResidual: return sigmoid_scale_residual_f32(t, scale);
    default: return t;
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
