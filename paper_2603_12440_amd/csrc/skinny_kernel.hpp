// Skinny products (M <= 16, decode-shaped): y[m,n] = sum_k x[m,k] * W[n,k].
//
// The weight matrix W (N x K, K contiguous) is read exactly once from HBM and
// nothing else matters: each wavefront owns RPW rows of W at a time, every lane
// streams 16-byte pieces of those rows, multiplies them with the matching
// pieces of the (tiny, cache-resident) x rows with packed dot products (fp32
// accumulate) on the vector ALUs, and
// the 64 partial sums are combined with DPP lane rotations.  No matrix cores,
// no workgroup barriers.  Paper taxonomy (Sec. 3.2): d_mem = 1 (coalesced,
// vectorised loads), d_sync = 2 (sub-group reductions).
#pragma once

#include "common.hpp"

namespace mi355gemm {

struct SkinnyArgs {
  const void* X; const void* W; void* Y; const float* bias;
  int M, N, K;
  int64_t ldx, ldw, ldy;                                // elements
  int64_t stride_x, stride_w, stride_y, stride_bias;    // elements between batches
  int has_bias, act, y_f32;
};

// Sum over the 64 lanes of a wavefront; every lane gets the total.
template <int CTRL> __device__ __forceinline__ float dpp_rot(float v) {
  int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
  return __builtin_bit_cast(float, r);
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_rot<0x128>(v);   // row_ror:8  (rotation inside each row of 16 lanes)
  v += dpp_rot<0x124>(v);   // row_ror:4
  v += dpp_rot<0x122>(v);   // row_ror:2
  v += dpp_rot<0x121>(v);   // row_ror:1
  const int b = __builtin_bit_cast(int, v);
  float s = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  s += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  s += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  s += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return s;
}

// acc + dot product of two 16-byte pieces (8 packed 16-bit values each), with the
// packed dot-product instructions (v_dot2c_f32_bf16 / v_dot2c_f32_f16): products
// of two 16-bit values are exact in fp32, the sums are rounded in fp32.
template <typename T> __device__ __forceinline__ float dot8(const u32x4_t& x, const u32x4_t& w, float acc);
template <> __device__ __forceinline__ float dot8<bf16_t>(const u32x4_t& x, const u32x4_t& w, float acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t xi = x[i], wi = w[i];   // scalars first: bit_cast of a vector element lvalue is unreliable
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, xi),
                                          __builtin_bit_cast(bf16x2_t, wi), acc, false);
  }
  return acc;
}
template <> __device__ __forceinline__ float dot8<f16_t>(const u32x4_t& x, const u32x4_t& w, float acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t xi = x[i], wi = w[i];
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, xi),
                                 __builtin_bit_cast(f16x2_t, wi), acc, false);
  }
  return acc;
}

// MB = number of x rows handled (M rounded up; rows past M are clamped for the
// loads and skipped at the store).  RPW = rows of W a wavefront carries at once.
template <typename T, int MB, int RPW, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void skinny_gemm_kernel(SkinnyArgs p) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t batch = blockIdx.y;
  const T* X = (const T*)p.X + batch * p.stride_x;
  const T* W = (const T*)p.W + batch * p.stride_w;
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;

  const int n_groups = (p.N + RPW - 1) / RPW;
  const int stride_groups = gridDim.x * WAVES;

  const T* xrow[MB];
#pragma unroll
  for (int m = 0; m < MB; ++m) xrow[m] = X + (int64_t)min(m, p.M - 1) * p.ldx;

  for (int g = blockIdx.x * WAVES + wave; g < n_groups; g += stride_groups) {
    const int n0 = g * RPW;
    const T* wrow[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) wrow[r] = W + (int64_t)min(n0 + r, p.N - 1) * p.ldw;

    float acc[MB][RPW];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
      for (int r = 0; r < RPW; ++r) acc[m][r] = 0.0f;

    // Each lane walks K in steps of 64 pieces (512 elements): lane l takes piece l.
#pragma unroll 2
    for (int k = lane * 8; k < p.K; k += 512) {
      u32x4_t wv[RPW];
#pragma unroll
      for (int r = 0; r < RPW; ++r)
        wv[r] = __builtin_nontemporal_load((const u32x4_t*)(wrow[r] + k));
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        const u32x4_t xv = *(const u32x4_t*)(xrow[m] + k);
#pragma unroll
        for (int r = 0; r < RPW; ++r) acc[m][r] = dot8<T>(xv, wv[r], acc[m][r]);
      }
    }

#pragma unroll
    for (int m = 0; m < MB; ++m) {
#pragma unroll
      for (int r = 0; r < RPW; ++r) {
        float t = wave_sum(acc[m][r]);
        const int n = n0 + r;
        if (lane == 0 && m < p.M && n < p.N) {
          if (bias) t += bias[n];
          t = apply_activation(p.act, t);
          const int64_t o = batch * p.stride_y + (int64_t)m * p.ldy + n;
          if (p.y_f32) ((float*)p.Y)[o] = t;
          else ((T*)p.Y)[o] = from_float<T>(t);
        }
      }
    }
  }
}

}  // namespace mi355gemm
