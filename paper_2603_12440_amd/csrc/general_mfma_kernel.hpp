// General LDS-tiled GEMM on the matrix cores with true fp32 products:
// v_mfma_f32_32x32x2_f32 multiplies fp32 operands exactly and accumulates in fp32, so it
// serves the same problems as the vector-ALU general kernel (fp32 operands; any dtype,
// layout and leading dimension through element strides) at up to twice its arithmetic
// rate.  Staging is the general kernel's: slabs of TK columns converted to fp32 and
// written to LDS k-major, the next slab's global loads in flight during the arithmetic.
// Four waves (2 x 2) own a TM x TN block of C, each a (TM/2) x (TN/2) sub-block of
// 32x32 MFMA tiles.  Paper taxonomy (Sec. 3.2): d_mem = 3, d_sync = 1.
#pragma once

#include "common.hpp"
#include "simt_kernel.hpp"

namespace mi355gemm {

template <typename TIn, typename TOut, int TM, int TN, int TK>
__global__ __launch_bounds__(256) void general_mfma_kernel(SimtArgs p) {
  static_assert((TM * TK) % 256 == 0 && (TN * TK) % 256 == 0, "slab must divide over 256 lanes");
  static_assert(TM % 64 == 0 && TN % 64 == 0 && TK % 2 == 0, "2 x 2 waves of 32x32 tiles, two columns of K per MFMA");
  constexpr int MT = TM / 64, NT = TN / 64;      // 32x32 tiles per wave
  constexpr int PAD = 4;
  __shared__ float As[TK][TM + PAD];
  __shared__ float Bs[TK][TN + PAD];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int fr = lane & 31, fh = lane >> 5;
  const int64_t i0 = (int64_t)blockIdx.y * TM;
  const int64_t j0 = (int64_t)blockIdx.x * TN;
  const int64_t b = blockIdx.z;
  const TIn* A = (const TIn*)p.A + b * p.stride_a;
  const TIn* B = (const TIn*)p.B + b * p.stride_b;
  TOut* C = (TOut*)p.C + b * p.stride_c;

  f32x16_t acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;

  // Lanes run along whichever index is contiguous in memory.
  const bool a_k_fast = (p.a_sk == 1);
  const bool b_k_fast = (p.b_sk == 1);
  constexpr int A_PER = TM * TK / 256, B_PER = TN * TK / 256;
  float ra[A_PER], rb[B_PER];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int u = 0; u < A_PER; ++u) {
      const int e = tid + u * 256;
      int i, k;
      if (a_k_fast) { i = e / TK; k = e % TK; } else { k = e / TM; i = e % TM; }
      ra[u] = 0.0f;
      if (i0 + i < p.M && k0 + k < p.K)
        ra[u] = to_float<TIn>(A[(i0 + i) * p.a_si + (k0 + k) * p.a_sk]);
    }
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      const int e = tid + u * 256;
      int j, k;
      if (b_k_fast) { j = e / TK; k = e % TK; } else { k = e / TN; j = e % TN; }
      rb[u] = 0.0f;
      if (j0 + j < p.N && k0 + k < p.K)
        rb[u] = to_float<TIn>(B[(k0 + k) * p.b_sk + (j0 + j) * p.b_sj]);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int u = 0; u < A_PER; ++u) {
      const int e = tid + u * 256;
      int i, k;
      if (a_k_fast) { i = e / TK; k = e % TK; } else { k = e / TM; i = e % TM; }
      As[k][i] = ra[u];
    }
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      const int e = tid + u * 256;
      int j, k;
      if (b_k_fast) { j = e / TK; k = e % TK; } else { k = e / TN; j = e % TN; }
      Bs[k][j] = rb[u];
    }
  };

  fetch(0);
  for (int64_t k0 = 0; k0 < p.K; k0 += TK) {
    stash();
    __syncthreads();
    if (k0 + TK < p.K) fetch(k0 + TK);
    // MFMA 32x32x2 operand: lane l holds row (column) l % 32 at k = l / 32.  Columns past K
    // were staged as zeros.  Operands go in swapped (B first) so that a lane ends up with one
    // row of C and runs of 4 consecutive columns.
#pragma unroll
    for (int k = 0; k < TK; k += 2) {
      float a[MT], w[NT];
#pragma unroll
      for (int m = 0; m < MT; ++m) a[m] = As[k + fh][wm * (TM / 2) + m * 32 + fr];
#pragma unroll
      for (int n = 0; n < NT; ++n) w[n] = Bs[k + fh][wn * (TN / 2) + n * 32 + fr];
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(w[n], a[m], acc[m][n], 0, 0, 0);
    }
    __syncthreads();
  }

  // register r of lane l: row l % 32, column 8 (r / 4) + 4 (l / 32) + r % 4 of the 32x32 tile
  const float* bias = p.has_bias ? p.bias + b * p.stride_bias : nullptr;
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int64_t i = i0 + wm * (TM / 2) + m * 32 + fr;
    if (i >= p.M) continue;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t j = j0 + wn * (TN / 2) + n * 32 + 8 * (r / 4) + 4 * fh + r % 4;
        if (j >= p.N) continue;
        float t = acc[m][n][r];
        if (bias) t += bias[j];
        C[i * p.c_si + j * p.c_sj] = from_float<TOut>(apply_activation(p.act, t, p.scale));
      }
    }
  }
}

}  // namespace mi355gemm
