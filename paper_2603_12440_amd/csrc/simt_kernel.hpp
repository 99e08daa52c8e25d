// General LDS-tiled GEMM on the vector ALUs, true fp32 multiply-add.
//
// This is the kernel for fp32 operands (whose products must not be narrowed to
// a matrix-core input type) and for every dtype / layout / leading-dimension
// combination the MFMA and skinny kernels do not take.  Each workgroup of 256
// lanes owns a TM x TN block of C; A and B slabs of TK columns are converted to
// fp32 and staged through LDS, and each lane keeps an RM x RN register block.
// In the paper's taxonomy (Sec. 3.2) this is d_mem = 3 (local memory tiling +
// register blocking), d_sync = 1 (workgroup barriers).
#pragma once

#include "common.hpp"

namespace mi355gemm {

struct SimtArgs {
  const void* A; const void* B; void* C; const float* bias;
  int64_t M, N, K;
  int64_t a_si, a_sk;          // element strides of A along i and k
  int64_t b_sk, b_sj;          // element strides of B along k and j
  int64_t c_si, c_sj;          // element strides of C along i and j
  int64_t stride_a, stride_b, stride_c, stride_bias;  // batch strides
  int has_bias, act;
  float scale;                 // scalar of the *_scale activations
};

template <typename TIn, typename TOut, int TM, int TN, int TK>
__global__ __launch_bounds__(256) void simt_gemm_kernel(SimtArgs p) {
  static_assert((TM * TK) % 256 == 0 && (TN * TK) % 256 == 0, "slab must divide over 256 lanes");
  constexpr int RM = TM / 16, RN = TN / 16;      // register block per lane
  constexpr int PAD = 4;
  __shared__ float As[TK][TM + PAD];
  __shared__ float Bs[TK][TN + PAD];

  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int64_t i0 = (int64_t)blockIdx.y * TM;
  const int64_t j0 = (int64_t)blockIdx.x * TN;
  const int64_t b = blockIdx.z;
  const TIn* A = (const TIn*)p.A + b * p.stride_a;
  const TIn* B = (const TIn*)p.B + b * p.stride_b;
  TOut* C = (TOut*)p.C + b * p.stride_c;

  float acc[RM][RN];
#pragma unroll
  for (int r = 0; r < RM; ++r)
#pragma unroll
    for (int c = 0; c < RN; ++c) acc[r][c] = 0.0f;

  // Lanes run along whichever index is contiguous in memory.
  const bool a_k_fast = (p.a_sk == 1);
  const bool b_k_fast = (p.b_sk == 1);

  // The next slab's global loads are issued before the current slab is multiplied
  // (registers as the second buffer), so that their latency overlaps the arithmetic.
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
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[RM], w[RN];
#pragma unroll
      for (int r = 0; r < RM; ++r) a[r] = As[k][ty * RM + r];
#pragma unroll
      for (int c = 0; c < RN; ++c) w[c] = Bs[k][tx * RN + c];
#pragma unroll
      for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int c = 0; c < RN; ++c) acc[r][c] = fmaf(a[r], w[c], acc[r][c]);
    }
    __syncthreads();
  }

  const float* bias = p.has_bias ? p.bias + b * p.stride_bias : nullptr;
#pragma unroll
  for (int r = 0; r < RM; ++r) {
    const int64_t i = i0 + ty * RM + r;
    if (i >= p.M) continue;
#pragma unroll
    for (int c = 0; c < RN; ++c) {
      const int64_t j = j0 + tx * RN + c;
      if (j >= p.N) continue;
      float t = acc[r][c];
      if (bias) t += bias[j];
      C[i * p.c_si + j * p.c_sj] = from_float<TOut>(apply_activation(p.act, t, p.scale));
    }
  }
}

}  // namespace mi355gemm
