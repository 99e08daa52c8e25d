// Second pass of a split-K product: C = act(sum over the K slices of the fp32 partial
// products + bias), rounded once to C's storage type.  In the paper's taxonomy (Sec. 3.2)
// split-K is d_sync = 3 (global coordination: a multi-pass product with a synchronisation
// between the passes, here the kernel boundary).  The slices are added in a fixed order
// (slice 0 first), so the result does not depend on which workgroup finished first.
//
// Streaming kernel: every lane takes 4 consecutive columns of one row (16-byte loads from
// each slice, eight slices requested at a time), a workgroup 1024 consecutive elements of the
// row-major partials.
#pragma once

#include "common.hpp"

namespace mi355gemm {

struct SplitKReduceArgs {
  const float* ws;             // [splits][M][N] fp32, packed
  void* C; const float* bias;
  int64_t M, N;
  int64_t c_si, c_sj;          // element strides of C along i and j
  int splits;
  int has_bias, act;
  float scale;
};

template <typename TOut>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(SplitKReduceArgs p) {
  const int64_t quads_per_row = (p.N + 3) / 4;
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= p.M * quads_per_row) return;
  const int64_t i = q / quads_per_row;
  const int64_t j = (q - i * quads_per_row) * 4;
  const int64_t slice = p.M * p.N;
  const float* src = p.ws + i * p.N + j;
  float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const bool full = (j + 3 < p.N) && (p.N % 4 == 0);       // whole, 16-byte aligned quad
  if (full) {
    // eight slices' loads in flight at a time, added in slice order
    int s = 0;
    for (; s + 8 <= p.splits; s += 8) {
      f32x4_t w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) w[u] = __builtin_nontemporal_load((const f32x4_t*)(src + (s + u) * slice));
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += w[u][e];
    }
    for (; s < p.splits; ++s) {
      const f32x4_t w = __builtin_nontemporal_load((const f32x4_t*)(src + s * slice));
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += w[e];
    }
  } else {
    for (int s = 0; s < p.splits; ++s) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < p.N) v[e] += src[s * slice + e];
    }
  }
  TOut* C = (TOut*)p.C;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (j + e >= p.N) break;
    float t = v[e];
    if (p.has_bias) t += p.bias[j + e];
    C[i * p.c_si + (j + e) * p.c_sj] = from_float<TOut>(apply_activation(p.act, t, p.scale));
  }
}

}  // namespace mi355gemm
