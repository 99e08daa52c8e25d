// fp32 GEMM on the matrix cores for operands that can be moved in 16-byte pieces:
// v_mfma_f32_32x32x2_f32 (exact fp32 products, fp32 accumulation), 128x128 (or 64x64) tiles, slabs of 32
// columns of K, two LDS buffers and one barrier per slab.  The general kernel next to it takes any
// element strides at 4 bytes per load and a barrier pair per 16 columns; this one needs the
// contiguous index of each operand to run in whole, 16-byte aligned float4 groups (the host checks
// leading dimensions and extents when it builds the plan and the pointers at launch, and falls back
// to the general kernel otherwise).  Paper taxonomy (Sec. 3.2): d_mem = 3, d_sync = 1.
//
// Layout in LDS follows the operand's layout in memory, so that both the global loads and the
// LDS writes are 16 bytes per lane:
//   * K contiguous ("k-fast", row-major A / column-major B): [row][32 + 4] floats.  An MFMA takes
//     two columns of K, one from each half of the wave; which two is free as long as A and B agree,
//     so lane l multiplies columns 16 (l / 32) + s in step s and reads its 16 values of a slab as
//     four 16-byte pieces;
//   * K strided (column-major A / row-major B): [k][tile rows + 4] floats, one 4-byte read per step.
#pragma once

#include "common.hpp"
#include "simt_kernel.hpp"

namespace mi355gemm {

constexpr int kF32TileK = 32;

template <bool KFAST, int ROWS_> struct F32Stage {
  static constexpr int ROWS = ROWS_, TK = kF32TileK;
  static constexpr int LD = KFAST ? TK + 4 : ROWS + 4;          // floats per LDS row
  static constexpr int SIZE = KFAST ? ROWS * LD : TK * LD;      // floats per buffer
};

template <bool A_KFAST, bool B_KFAST, int TM, int TN>
__global__ __launch_bounds__(256) void f32_mfma_kernel(SimtArgs p) {
  static_assert(TM % 64 == 0 && TN % 64 == 0, "2 x 2 waves of 32x32 tiles");
  constexpr int TK = kF32TileK;
  constexpr int MT = TM / 64, NT = TN / 64;                      // 32x32 tiles per wave
  using SA = F32Stage<A_KFAST, TM>;
  using SB = F32Stage<B_KFAST, TN>;
  __shared__ __attribute__((aligned(16))) float As[2 * SA::SIZE];
  __shared__ __attribute__((aligned(16))) float Bs[2 * SB::SIZE];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int fr = lane & 31, fh = lane >> 5;
  const int64_t i0 = (int64_t)blockIdx.y * TM;
  const int64_t j0 = (int64_t)blockIdx.x * TN;
  const int64_t b = blockIdx.z;
  const float* A = (const float*)p.A + b * p.stride_a;
  const float* B = (const float*)p.B + b * p.stride_b;
  float* C = (float*)p.C + b * p.stride_c;
  const int64_t lda = A_KFAST ? p.a_si : p.a_sk;                 // the strided index of each operand
  const int64_t ldb = B_KFAST ? p.b_sj : p.b_sk;

  f32x16_t acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;

  // A slab of an operand is ROWS x 32 / 4 float4 groups: ROWS / 32 per lane.  Groups outside the matrix
  // read as zeros (extents along the contiguous index are multiples of 4: a group is never split).
  f32x4_t ra[TM / 32], rb[TN / 32];
  auto fetch_one = [&](auto kfast_c, auto rows_c, const float* X, int64_t ld, int64_t r0, int64_t R, int64_t k0,
                       f32x4_t (&v)[decltype(rows_c)::value / 32]) {
    constexpr bool kfast = decltype(kfast_c)::value;
    constexpr int ROWS = decltype(rows_c)::value;
#pragma unroll
    for (int u = 0; u < ROWS / 32; ++u) {
      const int e = tid + u * 256;
      // (unconditional loads: a group outside the matrix is read from the matrix's first group
      // instead and replaced by zeros, so that no load waits for a branch)
      bool in;
      const float* src;
      if constexpr (kfast) {
        const int row = e >> 3, c4 = e & 7;
        in = r0 + row < R && k0 + 4 * c4 < p.K;
        src = X + (in ? (r0 + row) * ld + k0 + 4 * c4 : 0);
      } else {
        const int k = e / (ROWS / 4), c4 = e % (ROWS / 4);
        in = k0 + k < p.K && r0 + 4 * c4 < R;
        src = X + (in ? (k0 + k) * ld + r0 + 4 * c4 : 0);
      }
      const f32x4_t t = *(const f32x4_t*)src;
      v[u] = in ? t : f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
  };
  auto stash_one = [&](auto kfast_c, auto rows_c, float* S, const f32x4_t (&v)[decltype(rows_c)::value / 32]) {
    constexpr bool kfast = decltype(kfast_c)::value;
    constexpr int ROWS = decltype(rows_c)::value;
    constexpr int LD = F32Stage<kfast, ROWS>::LD;
#pragma unroll
    for (int u = 0; u < ROWS / 32; ++u) {
      const int e = tid + u * 256;
      if constexpr (kfast) *(f32x4_t*)(S + (e >> 3) * LD + 4 * (e & 7)) = v[u];
      else *(f32x4_t*)(S + (e / (ROWS / 4)) * LD + 4 * (e % (ROWS / 4))) = v[u];
    }
  };
  // the 16 values lane l multiplies in one slab, for the 32 rows (columns) from r0 on
  auto operand = [&](auto kfast_c, auto rows_c, const float* S, int r0, float (&x)[16]) {
    constexpr bool kfast = decltype(kfast_c)::value;
    constexpr int LD = F32Stage<kfast, decltype(rows_c)::value>::LD;
    if constexpr (kfast) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4_t t = *(const f32x4_t*)(S + (r0 + fr) * LD + fh * 16 + 4 * j);
        x[4 * j] = t[0]; x[4 * j + 1] = t[1]; x[4 * j + 2] = t[2]; x[4 * j + 3] = t[3];
      }
    } else {
#pragma unroll
      for (int s = 0; s < 16; ++s) x[s] = S[(fh * 16 + s) * LD + r0 + fr];
    }
  };
  using a_fast = std::integral_constant<bool, A_KFAST>;
  using b_fast = std::integral_constant<bool, B_KFAST>;
  using a_rows = std::integral_constant<int, TM>;
  using b_rows = std::integral_constant<int, TN>;

  const int64_t slabs = (p.K + TK - 1) / TK;
  fetch_one(a_fast(), a_rows(), A, lda, i0, p.M, 0, ra);
  fetch_one(b_fast(), b_rows(), B, ldb, j0, p.N, 0, rb);
  stash_one(a_fast(), a_rows(), As, ra);
  stash_one(b_fast(), b_rows(), Bs, rb);
  __syncthreads();
  int buf = 0;
  for (int64_t t = 0; t < slabs; ++t) {
    const bool more = t + 1 < slabs;
    if (more) {
      fetch_one(a_fast(), a_rows(), A, lda, i0, p.M, (t + 1) * TK, ra);
      fetch_one(b_fast(), b_rows(), B, ldb, j0, p.N, (t + 1) * TK, rb);
    }
    float a[MT][16], w[NT][16];
#pragma unroll
    for (int m = 0; m < MT; ++m) operand(a_fast(), a_rows(), As + buf * SA::SIZE, wm * (TM / 2) + m * 32, a[m]);
#pragma unroll
    for (int n = 0; n < NT; ++n) operand(b_fast(), b_rows(), Bs + buf * SB::SIZE, wn * (TN / 2) + n * 32, w[n]);
#pragma unroll
    for (int s = 0; s < 16; ++s)
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m][s], w[n][s], acc[m][n], 0, 0, 0);
    if (more) {
      stash_one(a_fast(), a_rows(), As + (buf ^ 1) * SA::SIZE, ra);
      stash_one(b_fast(), b_rows(), Bs + (buf ^ 1) * SB::SIZE, rb);
    }
    __syncthreads();
    buf ^= 1;
  }

  // register r of lane l: row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32 of the 32x32 tile:
  // a store instruction writes 128 contiguous bytes of two rows of a row-major C
  const float* bias = p.has_bias ? p.bias + b * p.stride_bias : nullptr;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int64_t j = j0 + wn * (TN / 2) + n * 32 + fr;
    if (j >= p.N) continue;
    const float bj = bias ? bias[j] : 0.0f;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t i = i0 + wm * (TM / 2) + m * 32 + 8 * (r / 4) + 4 * fh + r % 4;
        if (i >= p.M) continue;
        C[i * p.c_si + j * p.c_sj] = apply_activation(p.act, acc[m][n][r] + bj, p.scale);
      }
    }
  }
}

// ---- small fp32 problems: a 16x16 tile of C per workgroup, K split over its four waves ----------
// A problem with a few hundred 32x32 tiles leaves most of the chip idle and each tile's K loop runs
// as one long dependent chain.  Here a workgroup owns a 16x16 tile (256 workgroups for 256^3), its
// waves take 64 columns each of every 256 columns of K, operands go from global memory straight
// into v_mfma_f32_16x16x4_f32 operand registers (no LDS staging, no barrier in the K loop), and the
// four partial tiles are added through LDS at the end.  An MFMA takes four columns of K, one from
// each quarter of the wave; lane l multiplies columns 16 (l / 16) + s of its wave's 64 in step s
// (A and B agree on that), so a K-contiguous operand is four 16-byte loads per lane.
// vec_a / vec_b: that operand is K contiguous and can be read in aligned float4 groups (K % 4 == 0,
// leading dimension and batch stride multiples of 4, pointer 16-byte aligned); any other operand
// is read element by element through its strides.  Paper taxonomy (Sec. 3.2): d_mem = 1, d_sync = 2.
struct F32SmallArgs {
  SimtArgs g;
  int vec_a, vec_b;
};

// (VEC_A / VEC_B at compile time, one straight-line body each.  Loads are unconditional: a value
// outside the matrix is read from a valid address of the same row instead and replaced by zero
// afterwards, so that all of a chunk's loads are in flight together.)
template <bool VEC_A, bool VEC_B>
__device__ __forceinline__ void f32_small_body(const SimtArgs& p, float (*red)[4][64]) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int fr = lane & 15, fg = lane >> 4;
  const int64_t i0 = (int64_t)blockIdx.y * 16, j0 = (int64_t)blockIdx.x * 16;
  const int64_t b = blockIdx.z;
  const float* A = (const float*)p.A + b * p.stride_a;
  const float* B = (const float*)p.B + b * p.stride_b;
  float* C = (float*)p.C + b * p.stride_c;
  const int64_t i = i0 + fr, j = j0 + fr;               // this lane's row of A and column of B
  const bool row_ok = i < p.M, col_ok = j < p.N;
  const float* a_row = A + (row_ok ? i : 0) * p.a_si;
  const float* b_col = B + (col_ok ? j : 0) * p.b_sj;

  // the 16 values of one operand this lane multiplies in the chunk whose first column is k
  auto fetch = [&](auto vec_c, const float* base, int64_t sk, bool ok, int64_t k, float (&x)[16]) {
    if constexpr (decltype(vec_c)::value) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool in = ok && k + 4 * c < p.K;
        const f32x4_t t = *(const f32x4_t*)(base + (in ? k + 4 * c : 0));
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * c + e] = in ? t[e] : 0.0f;
      }
    } else {
#pragma unroll
      for (int s = 0; s < 16; ++s) {
        const bool in = ok && k + s < p.K;
        const float t = base[(in ? k + s : 0) * sk];
        x[s] = in ? t : 0.0f;
      }
    }
  };
  using va = std::integral_constant<bool, VEC_A>;
  using vb = std::integral_constant<bool, VEC_B>;

  f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float a0[16], b0[16], a1[16], b1[16];
  const int64_t kl = wave * 64 + fg * 16;               // this lane's first column within a chunk of 256
  fetch(va(), a_row, p.a_sk, row_ok, kl, a0);
  fetch(vb(), b_col, p.b_sk, col_ok, kl, b0);
  for (int64_t k0 = 0; k0 < p.K; k0 += 512) {           // two chunks per round: the next one's loads
    fetch(va(), a_row, p.a_sk, row_ok, k0 + 256 + kl, a1);   // are on their way during the MFMAs
    fetch(vb(), b_col, p.b_sk, col_ok, k0 + 256 + kl, b1);
#pragma unroll
    for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[s], b0[s], acc, 0, 0, 0);
    fetch(va(), a_row, p.a_sk, row_ok, k0 + 512 + kl, a0);
    fetch(vb(), b_col, p.b_sk, col_ok, k0 + 512 + kl, b0);
#pragma unroll
    for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[s], b1[s], acc, 0, 0, 0);
  }

  // register r of lane l: row 4 (l / 16) + r, column l % 16.  Wave w adds and stores register w.
#pragma unroll
  for (int r = 0; r < 4; ++r) red[wave][r][lane] = acc[r];
  __syncthreads();
  const float t = red[0][wave][lane] + red[1][wave][lane] + red[2][wave][lane] + red[3][wave][lane];
  const int64_t ci = i0 + 4 * fg + wave;
  if (ci < p.M && col_ok) {
    const float bj = p.has_bias ? (p.bias + b * p.stride_bias)[j] : 0.0f;
    C[ci * p.c_si + j * p.c_sj] = apply_activation(p.act, t + bj, p.scale);
  }
}

__global__ __launch_bounds__(256) void f32_small_kernel(F32SmallArgs q) {
  __shared__ float red[4][4][64];
  if (q.vec_a && q.vec_b) f32_small_body<true, true>(q.g, red);
  else if (q.vec_a) f32_small_body<true, false>(q.g, red);
  else if (q.vec_b) f32_small_body<false, true>(q.g, red);
  else f32_small_body<false, false>(q.g, red);
}

}  // namespace mi355gemm
