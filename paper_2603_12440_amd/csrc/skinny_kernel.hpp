// Skinny products (M <= 16, decode-shaped): y[m,n] = sum_k x[m,k] * W[n,k].
//
// The weight matrix W (N x K, K contiguous) is read exactly once from HBM and
// nothing else matters.  Each wavefront streams whole rows of W, one row at a
// time with every 16-byte load of the row's current 16 KB piece in flight at
// once (measured on MI355X: one row per wave with 16 loads outstanding per lane
// streams at the copy rate, four rows at once loses a third of it), and keeps
// the next row's loads in flight while it multiplies the current one.  One or two
// x rows stay in registers, more are staged per workgroup in LDS; the products use the packed
// dot-product instructions with fp32 accumulation on the vector ALUs, and the 64
// lane partials are combined with DPP lane rotations.  No matrix cores.  Paper
// taxonomy (Sec. 3.2): d_mem = 1 (coalesced, vectorised loads) with LDS reuse of
// x, d_sync = 2 (sub-group reductions).
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

constexpr int kSkinnyKC = 8192;                  // K elements handled per pass (x piece kept in LDS)
constexpr int kSkinnyPieces = kSkinnyKC / 512;   // 16-byte loads per lane per row and pass
constexpr int kSkinnyMaxRows = 32;               // rows one wave may own (the host sizes the grid for it)

// MB = number of x rows handled (M rounded up to 1, 2, 4 or 8).
template <typename T, int MB, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void skinny_gemm_kernel(SkinnyArgs p) {
  constexpr int P = kSkinnyPieces;
  // One or two x rows live in registers (each lane keeps the pieces it multiplies
  // with); more rows are staged in LDS and re-read for every row of W.
  constexpr bool kXInRegs = MB <= 2;
  __shared__ __attribute__((aligned(16))) unsigned char xs[kXInRegs ? 16 : MB * kSkinnyKC * 2];
  u32x4_t xr[kXInRegs ? MB : 1][P];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t batch = blockIdx.y;
  const T* X = (const T*)p.X + batch * p.stride_x;
  const T* W = (const T*)p.W + batch * p.stride_w;
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;

  const int first = blockIdx.x * WAVES + wave;          // this wave owns rows first, first + step, ...
  const int step = gridDim.x * WAVES;
  const int n_pass = (p.K + kSkinnyKC - 1) / kSkinnyKC;

  // One row's current piece: P loads of 16 bytes per lane, all in flight together.
  // Pieces past the end of K read as zero.
  auto load_row = [&](u32x4_t (&wv)[P], int n, int k0) {
    const T* row = W + (int64_t)n * p.ldw + k0 + lane * 8;
#pragma unroll
    for (int i = 0; i < P; ++i) {
      wv[i] = u32x4_t{0u, 0u, 0u, 0u};
      if (k0 + i * 512 + lane * 8 < p.K)
        wv[i] = __builtin_nontemporal_load((const u32x4_t*)(row + i * 512));
    }
  };
  // Dot products of the loaded piece with the staged x rows, reduced over the wave.
  auto dot_row = [&](const u32x4_t (&wv)[P], float (&t)[MB]) {
    float acc[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) acc[m] = 0.0f;
    if (!kXInRegs) asm volatile("" ::: "memory");   // re-read x from LDS, do not keep it in registers
#pragma unroll
    for (int i = 0; i < P; ++i) {
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        if constexpr (kXInRegs) {
          acc[m] = dot8<T>(xr[m][i], wv[i], acc[m]);
        } else {
          const u32x4_t xv = *(const u32x4_t*)(xs + (m * kSkinnyKC + i * 512 + lane * 8) * 2);
          acc[m] = dot8<T>(xv, wv[i], acc[m]);
        }
      }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) t[m] = wave_sum(acc[m]);
  };
  auto store_row = [&](const float (&t)[MB], int n) {
    if (lane != 0) return;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      if (m >= p.M) continue;
      float v = t[m];
      if (bias) v += bias[n];
      v = apply_activation(p.act, v);
      const int64_t o = batch * p.stride_y + (int64_t)m * p.ldy + n;
      if (p.y_f32) ((float*)p.Y)[o] = v;
      else ((T*)p.Y)[o] = from_float<T>(v);
    }
  };
  // Bring in the x piece [k0, k0 + KC) of every row (zero past K and past M): into
  // this lane's registers, or into LDS for the whole workgroup.
  auto stage_x = [&](int k0) {
    if constexpr (kXInRegs) {
#pragma unroll
      for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int i = 0; i < P; ++i) {
          xr[m][i] = u32x4_t{0u, 0u, 0u, 0u};
          if (m < p.M && k0 + i * 512 + lane * 8 < p.K)
            xr[m][i] = *(const u32x4_t*)(X + (int64_t)m * p.ldx + k0 + i * 512 + lane * 8);
        }
      return;
    }
    // all loads first (they are L2 hits and come back quickly), then the LDS writes
    constexpr int kPer = MB * (kSkinnyKC / 8) / (64 * WAVES);
    static_assert(MB * (kSkinnyKC / 8) % (64 * WAVES) == 0, "x piece must divide over the workgroup");
    u32x4_t v[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int e = tid + u * (64 * WAVES);
      const int m = e / (kSkinnyKC / 8), c = e % (kSkinnyKC / 8);
      v[u] = u32x4_t{0u, 0u, 0u, 0u};
      if (m < p.M && k0 + c * 8 < p.K) v[u] = *(const u32x4_t*)(X + (int64_t)m * p.ldx + k0 + c * 8);
    }
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int e = tid + u * (64 * WAVES);
      const int m = e / (kSkinnyKC / 8), c = e % (kSkinnyKC / 8);
      *(u32x4_t*)(xs + (m * kSkinnyKC + c * 8) * 2) = v[u];
    }
  };

  if (n_pass == 1) {
    // The common case: all of K in one pass.  Rows are double-buffered: the next
    // row's loads are issued before the current row is multiplied.
    u32x4_t w0[P], w1[P];
    float t[MB];
    int n = first;
    if (kXInRegs) {
      if (n < p.N) load_row(w0, n, 0);        // get the stream going before x arrives
      stage_x(0);
    } else {
      stage_x(0);                             // x loads are issued ahead of the W stream, so
      if (n < p.N) load_row(w0, n, 0);        // waiting for them does not wait for W
      __syncthreads();
    }
    while (n < p.N) {
      const int n1 = n + step;
      if (n1 < p.N) load_row(w1, n1, 0);
      dot_row(w0, t);
      store_row(t, n);
      if (n1 >= p.N) break;
      const int n2 = n1 + step;
      if (n2 < p.N) load_row(w0, n2, 0);
      dot_row(w1, t);
      store_row(t, n1);
      n = n2;
    }
  } else {
    // Long K: pass by pass over x pieces of KC elements; the partial sums of a wave's
    // rows wait in LDS between passes (slots are private to the wave: no barrier).
    __shared__ float part[WAVES][kSkinnyMaxRows][MB];
    for (int pass = 0; pass < n_pass; ++pass) {
      if (!kXInRegs) __syncthreads();          // nobody still reads the previous x piece
      stage_x(pass * kSkinnyKC);
      if (!kXInRegs) __syncthreads();
      int slot = 0;
      for (int n = first; n < p.N; n += step, ++slot) {
        u32x4_t w0[P];
        float t[MB];
        load_row(w0, n, pass * kSkinnyKC);
        dot_row(w0, t);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          if (pass > 0) t[m] += part[wave][slot][m];
          if (pass + 1 < n_pass && lane == 0) part[wave][slot][m] = t[m];
        }
        if (pass + 1 == n_pass) store_row(t, n);
      }
    }
  }
}


// ---- M up to 16 on the matrix cores --------------------------------------------------
// For more than a few x rows the vector ALUs (and the LDS re-reads of x) fall behind
// the HBM stream, so the products go to v_mfma_f32_16x16x32: a workgroup owns RB
// blocks of 16 rows of W, its four waves split K into contiguous quarters (so each
// wave streams 16 separate, but long, contiguous runs), x fragments come straight
// from global memory (x is small and stays in L2), and the four partial 16x16 results
// are added through LDS.  Still bound by the one pass over W, not by the MFMAs.
typedef float f32x4acc_t __attribute__((ext_vector_type(4)));
template <typename T> struct Mfma16;
template <> struct Mfma16<bf16_t> {
  static __device__ __forceinline__ f32x4acc_t run(const u32x4_t& a, const u32x4_t& b, f32x4acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};
template <> struct Mfma16<f16_t> {
  static __device__ __forceinline__ f32x4acc_t run(const u32x4_t& a, const u32x4_t& b, f32x4acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};

template <typename T, int RB, int UNROLL>
__global__ __launch_bounds__(256) void skinny_mfma_kernel(SkinnyArgs p) {
  __shared__ f32x4acc_t red[4][RB][64];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int col = lane & 15, oct = lane >> 4;         // MFMA operand: row/col lane%16, k-octet lane/16
  const int64_t batch = blockIdx.y;
  const T* X = (const T*)p.X + batch * p.stride_x;
  const T* W = (const T*)p.W + batch * p.stride_w;
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;

  const int steps = (p.K + 31) / 32;                  // MFMA k-steps over all of K
  const int per_wave = (steps + 3) / 4;
  const int s_begin = wave * per_wave;
  const int s_end = min(steps, s_begin + per_wave);
  const bool x_live = col < p.M;                      // x rows past M read as zero
  const T* xrow = X + (int64_t)min(col, p.M - 1) * p.ldx + oct * 8;

  const int n_blocks = (p.N + 16 * RB - 1) / (16 * RB);
  for (int blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
    const int n0 = blk * 16 * RB;
    const T* wrow[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) wrow[r] = W + (int64_t)min(n0 + r * 16 + col, p.N - 1) * p.ldw + oct * 8;

    f32x4acc_t acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = f32x4acc_t{0.f, 0.f, 0.f, 0.f};

    for (int s0 = s_begin; s0 < s_end; s0 += UNROLL) {
      u32x4_t wv[UNROLL][RB], xv[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const int k = (s0 + u) * 32;
        const bool live = (s0 + u < s_end) && (k + oct * 8 < p.K);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
          wv[u][r] = u32x4_t{0u, 0u, 0u, 0u};
          // (plain loads: the other half of each 128-byte line is wanted by the next step)
          if (live) wv[u][r] = *(const u32x4_t*)(wrow[r] + k);
        }
        xv[u] = u32x4_t{0u, 0u, 0u, 0u};
        if (live && x_live) xv[u] = *(const u32x4_t*)(xrow + k);
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = Mfma16<T>::run(xv[u], wv[u][r], acc[r]);
    }

    // add the four K quarters; lane l of the result holds rows m = 4*(l/16) + e, column l%16
    __syncthreads();                                  // previous block's reduction has been read
#pragma unroll
    for (int r = 0; r < RB; ++r) red[wave][r][lane] = acc[r];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        f32x4acc_t t = red[0][r][lane] + red[1][r][lane] + red[2][r][lane] + red[3][r][lane];
        const int n = n0 + r * 16 + col;
        if (n < p.N) {
          const float bv = bias ? bias[n] : 0.0f;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int m = oct * 4 + e;
            if (m < p.M) {
              const float v = apply_activation(p.act, t[e] + bv);
              const int64_t o = batch * p.stride_y + (int64_t)m * p.ldy + n;
              if (p.y_f32) ((float*)p.Y)[o] = v;
              else ((T*)p.Y)[o] = from_float<T>(v);
            }
          }
        }
      }
    }
  }
}

}  // namespace mi355gemm
