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
  float scale;                 // scalar of the *_scale activations
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
  constexpr int DEPTH = 2;                       // rows a wave keeps requested (more gains nothing)
  // One or two x rows live in registers (each lane keeps the pieces it multiplies
  // with); more rows are staged in LDS and re-read for every row of W.  Two rows of x plus
  // the two rows of W in flight are 256 registers: too many at two waves per SIMD, where a
  // wave has 256 in all.
  constexpr bool kXInRegs = MB == 1 || (MB == 2 && WAVES <= 4);
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
      v = apply_activation(p.act, v, p.scale);
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
    // The common case: all of K in one pass.  A wave keeps DEPTH rows requested: a
    // row's registers are refilled with the row DEPTH steps on as soon as it has been
    // multiplied.
    u32x4_t w[DEPTH][P];
    float t[MB];
    int n = first;
    if (!kXInRegs) stage_x(0);                // x loads go out ahead of the W stream, so
                                              // waiting for them does not wait for W
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
      if (n + d * step < p.N) load_row(w[d], n + d * step, 0);
    if (kXInRegs) stage_x(0); else __syncthreads();
    bool more = n < p.N;
    while (more) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        if (more) {
          dot_row(w[d], t);
          store_row(t, n);
          if (n + DEPTH * step < p.N) load_row(w[d], n + DEPTH * step, 0);
          n += step;
          more = n < p.N;
        }
      }
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
              const float v = apply_activation(p.act, t[e] + bv, p.scale);
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


// ---- M up to 16, weights through wave-private LDS rings -----------------------------------
// The 16x16x32 variant above reads 64 bytes of 16 different rows per load instruction; the
// memory system prefers whole 128-byte lines.  Here a workgroup owns 32 rows of W, its four
// waves split K into contiguous quarters, and every wave runs its own ring of NSTAGE slabs
// (32 rows x 64 columns of W, and the matching 64 columns of up to 16 x rows) filled by
// direct-to-LDS loads that move full lines, 8 rows per instruction.  The ring is private to
// the wave, so the K loop needs no workgroup barrier, only vmcnt waits.  Products by
// v_mfma_f32_32x32x16 (x rows past M are clamped copies and never stored); the four partial
// 32x32 blocks are added through LDS at the end.
typedef float f32x16acc_t __attribute__((ext_vector_type(16)));
template <typename T> struct Mfma32;
template <> struct Mfma32<bf16_t> {
  static __device__ __forceinline__ f32x16acc_t run(const u32x4_t& a, const u32x4_t& b, f32x16acc_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};
template <> struct Mfma32<f16_t> {
  static __device__ __forceinline__ f32x16acc_t run(const u32x4_t& a, const u32x4_t& b, f32x16acc_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};

template <typename T, int NSTAGE>
__global__ __launch_bounds__(256) void skinny_ring_kernel(SkinnyArgs p) {
  constexpr int kSlab = 6144;                          // bytes per stage: W 32 x 128 B, then x 16 x 128 B
  constexpr int kLoads = 6;                            // direct-to-LDS loads per slab and wave
  typedef __attribute__((address_space(3))) unsigned char lds_uchar;
  static_assert(4 * NSTAGE * kSlab >= 4 * 16 * 64 * 4, "the rings double as the reduction buffer");
  __shared__ __attribute__((aligned(1024))) unsigned char ring[4 * NSTAGE * kSlab];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t batch = blockIdx.y;
  const T* X = (const T*)p.X + batch * p.stride_x;
  const T* W = (const T*)p.W + batch * p.stride_w;
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;
  const int n0 = blockIdx.x * 32;

  // slab row r, 16-byte chunk c lives at chunk slot c ^ swz(r) of its 128-byte row
  auto swz = [](int r) { return (r & 7) ^ ((r >> 3) & 3); };
  // loads: instruction q covers slab rows 8q .. 8q+7; lane l writes row 8q + l/8, slot l%8
  uint32_t w_off[4], x_off[2];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = q * 8 + lane / 8;
    const int c = (lane % 8) ^ swz(r);
    w_off[q] = (uint32_t)(((int64_t)min(n0 + r, p.N - 1) - n0) * p.ldw * 2 + c * 16);
    if (q < 2) x_off[q] = (uint32_t)((int64_t)min(r, p.M - 1) * p.ldx * 2 + c * 16);
  }
  const char* Wb = (const char*)(W + (int64_t)n0 * p.ldw);
  const char* Xb = (const char*)X;
  unsigned char* my_ring = ring + wave * (NSTAGE * kSlab);
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(lds_uchar*)my_ring;

  auto issue_slab = [&](int s, int stage) {            // full slab s (64 columns from 64 s)
    const char* gw = Wb + (int64_t)s * 128;
    const char* gx = Xb + (int64_t)s * 128;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(ring_lds + stage * kSlab + q * 1024), "v"(w_off[q]), "s"(gw) : "memory", "m0");
#pragma unroll
    for (int q = 0; q < 2; ++q)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(ring_lds + stage * kSlab + 4096 + q * 1024), "v"(x_off[q]), "s"(gx) : "memory", "m0");
  };

  // fragments: MFMA 32x32x16 operand lane l = row l%32, k-octet l/32
  const int fr = lane & 31, fh = lane >> 5;
  // (x has 16 rows in LDS: the upper half of the x operand repeats them; those outputs are dropped)
  uint32_t rd[4], rdx[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    rd[kk] = fr * 128 + (((kk * 2 + fh) ^ swz(fr)) * 16);
    rdx[kk] = (fr & 15) * 128 + (((kk * 2 + fh) ^ swz(fr & 15)) * 16);
  }

  f32x16acc_t acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

  auto multiply = [&](int stage, int ksteps) {
    const unsigned char* s = my_ring + stage * kSlab;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk < ksteps) {
        const u32x4_t wf = *(const u32x4_t*)(s + rd[kk]);
        const u32x4_t xf = *(const u32x4_t*)(s + 4096 + rdx[kk]);
        acc = Mfma32<T>::run(xf, wf, acc);             // D[x row][W row]
      }
    }
  };

  const int s_full = p.K / 64;                         // full slabs, split over the four waves
  const int per_wave = (s_full + 3) / 4;
  const int s_begin = min(wave * per_wave, s_full);
  const int s_end = min(s_full, s_begin + per_wave);
  if (s_begin < s_end) {
#pragma unroll
    for (int i = 0; i < NSTAGE - 1; ++i) issue_slab(min(s_begin + i, s_end - 1), i);
    int stage = 0;
    for (int s = s_begin; s < s_end; ++s) {
      // slab s has landed when at most the NSTAGE-2 slabs issued after it are outstanding
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * kLoads) : "memory");
      // refill the stage the previous iteration multiplied from (its reads have been
      // consumed by MFMAs already issued); past the end, re-load the last slab: same count
      issue_slab(min(s + NSTAGE - 1, s_end - 1), stage == 0 ? NSTAGE - 1 : stage - 1);
      multiply(stage, 4);
      stage = stage + 1 == NSTAGE ? 0 : stage + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  if (wave == 3 && s_full * 64 < p.K) {
    // K tail: zero-filled slab through registers into stage 0 of this wave's ring
    const int k0 = s_full * 64, kvalid = p.K - k0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = q * 8 + lane / 8;
      const int c = (lane % 8) ^ swz(r);
      u32x4_t wv = {0u, 0u, 0u, 0u}, xv = {0u, 0u, 0u, 0u};
      if (c * 8 < kvalid) {
        wv = *(const u32x4_t*)(Wb + (int64_t)s_full * 128 + w_off[q]);
        if (q < 2) xv = *(const u32x4_t*)(Xb + (int64_t)s_full * 128 + x_off[q]);
      }
      *(u32x4_t*)(my_ring + q * 1024 + lane * 16) = wv;
      if (q < 2) *(u32x4_t*)(my_ring + 4096 + q * 1024 + lane * 16) = xv;
    }
    multiply(0, (kvalid + 15) / 16);
  }

  // add the four K quarters (the rings are free now), then bias, activation, store
  __syncthreads();
  float* red = (float*)ring;                           // [4 waves][16 regs][64 lanes]
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[r];
  __syncthreads();
  // wave w finishes accumulator registers 4w .. 4w+3: x rows 8w + 4*(lane/32) + e, column lane%32
  // (waves 2 and 3 hold only the repeated rows 16 .. 31 and store nothing)
  const int n = n0 + fr;
  const float bv = (bias && n < p.N) ? bias[n] : 0.0f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int r = wave * 4 + e;
    const float t = red[(0 * 16 + r) * 64 + lane] + red[(1 * 16 + r) * 64 + lane] +
                    red[(2 * 16 + r) * 64 + lane] + red[(3 * 16 + r) * 64 + lane];
    const int m = 8 * wave + 4 * fh + e;
    if (m < p.M && n < p.N) {
      const float v = apply_activation(p.act, t + bv, p.scale);
      const int64_t o = batch * p.stride_y + (int64_t)m * p.ldy + n;
      if (p.y_f32) ((float*)p.Y)[o] = v;
      else ((T*)p.Y)[o] = from_float<T>(v);
    }
  }
}

// ---- M up to 16, W staged through registers ------------------------------------------
// Same division of work as the ring kernel (a workgroup owns 32 rows of W, its four or
// eight waves split K into equal parts, one 32x32x16 MFMA tile per wave, the parts added
// at the end; eight waves = two per SIMD stream faster when there is one workgroup per CU), but W and x travel global -> registers -> LDS: plain 16-byte loads in which 16
// (or 32) lanes cover 256 (512) contiguous bytes of a row, DEPTH slabs requested ahead,
// then ds_write_b128 into one wave-private, swizzled LDS slab from which the MFMA
// fragments are read back.  For a stream that comes from HBM this moves more bytes per
// microsecond than direct-to-LDS loads do.
template <typename T, int DEPTH, int RB, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void skinny_stage_kernel(SkinnyArgs p) {
  constexpr int kRowBytes = RB;                        // RB/2 columns per slab: 256 or 512 bytes of each row
  constexpr int kCols = RB / 2;
  constexpr int kWBytes = 32 * kRowBytes, kXBytes = 16 * kRowBytes;
  constexpr int kLPR = RB / 16, kRPI = 64 / kLPR;      // lanes per row, rows per load instruction
  constexpr int kWLoads = 32 / kRPI, kXLoads = 16 / kRPI;   // 16-byte loads per lane and slab
  constexpr int kSteps = kCols / 16;                   // MFMAs per slab
  static_assert(WAVES == 4 || WAVES == 8, "K is split over four or eight waves");
  static_assert(kWBytes + kXBytes >= 16 * 64 * 4, "the slabs double as the reduction buffer");
  __shared__ __attribute__((aligned(1024))) unsigned char slabs[WAVES * (kWBytes + kXBytes)];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t batch = blockIdx.y;
  const T* X = (const T*)p.X + batch * p.stride_x;
  const T* W = (const T*)p.W + batch * p.stride_w;
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;
  const int n0 = blockIdx.x * 32;

  // Load q of a slab: kLPR lanes cover one row's piece, lane l takes its 16-byte chunk
  // l % kLPR of slab row kRPI q + l / kLPR.  In LDS the chunk sits at slot (chunk ^ row%16)
  // of its row, for W and x alike (16 slots of 16 bytes span all banks).
  const int lr = lane / kLPR, lc = lane % kLPR;
  const char* w_src[kWLoads];
  const char* x_src[kXLoads];
  uint32_t w_dst[kWLoads], x_dst[kXLoads];
#pragma unroll
  for (int q = 0; q < kWLoads; ++q) {
    const int r = kRPI * q + lr;
    w_src[q] = (const char*)(W + (int64_t)min(n0 + r, p.N - 1) * p.ldw) + lc * 16;
    w_dst[q] = r * kRowBytes + ((lc ^ (r & 15)) * 16);
    if (q < kXLoads) {
      x_src[q] = (const char*)(X + (int64_t)min(r, p.M - 1) * p.ldx) + lc * 16;
      x_dst[q] = kWBytes + r * kRowBytes + ((lc ^ (r & 15)) * 16);
    }
  }
  unsigned char* mine = slabs + wave * (kWBytes + kXBytes);

  u32x4_t wv[DEPTH][kWLoads], xv[DEPTH][kXLoads];
  // columns [kCols s, kCols s + kCols), all of them inside K
  auto load_slab = [&](u32x4_t (&w)[kWLoads], u32x4_t (&x)[kXLoads], int s) {
    const int64_t off = (int64_t)s * kRowBytes;
#pragma unroll
    for (int q = 0; q < kWLoads; ++q) w[q] = __builtin_nontemporal_load((const u32x4_t*)(w_src[q] + off));
#pragma unroll
    for (int q = 0; q < kXLoads; ++q) x[q] = *(const u32x4_t*)(x_src[q] + off);
  };
  auto write_slab = [&](const u32x4_t (&w)[kWLoads], const u32x4_t (&x)[kXLoads]) {
#pragma unroll
    for (int q = 0; q < kWLoads; ++q) *(u32x4_t*)(mine + w_dst[q]) = w[q];
#pragma unroll
    for (int q = 0; q < kXLoads; ++q) *(u32x4_t*)(mine + x_dst[q]) = x[q];
  };

  // fragments: MFMA 32x32x16 operand lane l = row l%32, k-octet l/32
  // (x has 16 rows in LDS: the upper half of the x operand repeats them; those outputs are dropped)
  const int fr = lane & 31, fh = lane >> 5;
  f32x16acc_t acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  auto multiply = [&]() {
#pragma unroll
    for (int k0 = 0; k0 < kSteps; k0 += 8) {
      u32x4_t wf[8], xf[8];                            // eight steps' reads first, then their MFMAs
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const int slot = (((k0 + kk) * 2 + fh) ^ (fr & 15)) * 16;
        wf[kk] = *(const u32x4_t*)(mine + fr * kRowBytes + slot);
        xf[kk] = *(const u32x4_t*)(mine + kWBytes + (fr & 15) * kRowBytes + slot);
      }
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) acc = Mfma32<T>::run(xf[kk], wf[kk], acc);   // D[x row][W row]
    }
  };

  const int s_full = p.K / kCols;                        // full slabs, split over the waves
  const int per_wave = (s_full + WAVES - 1) / WAVES;
  const int s_begin = min(wave * per_wave, s_full);
  const int s_end = min(s_full, s_begin + per_wave);
  int s = s_begin;
  if (s_end - s_begin >= 2 * DEPTH) {
    // Steady state: every refill is in range, so all loads are unconditional and the
    // wait for a slab leaves the DEPTH-1 younger ones in flight.  (The scheduling
    // barriers keep the next slab's LDS writes, and with them the wait for its loads,
    // behind this slab's MFMAs.)
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load_slab(wv[d], xv[d], s_begin + d);
    for (; s + 2 * DEPTH <= s_end; s += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        write_slab(wv[d], xv[d]);
        load_slab(wv[d], xv[d], s + d + DEPTH);
        multiply();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  } else {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
      if (s_begin + d < s_end) load_slab(wv[d], xv[d], s_begin + d);
  }
  // the last one or two rounds: registers d hold slab s + d (where that is below s_end)
  for (; s < s_end; s += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      if (s + d < s_end) {
        write_slab(wv[d], xv[d]);
        if (s + d + DEPTH < s_end) load_slab(wv[d], xv[d], s + d + DEPTH);
        multiply();
      }
    }
  }
  if (wave == WAVES - 1 && s_full * kCols < p.K) {
    // K tail: chunks past K are written as zeros
    const bool live = s_full * kCols + lc * 8 < p.K;
    const int64_t off = (int64_t)s_full * kRowBytes;
#pragma unroll
    for (int q = 0; q < kWLoads; ++q) {
      wv[0][q] = u32x4_t{0u, 0u, 0u, 0u};
      if (live) wv[0][q] = *(const u32x4_t*)(w_src[q] + off);
    }
#pragma unroll
    for (int q = 0; q < kXLoads; ++q) {
      xv[0][q] = u32x4_t{0u, 0u, 0u, 0u};
      if (live) xv[0][q] = *(const u32x4_t*)(x_src[q] + off);
    }
    write_slab(wv[0], xv[0]);
    multiply();
  }

  // add the four K quarters (the slabs are free now), then bias, activation, store
  __syncthreads();
  float* red = (float*)slabs;                          // [WAVES][16 regs][64 lanes]
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[r];
  __syncthreads();
  // each wave finishes 16 / WAVES accumulator registers; register r of lane l is x row
  // 8*(r/4) + 4*(l/32) + r%4, column l%32 (rows 16 .. 31 repeat rows 0 .. 15 and are dropped)
  const int n = n0 + fr;
  const float bv = (bias && n < p.N) ? bias[n] : 0.0f;
  constexpr int kPerWave = 16 / WAVES;
#pragma unroll
  for (int e = 0; e < kPerWave; ++e) {
    const int r = wave * kPerWave + e;
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) t += red[(w * 16 + r) * 64 + lane];
    const int m = 8 * (r / 4) + 4 * fh + r % 4;
    if (m < p.M && n < p.N) {
      const float v = apply_activation(p.act, t + bv, p.scale);
      const int64_t o = batch * p.stride_y + (int64_t)m * p.ldy + n;
      if (p.y_f32) ((float*)p.Y)[o] = v;
      else ((T*)p.Y)[o] = from_float<T>(v);
    }
  }
}

}  // namespace mi355gemm
