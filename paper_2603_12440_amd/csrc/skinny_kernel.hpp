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
  // Register i of a row holds piece (i + rot) % P, rot different from wave to wave: rows of W are a
  // power of two apart in most problems, and waves that all read the same columns of their rows at
  // the same time would crowd the few memory channels those addresses share.
  static_assert((P & (P - 1)) == 0, "pieces per pass: a power of two");
  const int rot = first & (P - 1);
  auto piece = [&](int i) { return ((i + rot) & (P - 1)) * 512 + lane * 8; };   // first column of register i

  // One row's current piece: P loads of 16 bytes per lane, all in flight together.
  // Pieces past the end of K read as zero.
  auto load_row = [&](u32x4_t (&wv)[P], int n, int k0) {
    const T* row = W + (int64_t)n * p.ldw + k0;
#pragma unroll
    for (int i = 0; i < P; ++i) {
      wv[i] = u32x4_t{0u, 0u, 0u, 0u};
      if (k0 + piece(i) < p.K)
        wv[i] = __builtin_nontemporal_load((const u32x4_t*)(row + piece(i)));
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
          const u32x4_t xv = *(const u32x4_t*)(xs + (m * kSkinnyKC + piece(i)) * 2);
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
          if (m < p.M && k0 + piece(i) < p.K)
            xr[m][i] = *(const u32x4_t*)(X + (int64_t)m * p.ldx + k0 + piece(i));
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


// ---- matrix-core products for M up to 16 -------------------------------------------------
// For more than a few x rows the vector ALUs (and the LDS re-reads of x) fall behind the HBM
// stream, so the products go to the matrix cores: operands are 8 consecutive k per lane.
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

// ---- M up to 16, W staged through registers ------------------------------------------
// A workgroup owns 32 rows of W, its four waves split K into equal contiguous parts, one
// 32x32x16 MFMA tile per wave (x rows past M are clamped copies and never stored), the parts
// added through LDS at the end.  W and x travel global -> registers -> LDS: plain 16-byte loads in
// which 16 (or 32) lanes cover 256 (512) contiguous bytes of a row, DEPTH slabs requested ahead,
// then ds_write_b128 into one wave-private, swizzled LDS slab from which the MFMA fragments are
// read back.  The slab is private to the wave, so the K loop needs no workgroup barrier.  For a
// stream that comes from HBM this moves more bytes per microsecond than direct-to-LDS loads do.
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

// ---- M up to 16: W staged through LDS, x fragments straight from L2 ------------------------
// As skinny_stage_kernel (a workgroup owns 32 rows of W, its waves split K into contiguous
// parts, every wave moves slabs of RB bytes per row global -> registers -> its own swizzled LDS
// slab -> MFMA fragments), with two changes that shorten everything around the stream:
//   * the products are v_mfma_f32_16x16x32 on (16 x rows) x (16 W rows), two W tiles per wave,
//     and the x operand is loaded from global memory directly in fragment layout (lane l: row
//     l % 16, k-octet l / 16; x is a few hundred KB and stays in L2): no LDS space, writes or
//     reads for x, a third less LDS traffic;
//   * with 16 KB (RB = 512) of LDS per wave instead of 24, eight waves fit a CU: two per SIMD,
//     each with two slabs requested ahead, i.e. 256 KB in flight per CU as in the M = 1 kernel.
// M <= 4 runs here as well (x rows past M repeat the last row, their results are dropped): the
// matrix cores do not care, and the vector-ALU kernel's tail of dot products is gone.
template <typename T, int DEPTH, int RB, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void skinny_direct_kernel(SkinnyArgs p) {
  constexpr int kRowBytes = RB;                        // RB/2 columns per slab: 256 or 512 bytes of each row
  constexpr int kCols = RB / 2;
  constexpr int kWBytes = 32 * kRowBytes;
  constexpr int kLPR = RB / 16, kRPI = 64 / kLPR;      // lanes per row, rows per load instruction
  constexpr int kWLoads = 32 / kRPI;                   // 16-byte W loads per lane and slab
  constexpr int kSteps = kCols / 32;                   // k-steps (MFMAs per W tile) per slab
  static_assert(WAVES == 4 || WAVES == 8, "K is split over four or eight waves");
  static_assert(kWBytes >= 8 * 64 * 4, "the slabs double as the reduction buffer");
  __shared__ __attribute__((aligned(1024))) unsigned char slabs[WAVES * kWBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t batch = blockIdx.y;
  const T* X = (const T*)p.X + batch * p.stride_x;
  const T* W = (const T*)p.W + batch * p.stride_w;
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;
  const int n0 = blockIdx.x * 32;

  // W load q of a slab: kLPR lanes cover one row's piece, lane l takes its 16-byte chunk l % kLPR
  // of slab row kRPI q + l / kLPR; in LDS the chunk sits at slot (chunk ^ row % 16) of its row.
  const int lr = lane / kLPR, lc = lane % kLPR;
  // (byte offsets from the panel's first row: 32 bits, the host checks that a panel spans less than 4 GB)
  const char* const w_base = (const char*)(W + (int64_t)n0 * p.ldw);
  // LDS slot: (chunk ^ row % 16), and row % 16 = (kRPI q) % 16 + l / kLPR (no carry), so the
  // lane's part of the xor is fixed and load q's part is a constant
  const int w_last_row = p.N - 1 - n0;                 // rows past N repeat the last one
  const uint32_t w_ld_bytes = (uint32_t)p.ldw * 2u, w_src_col = (uint32_t)lc * 16u;
  const uint32_t w_dst_row = lr * kRowBytes, w_dst_slot0 = (uint32_t)(lc ^ lr) * 16u;
  // x fragment of k-step kk of a slab: 16 bytes at column 32 kk + 8 (l / 16) of x row l % 16
  const int fr = lane & 15, fo = lane >> 4;
  const char* x_src = (const char*)(X + (int64_t)min(fr, p.M - 1) * p.ldx) + fo * 16;
  unsigned char* mine = slabs + wave * kWBytes;

  // DEPTH slabs of W are on their way at any time; the x fragments (L2 hits) of the next slab only:
  // they are requested after the current slab's products and before the refill of its W registers,
  // so waiting for them never waits for a younger W load.
  u32x4_t wv[DEPTH][kWLoads], xv[kSteps];
  // Full slabs are split over the waves in contiguous parts.  Every workgroup starts its parts at
  // a different slab and wraps around: the rows of W are a power of two apart in most problems, and
  // workgroups that all read the same columns of their rows at the same time would crowd the few
  // memory channels those addresses share.
  const int s_full = p.K / kCols;
  const int per_wave = (s_full + WAVES - 1) / WAVES;
  const int s_first = min(wave * per_wave, s_full);
  const int s_count = min(s_full, s_first + per_wave) - s_first;
  const int s_rot = s_count > 0 ? (int)(blockIdx.x % (unsigned)s_count) : 0;
  auto slab_of = [&](int j) {                          // the wave's j-th slab, 0 <= j < s_count
    const int r = j + s_rot;
    return s_first + (r >= s_count ? r - s_count : r);
  };
  const int s_begin = 0, s_end = s_count;
  auto w_src = [&](int q, int row_l) {
    return (uint32_t)min(kRPI * q + row_l, w_last_row) * w_ld_bytes + w_src_col;
  };
  auto load_w = [&](u32x4_t (&w)[kWLoads], int j) {
    const int64_t off = (int64_t)slab_of(j) * kRowBytes;
    int row_l = lr;
    asm volatile("" : "+v"(row_l));                    // the offsets are formed here, not kept in registers
#pragma unroll
    for (int q = 0; q < kWLoads; ++q) w[q] = __builtin_nontemporal_load((const u32x4_t*)(w_base + off + w_src(q, row_l)));
  };
  auto load_x = [&](u32x4_t (&x)[kSteps], int j) {
    const int64_t off = (int64_t)slab_of(j) * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < kSteps; ++kk) x[kk] = *(const u32x4_t*)(x_src + off + kk * 64);
  };
  auto write_slab = [&](const u32x4_t (&w)[kWLoads]) {
    uint32_t w_dst_slot = w_dst_slot0;
    asm volatile("" : "+v"(w_dst_slot));               // the addresses are formed here, not kept in registers
#pragma unroll
    for (int q = 0; q < kWLoads; ++q)
      *(u32x4_t*)(mine + w_dst_row + q * kRPI * kRowBytes + (w_dst_slot ^ (uint32_t)(((kRPI * q) & 15) * 16))) = w[q];
  };
  f32x4acc_t acc[2];
  acc[0] = acc[1] = f32x4acc_t{0.f, 0.f, 0.f, 0.f};
  auto multiply = [&](const u32x4_t (&x)[kSteps]) {
    constexpr int kGroup = 2;                          // a group's reads first, then its MFMAs
#pragma unroll
    for (int k0 = 0; k0 < kSteps; k0 += kGroup) {
      u32x4_t wf[2][kGroup];
#pragma unroll
      for (int kk = 0; kk < kGroup; ++kk)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          wf[t][kk] = *(const u32x4_t*)(mine + (t * 16 + fr) * kRowBytes + ((((k0 + kk) * 4 + fo) ^ fr) * 16));
#pragma unroll
      for (int kk = 0; kk < kGroup; ++kk)
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[t] = Mfma16<T>::run(x[k0 + kk], wf[t][kk], acc[t]);   // D[x row][W row]
    }
  };

  int s = s_begin;
  if (s_begin < s_end) load_w(wv[0], s_begin);
  if (s_begin < s_end) load_x(xv, s_begin);
#pragma unroll
  for (int d = 1; d < DEPTH; ++d)
    if (s_begin + d < s_end) load_w(wv[d], s_begin + d);
  // steady state: every refill is in range, all loads unconditional
  for (; s + 2 * DEPTH <= s_end; s += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      write_slab(wv[d]);
      multiply(xv);
      load_x(xv, s + d + 1);
      load_w(wv[d], s + d + DEPTH);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // the last rounds: registers d hold slab s + d (where that is below s_end)
  for (; s < s_end; s += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      if (s + d < s_end) {
        write_slab(wv[d]);
        multiply(xv);
        if (s + d + 1 < s_end) load_x(xv, s + d + 1);
        if (s + d + DEPTH < s_end) load_w(wv[d], s + d + DEPTH);
      }
    }
  }
  if (wave == WAVES - 1 && s_full * kCols < p.K) {
    // K tail: chunks past K count as zeros (K is a multiple of 8: chunks are never split)
    const int k0 = s_full * kCols;
    const int64_t off = (int64_t)s_full * kRowBytes;
#pragma unroll
    for (int q = 0; q < kWLoads; ++q) {
      wv[0][q] = u32x4_t{0u, 0u, 0u, 0u};
      if (k0 + lc * 8 < p.K) wv[0][q] = *(const u32x4_t*)(w_base + off + w_src(q, lr));
    }
#pragma unroll
    for (int kk = 0; kk < kSteps; ++kk) {
      xv[kk] = u32x4_t{0u, 0u, 0u, 0u};
      if (k0 + kk * 32 + fo * 8 < p.K) xv[kk] = *(const u32x4_t*)(x_src + off + kk * 64);
    }
    write_slab(wv[0]);
    multiply(xv);
  }

  // add the waves' parts of K (the slabs are free now), then bias, activation, store.
  // Register r of tile t in lane l: x row 4 (l / 16) + r, W row 16 t + l % 16.
  __syncthreads();
  float* red = (float*)slabs;                          // [WAVES][8 regs][64 lanes]
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[(wave * 8 + t * 4 + r) * 64 + lane] = acc[t][r];
  __syncthreads();
  constexpr int kPerWave = 8 / WAVES;
#pragma unroll
  for (int e = 0; e < kPerWave; ++e) {
    const int q = wave * kPerWave + e;                 // tile q / 4, register q % 4
    float sum = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) sum += red[(w * 8 + q) * 64 + lane];
    const int m = 4 * fo + q % 4;
    const int n = n0 + (q / 4) * 16 + fr;
    if (m < p.M && n < p.N) {
      const float v = apply_activation(p.act, sum + (bias ? bias[n] : 0.0f), p.scale);
      const int64_t o = batch * p.stride_y + (int64_t)m * p.ldy + n;
      if (p.y_f32) ((float*)p.Y)[o] = v;
      else ((T*)p.Y)[o] = from_float<T>(v);
    }
  }
}

}  // namespace mi355gemm
