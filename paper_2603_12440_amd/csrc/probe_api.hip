// Measured peaks: an MFMA-only register loop and a streaming read (include/probe.h).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/probe.h"
#include "common.hpp"
#include "device_check.hpp"

using namespace mi355gemm;

namespace {

typedef float f32x16acc __attribute__((ext_vector_type(16)));

template <typename T> struct ProbeMfma;
template <> struct ProbeMfma<bf16_t> {
  static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x16acc& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                c, 0, 0, 0);
  }
  static constexpr uint32_t kFlipMask = 0x807f807fu;       // sign and significand bits of both halves
  // sign and 7 significand bits random, exponent 2^-6 .. 2^-5
  static __device__ __forceinline__ uint32_t pair(uint32_t r) {
    const uint32_t lo = (r & 0x807fu) | 0x3c80u, hi = ((r >> 16) & 0x807fu) | 0x3c80u;
    return lo | (hi << 16);
  }
};
template <> struct ProbeMfma<f16_t> {
  static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x16acc& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b),
                                               c, 0, 0, 0);
  }
  static constexpr uint32_t kFlipMask = 0x83ff83ffu;
  // sign and 10 significand bits random, exponent 2^-6
  static __device__ __forceinline__ uint32_t pair(uint32_t r) {
    const uint32_t lo = (r & 0x83ffu) | 0x2400u, hi = ((r >> 16) & 0x83ffu) | 0x2400u;
    return lo | (hi << 16);
  }
};

// fp8 (E4M3): operands of 8 registers, v_mfma_f32_32x32x64_f8f6f4
typedef int i32x8_t __attribute__((ext_vector_type(8)));
struct ProbeMfma8 {
  static constexpr uint32_t kFlipMask = 0x87878787u;       // sign and significand bits of the four bytes
  static __device__ __forceinline__ uint32_t word(uint32_t r) { return (r & kFlipMask) | 0x28282828u; }  // 2^-2 ..
  static __device__ __forceinline__ void run(const i32x8_t& a, const i32x8_t& b, f32x16acc& c) {
    c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);   // fp8 x fp8, no block scales
  }
};

__device__ __forceinline__ uint32_t mix(uint32_t x) {      // integer hash (xorshift-multiply)
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

constexpr int kMfmaPerStep = 8;      // 4 x 2 accumulators, as a wave of the 256x256 tile

// REFRESH: the sign and significand bits of every operand register are flipped by a new
// pseudo-random word before every step (one XOR per register, well within the vector ALU's
// spare slots), so that no MFMA sees operands it has seen before, as in a real product.
template <typename T, bool REFRESH>
__global__ __launch_bounds__(512) void mfma_peak_kernel(int steps, float* sink) {
  u32x4_t a[4], b[2];
  const uint32_t id = (blockIdx.x * 512u + threadIdx.x) * 64u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) a[i][e] = ProbeMfma<T>::pair(mix(id + i * 4 + e));
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) b[i][e] = ProbeMfma<T>::pair(mix(id + 32 + i * 4 + e));
  f32x16acc acc[4][2];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;
  // four steps per trip; the A operands rotate by one register set each step (by renaming)
  uint32_t rnd = 0x9e3779b9u;
  for (int s = 0; s < steps; s += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (REFRESH) {
        rnd = rnd * 1664525u + 1013904223u;               // wave-uniform: scalar ALU
        const uint32_t flip = rnd & ProbeMfma<T>::kFlipMask;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) a[i][e] ^= flip;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) b[i][e] ^= (flip >> 1) & ProbeMfma<T>::kFlipMask;
      }
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n) ProbeMfma<T>::run(b[(n + u) & 1], a[(m + u) & 3], acc[m][n]);
    }
  }
  float t = 0.0f;
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) t += acc[m][n][r];
  if (t == 1.2345e38f) *sink = t;                        // never true; keeps the loop alive
}

// The same loop on v_mfma_f32_16x16x32: the accumulator footprint of a 128x64 wave block of the
// 256x256 tile (8 x 4 accumulators of 16x16), 8 + 4 operand registers sets, 32 MFMAs per step of
// 32 columns of K.
template <typename T> struct ProbeMfma16;
template <> struct ProbeMfma16<bf16_t> {
  static __device__ __forceinline__ f32x4_t run(const u32x4_t& a, const u32x4_t& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};
template <> struct ProbeMfma16<f16_t> {
  static __device__ __forceinline__ f32x4_t run(const u32x4_t& a, const u32x4_t& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};

template <typename T, bool REFRESH>
__global__ __launch_bounds__(512) void mfma16_peak_kernel(int steps, float* sink) {
  u32x4_t op[12];                                         // 0..7: row fragments, 8..11: column fragments
  const uint32_t id = (blockIdx.x * 512u + threadIdx.x) * 64u;
#pragma unroll
  for (int i = 0; i < 12; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) op[i][e] = ProbeMfma<T>::pair(mix(id + i * 4 + e));
  f32x4_t acc[8][4];
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int n = 0; n < 4; ++n) acc[m][n] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  uint32_t rnd = 0x9e3779b9u;
  for (int s = 0; s < steps; ++s) {
    if (REFRESH) {
      rnd = rnd * 1664525u + 1013904223u;                 // wave-uniform: scalar ALU
      const uint32_t flip = rnd & ProbeMfma<T>::kFlipMask;
#pragma unroll
      for (int i = 0; i < 12; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) op[i][e] ^= (i & 1) ? flip : ((flip >> 1) & ProbeMfma<T>::kFlipMask);
    }
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[m][n] = ProbeMfma16<T>::run(op[8 + n], op[m], acc[m][n]);
  }
  float t = 0.0f;
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int r = 0; r < 4; ++r) t += acc[m][n][r];
  if (t == 1.2345e38f) *sink = t;                        // never true; keeps the loop alive
}

template <bool REFRESH>
__global__ __launch_bounds__(512) void mfma8_peak_kernel(int steps, float* sink) {
  i32x8_t a[4], b[2];
  const uint32_t id = (blockIdx.x * 512u + threadIdx.x) * 64u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) a[i][e] = (int)ProbeMfma8::word(mix(id + i * 8 + e));
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) b[i][e] = (int)ProbeMfma8::word(mix(id + 32 + i * 8 + e));
  f32x16acc acc[4][2];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;
  uint32_t rnd = 0x9e3779b9u;
  for (int s = 0; s < steps; s += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (REFRESH) {
        rnd = rnd * 1664525u + 1013904223u;
        const int flip = (int)(rnd & ProbeMfma8::kFlipMask);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 8; ++e) a[i][e] ^= flip;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int e = 0; e < 8; ++e) b[i][e] ^= (int)(((uint32_t)flip >> 1) & ProbeMfma8::kFlipMask);
      }
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n) ProbeMfma8::run(b[(n + u) & 1], a[(m + u) & 3], acc[m][n]);
    }
  }
  float t = 0.0f;
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) t += acc[m][n][r];
  if (t == 1.2345e38f) *sink = t;
}

// a wave reads whole 16 KB pieces, 16 loads of 16 bytes per lane in flight
__global__ __launch_bounds__(256) void read_peak_kernel(const u32x4_t* __restrict__ src, int64_t pieces,
                                                        float* sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  u32x4_t acc = {0u, 0u, 0u, 0u};
  for (int64_t p = (int64_t)blockIdx.x * 4 + wave; p < pieces; p += (int64_t)gridDim.x * 4) {
    const u32x4_t* base = src + p * 1024 + lane;
    u32x4_t v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = __builtin_nontemporal_load(base + i * 64);
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= v[i];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) *sink = 1.0f;   // practically never; keeps the loads
}

// launch() enqueues one launch; returns average seconds per launch over at least min_seconds
template <typename F>
int timed(F launch, hipStream_t s, double min_seconds, double* sec_per_launch) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return GEMM_ERR_LAUNCH;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return GEMM_ERR_LAUNCH; }
  int rc = GEMM_OK;
  double total = 0;
  int64_t launches = 0;
  int batch = 1;
  launch();                                                         // warm-up
  if (hipStreamSynchronize(s) != hipSuccess) rc = GEMM_ERR_LAUNCH;
  while (rc == GEMM_OK && (total < min_seconds || launches < 3)) {
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < batch; ++i) launch();
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) { rc = GEMM_ERR_LAUNCH; break; }
    float ms = 0;
    (void)hipEventElapsedTime(&ms, e0, e1);
    total += ms * 1e-3;
    launches += batch;
    if (ms < 20.0f && batch < 1024) batch *= 2;                      // longer inner loops for short launches
    if (launches > (1 << 20)) break;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == GEMM_OK) *sec_per_launch = total / (double)launches;
  return rc;
}

}  // namespace

extern "C" int probe_mfma_peak(int dtype, int refresh_operands, void* sink, void* hip_stream,
                               double min_seconds, double* tflops) {
  if (!sink || !tflops) return GEMM_ERR_NULL;
  if (dtype != GEMM_BF16 && dtype != GEMM_F16 && dtype != GEMM_F8E4M3) return GEMM_ERR_UNSUPPORTED;
  if (refresh_operands != 0 && refresh_operands != 1) return GEMM_ERR_BAD_ENUM;
  if ((uintptr_t)sink & 3) return GEMM_ERR_MISALIGNED;
  if (!(min_seconds >= 0.0)) min_seconds = 0.0;
  int rc = check_device_gfx950();
  if (rc != GEMM_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  const int steps = 4096, grid = 256;                               // ~0.3 ms per launch
  double sec = 0;
  float* sk = (float*)sink;
  if (dtype == GEMM_F8E4M3) {
    if (!refresh_operands)
      rc = timed([&] { mfma8_peak_kernel<false><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
    else
      rc = timed([&] { mfma8_peak_kernel<true><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
    if (rc != GEMM_OK) return rc;
    *tflops = 2.0 * 32 * 32 * 64 * kMfmaPerStep * (double)steps * 8.0 * grid / sec / 1e12;
    return GEMM_OK;
  }
  if (dtype == GEMM_BF16 && !refresh_operands)
    rc = timed([&] { mfma_peak_kernel<bf16_t, false><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  else if (dtype == GEMM_BF16)
    rc = timed([&] { mfma_peak_kernel<bf16_t, true><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  else if (!refresh_operands)
    rc = timed([&] { mfma_peak_kernel<f16_t, false><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  else
    rc = timed([&] { mfma_peak_kernel<f16_t, true><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  if (rc != GEMM_OK) return rc;
  const double flops = 2.0 * 32 * 32 * 16 * kMfmaPerStep * (double)steps * 8.0 * grid;
  *tflops = flops / sec / 1e12;
  return GEMM_OK;
}

extern "C" int probe_mfma16_peak(int dtype, int refresh_operands, void* sink, void* hip_stream,
                                 double min_seconds, double* tflops) {
  if (!sink || !tflops) return GEMM_ERR_NULL;
  if (dtype != GEMM_BF16 && dtype != GEMM_F16) return GEMM_ERR_UNSUPPORTED;
  if (refresh_operands != 0 && refresh_operands != 1) return GEMM_ERR_BAD_ENUM;
  if ((uintptr_t)sink & 3) return GEMM_ERR_MISALIGNED;
  if (!(min_seconds >= 0.0)) min_seconds = 0.0;
  int rc = check_device_gfx950();
  if (rc != GEMM_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  const int steps = 2048, grid = 256;                               // ~0.3 ms per launch
  double sec = 0;
  float* sk = (float*)sink;
  if (dtype == GEMM_BF16 && !refresh_operands)
    rc = timed([&] { mfma16_peak_kernel<bf16_t, false><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  else if (dtype == GEMM_BF16)
    rc = timed([&] { mfma16_peak_kernel<bf16_t, true><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  else if (!refresh_operands)
    rc = timed([&] { mfma16_peak_kernel<f16_t, false><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  else
    rc = timed([&] { mfma16_peak_kernel<f16_t, true><<<grid, 512, 0, s>>>(steps, sk); }, s, min_seconds, &sec);
  if (rc != GEMM_OK) return rc;
  *tflops = 2.0 * 16 * 16 * 32 * 32 * (double)steps * 8.0 * grid / sec / 1e12;   // 32 MFMAs per step and wave
  return GEMM_OK;
}

extern "C" int probe_read_peak(const void* src, size_t bytes, void* sink, void* hip_stream, double min_seconds,
                               double* gbytes_per_s) {
  if (!src || !sink || !gbytes_per_s) return GEMM_ERR_NULL;
  if (bytes < ((size_t)1 << 30) || bytes % 16384 != 0) return GEMM_ERR_BAD_DIM;
  if (((uintptr_t)src & 15) || ((uintptr_t)sink & 3)) return GEMM_ERR_MISALIGNED;
  if (!(min_seconds >= 0.0)) min_seconds = 0.0;
  int rc = check_device_gfx950();
  if (rc != GEMM_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  const int64_t pieces = (int64_t)(bytes / 16384);
  double sec = 0;
  rc = timed([&] { read_peak_kernel<<<256, 256, 0, s>>>((const u32x4_t*)src, pieces, (float*)sink); }, s,
             min_seconds, &sec);
  if (rc != GEMM_OK) return rc;
  *gbytes_per_s = (double)bytes / sec / 1e9;
  return GEMM_OK;
}
