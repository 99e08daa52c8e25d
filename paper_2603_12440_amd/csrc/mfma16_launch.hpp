// Launcher of the 16x16x32 matrix-core kernel and the list of its compiled tile shapes.  The
// instantiations live in one translation unit per operand type (mfma16_bf16_inst.hip,
// mfma16_f16_inst.hip); the table in gemm_api.hip only refers to them.
#pragma once

#include "plan.hpp"
#include "mfma16_kernel.hpp"

namespace mi355gemm {

template <typename T, typename TO, int BM, int BN, int WM, int WN, int G, bool PERSIST>
hipError_t launch_mfma16(const gemm_plan& pl, const void* A, const void* B, void* C,
                         const void* bias, hipStream_t s) {
  const gemm_desc_t& d = pl.d;
  MfmaArgs a;
  a.A = A; a.B = B; a.C = C; a.bias = (const float*)bias;
  a.M = (int)d.M; a.N = (int)d.N; a.K = (int)d.K;
  a.lda = d.lda; a.ldb = d.ldb; a.ldc = d.ldc;
  a.stride_a = d.stride_a; a.stride_b = d.stride_b; a.stride_c = d.stride_c;
  a.stride_bias = d.stride_bias;
  a.has_bias = epilogue_has_bias(d.epilogue);
  a.act = epilogue_activation(d.epilogue);
  a.scale = d.scale;
  a.c_f32 = d.dtype_c == GEMM_F32;
  a.tiles_m = (int)((d.M + BM - 1) / BM);
  a.tiles_n = (int)((d.N + BN - 1) / BN);
  a.group_m = pl.group_m;
  a.xcd_remap = pl.xcd_remap;
  a.c_cached = pl.c_cached;
  a.batches = (int)d.batch;
  if constexpr (PERSIST) {
    // The persistent kernel only has the staged output routes (whole-line stores): C rows that are
    // not 16-byte aligned run one tile per workgroup instead.
    const int64_t unit = a.c_f32 ? 4 : 8;
    const bool staged = d.ldc % unit == 0 && d.stride_c % unit == 0 && ((uintptr_t)C & 15) == 0;
    if (!staged) {
      const dim3 grid((unsigned)(a.tiles_m * a.tiles_n), (unsigned)d.batch, 1);
      mfma16_gemm_kernel<T, TO, BM, BN, WM, WN, G, false><<<grid, pl.block, 0, s>>>(a);
      return hipGetLastError();
    }
  }
  mfma16_gemm_kernel<T, TO, BM, BN, WM, WN, G, PERSIST><<<pl.grid, pl.block, 0, s>>>(a);
  return hipGetLastError();
}

// X(BM, BN, WM, WN, G, PERSIST): tile, wave grid, sub-steps per k-step (slabs of 64 columns of K, two
// stages), one tile per workgroup or a persistent workgroup walking over several
#define MI355GEMM_MFMA16_TILES(X) \
  X(256, 256, 2, 4, 2, false)     \
  X(256, 256, 2, 2, 2, false)     \
  X(128, 128, 2, 2, 2, false)
#define MI355GEMM_MFMA16P_TILES(X) \
  X(256, 256, 2, 4, 2, true)       \
  X(128, 128, 2, 2, 2, true)

#define MI355GEMM_MFMA16_DECLARE(T, TO, BM, BN, WM, WN, G, P)                               \
  extern template hipError_t launch_mfma16<T, TO, BM, BN, WM, WN, G, P>(                      \
      const gemm_plan&, const void*, const void*, void*, const void*, hipStream_t);
#define MI355GEMM_MFMA16_DEFINE(T, TO, BM, BN, WM, WN, G, P)                                \
  template hipError_t launch_mfma16<T, TO, BM, BN, WM, WN, G, P>(                             \
      const gemm_plan&, const void*, const void*, void*, const void*, hipStream_t);

}  // namespace mi355gemm
