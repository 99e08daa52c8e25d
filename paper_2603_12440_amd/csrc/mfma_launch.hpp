// Launcher of the matrix-core kernel and the list of its compiled tile shapes.  The
// instantiations are spread over one translation unit per operand type
// (mfma_bf16_inst.hip, mfma_f16_inst.hip, mfma_f8_inst.hip); the table in gemm_api.hip
// only refers to them.
#pragma once

#include "plan.hpp"
#include "mfma_kernel.hpp"

namespace mi355gemm {

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int NS>
hipError_t launch_mfma(const gemm_plan& pl, const void* A, const void* B, void* C,
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
  mfma_gemm_kernel<T, TO, BM, BN, BK, WM, WN, NS><<<pl.grid, pl.block, 0, s>>>(a);
  return hipGetLastError();
}

// X(BM, BN, BK, WM, WN, NSTAGE): tile, wave grid, LDS stages.  16-bit operands:
#define MI355GEMM_MFMA_TILES(X) \
  X(256, 256, 64, 2, 4, 2)      \
  X(256, 256, 64, 2, 2, 2)      \
  X(256, 128, 64, 2, 2, 2)      \
  X(128, 128, 64, 2, 2, 2)      \
  X(256, 192, 64, 4, 2, 2)
// fp8 operands (BK is twice as many values: the same slabs in bytes):
#define MI355GEMM_MFMA8_TILES(X) \
  X(256, 256, 128, 2, 4, 2)      \
  X(128, 128, 128, 2, 2, 2)      \
  X(256, 192, 128, 4, 2, 2)

#define MI355GEMM_MFMA_DECLARE(T, TO, BM, BN, BK, WM, WN, NS)                               \
  extern template hipError_t launch_mfma<T, TO, BM, BN, BK, WM, WN, NS>(                      \
      const gemm_plan&, const void*, const void*, void*, const void*, hipStream_t);
#define MI355GEMM_MFMA_DEFINE(T, TO, BM, BN, BK, WM, WN, NS)                                \
  template hipError_t launch_mfma<T, TO, BM, BN, BK, WM, WN, NS>(                             \
      const gemm_plan&, const void*, const void*, void*, const void*, hipStream_t);

}  // namespace mi355gemm
