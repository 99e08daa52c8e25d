// Host side of the mi355gemm C ABI (include/gemm.h): descriptor validation, the
// table of compiled kernel instantiations, the choice among them, and launches.
//
// The table-plus-dispatcher shape follows the paper's templated kernels
// (Sec. 3.4 and the templated-kernel example in the appendix): every tile
// shape is a template instantiation, a dispatch function maps integer
// parameters to the instantiation, and a tuner may time each applicable one.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/gemm.h"
#include "common.hpp"
#include "plan.hpp"
#include "mfma_launch.hpp"
#include "mfma16_launch.hpp"
#include "simt_kernel.hpp"
#include "general_mfma_kernel.hpp"
#include "f32_mfma_kernel.hpp"
#include "skinny_kernel.hpp"
#include "splitk_kernel.hpp"
#include "device_check.hpp"

using namespace mi355gemm;

namespace mi355gemm {
#define X(BM, BN, BK, WM, WN, NS) MI355GEMM_MFMA_DECLARE(bf16_t, bf16_t, BM, BN, BK, WM, WN, NS) \
                                 MI355GEMM_MFMA_DECLARE(f16_t, f16_t, BM, BN, BK, WM, WN, NS)
MI355GEMM_MFMA_TILES(X)
#undef X
#define X(BM, BN, BK, WM, WN, NS) MI355GEMM_MFMA_DECLARE(f8e4m3_t, bf16_t, BM, BN, BK, WM, WN, NS)
MI355GEMM_MFMA8_TILES(X)
#undef X
#define X(BM, BN, WM, WN, G, P) MI355GEMM_MFMA16_DECLARE(bf16_t, bf16_t, BM, BN, WM, WN, G, P) \
                                MI355GEMM_MFMA16_DECLARE(f16_t, f16_t, BM, BN, WM, WN, G, P)
MI355GEMM_MFMA16_TILES(X)
MI355GEMM_MFMA16P_TILES(X)
#undef X
}  // namespace mi355gemm

namespace {

// ---- launchers ---------------------------------------------------------------------

// the argument block of the general kernels: layouts become element strides
SimtArgs simt_args(const gemm_plan& pl, const void* A, const void* B, void* C, const void* bias) {
  const gemm_desc_t& d = pl.d;
  SimtArgs a;
  a.A = A; a.B = B; a.C = C; a.bias = (const float*)bias;
  a.M = d.M; a.N = d.N; a.K = d.K;
  a.a_si = d.layout_a == GEMM_ROW_MAJOR ? d.lda : 1;
  a.a_sk = d.layout_a == GEMM_ROW_MAJOR ? 1 : d.lda;
  a.b_sk = d.layout_b == GEMM_ROW_MAJOR ? d.ldb : 1;
  a.b_sj = d.layout_b == GEMM_ROW_MAJOR ? 1 : d.ldb;
  a.c_si = d.layout_c == GEMM_ROW_MAJOR ? d.ldc : 1;
  a.c_sj = d.layout_c == GEMM_ROW_MAJOR ? 1 : d.ldc;
  a.stride_a = d.stride_a; a.stride_b = d.stride_b; a.stride_c = d.stride_c;
  a.stride_bias = d.stride_bias;
  a.has_bias = epilogue_has_bias(d.epilogue);
  a.act = epilogue_activation(d.epilogue);
  a.scale = d.scale;
  return a;
}

template <typename TIn, typename TOut, int TM, int TN, int TK>
hipError_t launch_simt_typed(const gemm_plan& pl, const void* A, const void* B, void* C,
                             const void* bias, hipStream_t s) {
  const SimtArgs a = simt_args(pl, A, B, C, bias);
  simt_gemm_kernel<TIn, TOut, TM, TN, TK><<<pl.grid, pl.block, 0, s>>>(a);
  return hipGetLastError();
}

template <typename TIn, typename TOut, int TM, int TN, int TK>
hipError_t launch_general_mfma_typed(const gemm_plan& pl, const void* A, const void* B, void* C,
                                     const void* bias, hipStream_t s) {
  const SimtArgs a = simt_args(pl, A, B, C, bias);
  general_mfma_kernel<TIn, TOut, TM, TN, TK><<<pl.grid, pl.block, 0, s>>>(a);
  return hipGetLastError();
}

template <typename TIn, int TM, int TN, int TK>
hipError_t launch_general_mfma(const gemm_plan& pl, const void* A, const void* B, void* C,
                               const void* bias, hipStream_t s) {
  if (pl.d.dtype_c == GEMM_F32)
    return launch_general_mfma_typed<TIn, float, TM, TN, TK>(pl, A, B, C, bias, s);
  return launch_general_mfma_typed<TIn, TIn, TM, TN, TK>(pl, A, B, C, bias, s);
}

// fp32 operands in 16-byte pieces (the plan's extents and leading dimensions allow it: applicable());
// pointers that are not 16-byte aligned take the general kernel on the same grid
template <int TM, int TN>
hipError_t launch_f32_mfma(const gemm_plan& pl, const void* A, const void* B, void* C,
                           const void* bias, hipStream_t s) {
  const gemm_desc_t& d = pl.d;
  if (((uintptr_t)A & 15) || ((uintptr_t)B & 15))
    return launch_general_mfma_typed<float, float, TM, TN, 16>(pl, A, B, C, bias, s);
  const SimtArgs a = simt_args(pl, A, B, C, bias);
  const bool ak = d.layout_a == GEMM_ROW_MAJOR, bk = d.layout_b == GEMM_COL_MAJOR;   // K contiguous?
  if (ak && bk) f32_mfma_kernel<true, true, TM, TN><<<pl.grid, pl.block, 0, s>>>(a);
  else if (ak) f32_mfma_kernel<true, false, TM, TN><<<pl.grid, pl.block, 0, s>>>(a);
  else if (bk) f32_mfma_kernel<false, true, TM, TN><<<pl.grid, pl.block, 0, s>>>(a);
  else f32_mfma_kernel<false, false, TM, TN><<<pl.grid, pl.block, 0, s>>>(a);
  return hipGetLastError();
}

// small fp32 problems: 16x16 tiles, K split over the waves of a workgroup; each K-contiguous operand
// is read in float4 groups when its extents, strides and pointer allow it
hipError_t launch_f32_small(const gemm_plan& pl, const void* A, const void* B, void* C,
                            const void* bias, hipStream_t s) {
  const gemm_desc_t& d = pl.d;
  F32SmallArgs a;
  a.g = simt_args(pl, A, B, C, bias);
  a.vec_a = d.layout_a == GEMM_ROW_MAJOR && d.K % 4 == 0 && d.lda % 4 == 0 && d.stride_a % 4 == 0 &&
            ((uintptr_t)A & 15) == 0;
  a.vec_b = d.layout_b == GEMM_COL_MAJOR && d.K % 4 == 0 && d.ldb % 4 == 0 && d.stride_b % 4 == 0 &&
            ((uintptr_t)B & 15) == 0;
  f32_small_kernel<<<pl.grid, pl.block, 0, s>>>(a);
  return hipGetLastError();
}

template <typename TIn, int TM, int TN, int TK>
hipError_t launch_simt(const gemm_plan& pl, const void* A, const void* B, void* C,
                       const void* bias, hipStream_t s) {
  if (pl.d.dtype_c == GEMM_F32)
    return launch_simt_typed<TIn, float, TM, TN, TK>(pl, A, B, C, bias, s);
  return launch_simt_typed<TIn, TIn, TM, TN, TK>(pl, A, B, C, bias, s);
}

// the argument block every skinny kernel takes
SkinnyArgs skinny_args(const gemm_plan& pl, const void* A, const void* B, void* C, const void* bias) {
  const gemm_desc_t& d = pl.d;
  SkinnyArgs a;
  a.X = A; a.W = B; a.Y = C; a.bias = (const float*)bias;
  a.M = (int)d.M; a.N = (int)d.N; a.K = (int)d.K;
  a.ldx = d.lda; a.ldw = d.ldb; a.ldy = d.ldc;
  a.stride_x = d.stride_a; a.stride_w = d.stride_b; a.stride_y = d.stride_c;
  a.stride_bias = d.stride_bias;
  a.has_bias = epilogue_has_bias(d.epilogue);
  a.act = epilogue_activation(d.epilogue);
  a.scale = d.scale;
  a.y_f32 = d.dtype_c == GEMM_F32;
  return a;
}

template <typename T, int MB, int WAVES>
hipError_t launch_skinny(const gemm_plan& pl, const void* A, const void* B, void* C,
                         const void* bias, hipStream_t s) {
  skinny_gemm_kernel<T, MB, WAVES><<<pl.grid, pl.block, 0, s>>>(skinny_args(pl, A, B, C, bias));
  return hipGetLastError();
}

template <typename T, int DEPTH, int RB, int WAVES>
hipError_t launch_skinny_stage(const gemm_plan& pl, const void* A, const void* B, void* C,
                               const void* bias, hipStream_t s) {
  skinny_stage_kernel<T, DEPTH, RB, WAVES><<<pl.grid, pl.block, 0, s>>>(skinny_args(pl, A, B, C, bias));
  return hipGetLastError();
}

template <typename T, int DEPTH, int RB, int WAVES>
hipError_t launch_skinny_direct(const gemm_plan& pl, const void* A, const void* B, void* C,
                                const void* bias, hipStream_t s) {
  skinny_direct_kernel<T, DEPTH, RB, WAVES><<<pl.grid, pl.block, 0, s>>>(skinny_args(pl, A, B, C, bias));
  return hipGetLastError();
}

// ---- the table of compiled instantiations ----------------------------------------------

#define SIMT_CFG(TM, TN, TK)                                                               \
  { "simt_" #TM "x" #TN "x" #TK, KIND_SIMT, TM, TN, TK, 256,                               \
    (int)(sizeof(float) * TK * (TM + 4 + TN + 4)),                                         \
    { launch_simt<float, TM, TN, TK>, launch_simt<bf16_t, TM, TN, TK>,                     \
      launch_simt<f16_t, TM, TN, TK> } }

// the general kernel on the matrix cores (fp32 MFMA): same problems, same grid as SIMT_CFG
#define GENERAL_MFMA_CFG(TM, TN, TK)                                                       \
  { "general_mfma32_" #TM "x" #TN "x" #TK, KIND_SIMT, TM, TN, TK, 256,                     \
    (int)(sizeof(float) * TK * (TM + 4 + TN + 4)),                                         \
    { launch_general_mfma<float, TM, TN, TK>, launch_general_mfma<bf16_t, TM, TN, TK>,     \
      launch_general_mfma<f16_t, TM, TN, TK> } }

// fp32 operands and output moved as float4 groups: 128x128 tiles, slabs of 32 columns of K
#define F32_MFMA_CFG(TM, TN)                                                               \
  { "f32mfma_" #TM "x" #TN "x32", KIND_F32_VEC, TM, TN, kF32TileK, 256,                    \
    (int)(sizeof(float) * 2 * (F32Stage<true, TM>::SIZE + F32Stage<true, TN>::SIZE)),      \
    { launch_f32_mfma<TM, TN>, nullptr, nullptr } }

// small fp32 problems: 16x16 tiles, 256 columns of K per round of the four waves
#define F32_SMALL_CFG()                                                                    \
  { "f32small_16x16x256", KIND_SIMT, 16, 16, 256, 256, 4096, { launch_f32_small, nullptr, nullptr } }

#define MFMA_CFG(BM, BN, BK, WM, WN, NS)                                                   \
  { "mfma_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS, KIND_MFMA, BM, BN, BK,          \
    64 * WM * WN, MfmaTile<bf16_t, BM, BN, BK, WM, WN, NS>::LDS_BYTES,                     \
    { nullptr, launch_mfma<bf16_t, bf16_t, BM, BN, BK, WM, WN, NS>,                        \
      launch_mfma<f16_t, f16_t, BM, BN, BK, WM, WN, NS> } }
// the same product on the 16x16x32 MFMA shape (slabs of 64 columns of K, two stages)
#define MFMA16_CFG(BM, BN, WM, WN, G)                                                      \
  { "mfma16_" #BM "x" #BN "x64_w" #WM "x" #WN, KIND_MFMA, BM, BN, 64,                      \
    64 * WM * WN, Mfma16Tile<bf16_t, BM, BN, WM, WN, G>::LDS_BYTES,                        \
    { nullptr, launch_mfma16<bf16_t, bf16_t, BM, BN, WM, WN, G, false>,                    \
      launch_mfma16<f16_t, f16_t, BM, BN, WM, WN, G, false> }, 0 }
// persistent workgroups (K a whole number of slabs, at least two): the grid is the number of
// workgroups the chip holds at once, each walks over its share of the tiles
#define MFMA16P_CFG(BM, BN, WM, WN, G)                                                     \
  { "mfma16_" #BM "x" #BN "x64_w" #WM "x" #WN "_p", KIND_MFMA, BM, BN, 64,                 \
    64 * WM * WN, Mfma16Tile<bf16_t, BM, BN, WM, WN, G>::LDS_BYTES +                       \
                      Mfma16Tile<bf16_t, BM, BN, WM, WN, G>::EPI_BYTES,                    \
    { nullptr, launch_mfma16<bf16_t, bf16_t, BM, BN, WM, WN, G, true>,                     \
      launch_mfma16<f16_t, f16_t, BM, BN, WM, WN, G, true> }, 1 }
// fp8 (E4M3) operands, bf16 or fp32 output: the same slabs in bytes (BK is twice as many values)
#define MFMA8_CFG(BM, BN, BK, WM, WN, NS)                                                  \
  { "mfma8_" #BM "x" #BN "x" #BK "_w" #WM "x" #WN "_s" #NS, KIND_MFMA, BM, BN, BK,         \
    64 * WM * WN, MfmaTile<f8e4m3_t, BM, BN, BK, WM, WN, NS>::LDS_BYTES,                   \
    { nullptr, nullptr, nullptr, launch_mfma<f8e4m3_t, bf16_t, BM, BN, BK, WM, WN, NS> } }

// bn = workgroups per CU the grid is sized for
#define SKINNY_CFG(MB, WAVES, PER_CU)                                                      \
  { "skinny_m" #MB "_w" #WAVES "_g" #PER_CU, KIND_SKINNY, MB, PER_CU, kSkinnyKC,           \
    64 * WAVES, (MB == 1 || (MB == 2 && WAVES <= 4)) ? 16 : MB * kSkinnyKC * 2,            \
    { nullptr, launch_skinny<bf16_t, MB, WAVES>, launch_skinny<f16_t, MB, WAVES> } }

// skinny on the matrix cores, W staged through registers into wave-private LDS slabs:
// bm = 16 x rows, bn = 32 rows of W per workgroup, bk = k per slab
#define SKINNY_STAGE_CFG(DEPTH, RB)                                                        \
  { "skinnystage_d" #DEPTH "_b" #RB, KIND_SKINNY_PANEL, 16, 32, RB / 2, 256, 4 * 48 * RB,     \
    { nullptr, launch_skinny_stage<bf16_t, DEPTH, RB, 4>, launch_skinny_stage<f16_t, DEPTH, RB, 4> } }
// skinny with W staged through LDS and x fragments straight from L2 (16x16x32 MFMA): same panel shape
#define SKINNY_DIRECT_CFG(DEPTH, RB, WAVES)                                                \
  { "skinnydirect_d" #DEPTH "_b" #RB "_w" #WAVES, KIND_SKINNY_PANEL, 16, 32, RB / 2, 64 * WAVES, WAVES * 32 * RB, \
    { nullptr, launch_skinny_direct<bf16_t, DEPTH, RB, WAVES>, launch_skinny_direct<f16_t, DEPTH, RB, WAVES> } }
const Config kConfigs[] = {
    SIMT_CFG(64, 64, 16),
    SIMT_CFG(32, 32, 16),
    SIMT_CFG(32, 32, 64),
    MFMA16P_CFG(256, 256, 2, 4, 2),
    MFMA16P_CFG(128, 128, 2, 2, 2),
    MFMA16_CFG(256, 256, 2, 4, 2),
    MFMA16_CFG(256, 256, 2, 2, 2),
    MFMA16_CFG(128, 128, 2, 2, 2),
    MFMA_CFG(256, 256, 64, 2, 4, 2),
    MFMA_CFG(256, 256, 64, 2, 2, 2),
    MFMA_CFG(256, 128, 64, 2, 2, 2),
    MFMA_CFG(128, 128, 64, 2, 2, 2),
    MFMA_CFG(256, 192, 64, 4, 2, 2),
    MFMA8_CFG(256, 256, 128, 2, 4, 2),
    MFMA8_CFG(128, 128, 128, 2, 2, 2),
    MFMA8_CFG(256, 192, 128, 4, 2, 2),
    F32_MFMA_CFG(128, 128),
    F32_MFMA_CFG(64, 64),
    F32_SMALL_CFG(),
    GENERAL_MFMA_CFG(128, 128, 16),
    GENERAL_MFMA_CFG(64, 64, 16),
    SKINNY_CFG(1, 4, 1),
    SKINNY_CFG(2, 4, 1),
    SKINNY_CFG(4, 4, 1),
    SKINNY_CFG(8, 4, 1),
    SKINNY_CFG(1, 8, 1),
    SKINNY_CFG(1, 8, 2),
    SKINNY_CFG(2, 8, 1),
    SKINNY_CFG(4, 8, 1),
    SKINNY_STAGE_CFG(3, 256),
    SKINNY_STAGE_CFG(2, 512),
    SKINNY_DIRECT_CFG(2, 512, 4),
    SKINNY_DIRECT_CFG(3, 512, 4),
    SKINNY_DIRECT_CFG(2, 256, 8),
};
constexpr int kNumConfigs = (int)(sizeof(kConfigs) / sizeof(kConfigs[0]));

// Compute units of the device the plans are made for: asked of the runtime once (the current
// device at the first plan); 256, an MI355X, where no device can be asked (plans can be made
// and inspected on a machine without a GPU).
int num_cus() {
  static const int n = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      return cus;
    (void)hipGetLastError();
    return 256;
  }();
  return n;
}

// ---- validation -----------------------------------------------------------------------

bool in_range(int v, int lo, int hi) { return v >= lo && v <= hi; }

// Resolve packed (0) leading dimensions / strides and check every field.
int resolve(const gemm_desc_t* in, gemm_desc_t* out) {
  gemm_desc_t d = *in;
  if (!in_range(d.layout_a, 0, 1) || !in_range(d.layout_b, 0, 1) || !in_range(d.layout_c, 0, 1) ||
      !in_range(d.dtype_a, 0, 3) || !in_range(d.dtype_b, 0, 3) || !in_range(d.dtype_c, 0, 3) ||
      !in_range(d.dtype_bias, 0, 2) || !in_range(d.epilogue, 0, GEMM_EPI_SIGMOID_SCALE_RESIDUAL))
    return GEMM_ERR_BAD_ENUM;
  if (epilogue_has_scale(d.epilogue)) {
    if (!std::isfinite(d.scale)) return GEMM_ERR_BAD_SCALE;
  } else {
    d.scale = 1.0f;                              // ignored: keep the plan's copy tidy
  }
  if (d.M <= 0 || d.N <= 0 || d.K <= 0 || d.batch < 1) return GEMM_ERR_BAD_DIM;
  const int64_t kMaxDim = (int64_t)1 << 30;
  if (d.M > kMaxDim || d.N > kMaxDim || d.K > kMaxDim || d.batch > 65535) return GEMM_ERR_BAD_DIM;
  if (d.lda < 0 || d.ldb < 0 || d.ldc < 0 || d.stride_a < 0 || d.stride_b < 0 ||
      d.stride_c < 0 || d.stride_bias < 0)
    return GEMM_ERR_BAD_LD;

  const int64_t a_minor = d.layout_a == GEMM_ROW_MAJOR ? d.K : d.M;
  const int64_t a_major = d.layout_a == GEMM_ROW_MAJOR ? d.M : d.K;
  const int64_t b_minor = d.layout_b == GEMM_ROW_MAJOR ? d.N : d.K;
  const int64_t b_major = d.layout_b == GEMM_ROW_MAJOR ? d.K : d.N;
  const int64_t c_minor = d.layout_c == GEMM_ROW_MAJOR ? d.N : d.M;
  const int64_t c_major = d.layout_c == GEMM_ROW_MAJOR ? d.M : d.N;
  if (d.lda == 0) d.lda = a_minor;
  if (d.ldb == 0) d.ldb = b_minor;
  if (d.ldc == 0) d.ldc = c_minor;
  if (d.lda < a_minor || d.ldb < b_minor || d.ldc < c_minor) return GEMM_ERR_BAD_LD;
  const int64_t kMaxLd = (int64_t)1 << 40;
  if (d.lda > kMaxLd || d.ldb > kMaxLd || d.ldc > kMaxLd) return GEMM_ERR_BAD_LD;
  // extents in elements: major * ld must stay below 2^62 (no signed overflow anywhere below)
  int64_t a_full, b_full, c_full;
  const int64_t kMaxSpan = (int64_t)1 << 62;
  if (__builtin_mul_overflow(a_major, d.lda, &a_full) || a_full >= kMaxSpan ||
      __builtin_mul_overflow(b_major, d.ldb, &b_full) || b_full >= kMaxSpan ||
      __builtin_mul_overflow(c_major, d.ldc, &c_full) || c_full >= kMaxSpan)
    return GEMM_ERR_BAD_LD;
  const int64_t a_span = a_full - d.lda + a_minor;
  const int64_t b_span = b_full - d.ldb + b_minor;
  const int64_t c_span = c_full - d.ldc + c_minor;
  if (d.stride_a == 0) d.stride_a = a_full;
  if (d.stride_b == 0) d.stride_b = b_full;
  if (d.stride_c == 0) d.stride_c = c_full;
  if (d.batch > 1) {
    // Reading one A or B slab for several batches would be legal, but the stride
    // field uses 0 for "packed", so overlapping inputs are not expressible; an
    // overlapping output is always an error.
    if (d.stride_a < a_span || d.stride_b < b_span || d.stride_c < c_span) return GEMM_ERR_BAD_LD;
    if (d.stride_bias != 0 && d.stride_bias < d.N) return GEMM_ERR_BAD_LD;
  }
  if (d.dtype_a != d.dtype_b) return GEMM_ERR_UNSUPPORTED;
  if (d.dtype_a == GEMM_F8E4M3) {
    if (d.dtype_c != GEMM_BF16 && d.dtype_c != GEMM_F32) return GEMM_ERR_UNSUPPORTED;
  } else if (d.dtype_c != d.dtype_a && d.dtype_c != GEMM_F32) {
    return GEMM_ERR_UNSUPPORTED;
  }
  if (d.dtype_bias != GEMM_F32) return GEMM_ERR_UNSUPPORTED;
  *out = d;
  return GEMM_OK;
}

// Can instantiation c run problem d?
bool applicable(const Config& c, const gemm_desc_t& d) {
  if (!c.launch[d.dtype_a]) return false;
  if (c.kind == KIND_SIMT) return true;
  if (c.kind == KIND_F32_VEC) {
    // float4 groups along the contiguous index of A and of B: extents, leading dimensions and batch
    // strides in multiples of 4 elements; fp32 result
    const bool ak = d.layout_a == GEMM_ROW_MAJOR, bk = d.layout_b == GEMM_COL_MAJOR;
    return d.dtype_c == GEMM_F32 && d.lda % 4 == 0 && d.ldb % 4 == 0 && d.stride_a % 4 == 0 &&
           d.stride_b % 4 == 0 && (ak ? d.K : d.M) % 4 == 0 && (bk ? d.K : d.N) % 4 == 0;
  }
  // The MFMA and skinny kernels take K-contiguous A and B, row-major C, and move
  // 16-byte pieces: every row start must be 16-byte aligned.
  if (d.layout_a != GEMM_ROW_MAJOR || d.layout_b != GEMM_COL_MAJOR || d.layout_c != GEMM_ROW_MAJOR)
    return false;
  const int64_t epc = 16 / esize(d.dtype_a);                 // operand elements per 16-byte piece
  if (d.K % epc || d.lda % epc || d.ldb % epc || d.stride_a % epc || d.stride_b % epc) return false;
  if (d.M >= ((int64_t)1 << 31) - 512 || d.N >= ((int64_t)1 << 31) - 512 ||
      d.K >= ((int64_t)1 << 31) - 512)
    return false;
  if (c.kind == KIND_SKINNY) return d.M <= c.bm;
  if (c.kind == KIND_SKINNY_PANEL)   // 32-bit lane offsets inside a 32-row panel
    return d.M <= c.bm && 32 * d.ldb * 2 < ((int64_t)1 << 32) && 32 * d.lda * 2 < ((int64_t)1 << 32) &&
           (d.N + 31) / 32 < ((int64_t)1 << 31);
  // MFMA: per-lane byte offsets inside a tile's row panel are 32-bit.
  if ((int64_t)c.bm * d.lda * esize(d.dtype_a) >= ((int64_t)1 << 32) ||
      (int64_t)c.bn * d.ldb * esize(d.dtype_a) >= ((int64_t)1 << 32))
    return false;
  if (c.persist && (d.K % c.bk != 0 || d.K < 2 * c.bk)) return false;   // whole slabs, at least two
  const int64_t tiles = ((d.M + c.bm - 1) / c.bm) * ((d.N + c.bn - 1) / c.bn);
  return (c.persist ? tiles * d.batch : tiles) < ((int64_t)1 << 31);
}

int find_config(const char* name) {
  for (int i = 0; i < kNumConfigs; ++i)
    if (!std::strcmp(kConfigs[i].name, name)) return i;
  return -1;
}

// Cost model of one MFMA tile shape on an M x N x K (x batch) problem:
// time ~ rounds over the CUs * work per round / measured relative efficiency of the tile
// shape; a fixed per-tile cost (prologue latency, epilogue) is worth ~600 columns of K.
// In these units one microsecond is about 2.7e6.
double mfma_cost(const Config& c, int64_t M, int64_t N, int64_t K, int64_t batch) {
  const int area = c.bm * c.bn;
  const int per_cu = area <= 128 * 128 ? 2 : 1;                 // workgroups that fit one CU's LDS
  // (256x192 measured: 0.85 - 1.03 of the 256x256 tile per FLOP on 4096x6144x4096, 4096x14336x4096, 8192^3)
  double eff = area >= 256 * 256 ? 1.0 : (area >= 256 * 192 ? 0.88 : (area >= 256 * 128 ? 0.75 : 0.84));
  // the 16x16x32 kernels: about a tenth faster per FLOP than the 32x32x16 ones at the same tile shape
  // (8192^3: 732 against 800 us); of the two 256x256 shapes the eight-wave one goes first
  if (!std::strncmp(c.name, "mfma16_", 7)) eff *= c.threads == 256 && area >= 256 * 256 ? 1.08 : 1.10;
  const double tiles = (double)((M + c.bm - 1) / c.bm) * (double)((N + c.bn - 1) / c.bn) * (double)batch;
  const double rounds = (double)(int64_t)((tiles + num_cus() * per_cu - 1) / (num_cus() * per_cu));
  // workgroups that actually share a CU (a lone workgroup runs about per_cu times faster)
  const double sharing = tiles >= (double)num_cus() * per_cu ? per_cu : (tiles > num_cus() ? tiles / num_cus() : 1.0);
  return rounds * area * sharing / eff * ((double)K + 600.0);
}

int best_mfma(const gemm_desc_t& d, double* cost_out) {
  int best = -1;
  double best_cost = 0;
  for (int i = 0; i < kNumConfigs; ++i) {
    const Config& c = kConfigs[i];
    if (c.kind != KIND_MFMA || !applicable(c, d)) continue;
    const double cost = mfma_cost(c, d.M, d.N, d.K, d.batch);
    if (best < 0 || cost < best_cost) { best = i; best_cost = cost; }
  }
  if (cost_out) *cost_out = best_cost;
  return best;
}

// Wave quantisation: when the 256x256 tiles of a problem fill some whole rounds of the 256
// CUs and then a partial one, give the whole rounds to the big tile and the remaining
// columns to whatever tile shape suits them best (usually 128x128, two per CU).  Returns
// the number of leading columns for the first launch, or 0 for "do not split".
int64_t split_columns(const gemm_desc_t& d, int big, double single_cost) {
  if (big < 0 || d.batch != 1) return 0;
  const Config& c = kConfigs[big];
  if (c.bm != 256 || c.bn != 256) return 0;
  const int64_t tiles_m = (d.M + c.bm - 1) / c.bm, tiles_n = (d.N + c.bn - 1) / c.bn;
  if (tiles_m > num_cus() || num_cus() % tiles_m != 0) return 0;
  const int64_t cols_per_round = num_cus() / tiles_m;
  const int64_t cols_big = tiles_n / cols_per_round * cols_per_round;
  if (cols_big == 0 || cols_big == tiles_n) return 0;
  const int64_t n_first = cols_big * c.bn;
  gemm_desc_t rest = d;
  rest.N = d.N - n_first;
  double rest_cost = 0;
  if (best_mfma(rest, &rest_cost) < 0) return 0;
  const double launch = 3.0 * 2.7e6;
  const double split_cost = mfma_cost(c, d.M, n_first, d.K, 1) + rest_cost + launch;
  // (the model is optimistic about the second launch: where it sees 7.5 %, as for 4096 x 14336 x 4096,
  // 2 - 3 % were measured; where it sees 5 % against the 256x192 tile, the single launch wins by 8 %)
  return split_cost < 0.93 * single_cost ? n_first : 0;
}

// Built-in choice.  MFMA tile: cheapest under a small cost model (wave quantisation over
// the 256 CUs, measured efficiency per tile shape); first entry of the table on ties.
int choose(const gemm_desc_t& d) {
  // skinny: up to 4 rows of x on the vector ALUs (smallest padded M that fits, first
  // such entry of the table), up to 16 on the matrix cores
  if (d.M > 1 && d.M <= 16) {
    // W through wave-private LDS slabs, x fragments straight from L2, 16x16x32 MFMA, two slabs
    // requested ahead per wave (M = 16: 24.3 us at N = K = 8192, 80 us at N = 28672; M = 4: 23.0 and
    // 72 us, where the vector-ALU kernel below needs 26 and 75 us)
    const int i = find_config("skinnydirect_d2_b512_w4");
    if (i >= 0 && applicable(kConfigs[i], d)) return i;
  }
  if (d.M <= 4) {
    // two waves per SIMD (8 per workgroup, one workgroup per CU) stream faster than one; for
    // long weight matrices two such workgroups per CU are a little better still (M = 1)
    const char* name = d.M == 1 ? (d.N >= 16384 ? "skinny_m1_w8_g2" : "skinny_m1_w8_g1")
                       : d.M == 2 ? "skinny_m2_w8_g1" : "skinny_m4_w8_g1";
    const int i = find_config(name);
    if (i >= 0 && applicable(kConfigs[i], d)) return i;
    int best = -1;
    for (int q = 0; q < kNumConfigs; ++q)
      if (kConfigs[q].kind == KIND_SKINNY && applicable(kConfigs[q], d) &&
          (best < 0 || kConfigs[q].bm < kConfigs[best].bm))
        best = q;
    if (best >= 0) return best;
  }
  const int best = best_mfma(d, nullptr);
  if (best >= 0) return best;
  // general kernels (fp32 operands, or layouts / leading dimensions the tiled kernels do not take).
  //   * fp32, at most four 16x16 tiles per CU: 16x16 tiles with K split over the waves of a workgroup
  //     (256^3: 5 us against 11 us for the next choice; 512^3: 11 to 12 against 19 us);
  //   * very few 32x32 tiles (16-bit operands in layouts the tiled kernels do not take): the vector-ALU
  //     kernel with 32x32 tiles and the long K step;
  //   * fp32 in float4 groups: the fp32-MFMA kernel with double-buffered slabs, 128x128 tiles from two
  //     tiles per CU on (4096^3: 1.13 to 1.18 ms = 116 to 122 TFLOP/s; the general kernel needs 1.47 ms),
  //     64x64 tiles below (2048^3: 184 us, 1024^3: 42 us; general kernel 219 / 53 us);
  //   * otherwise the general fp32-MFMA kernel: 64x64 tiles until there are four 128x128 tiles per CU.
  const double tiles32 = (double)((d.M + 31) / 32) * (double)((d.N + 31) / 32) * d.batch;
  const double tiles128 = (double)((d.M + 127) / 128) * (double)((d.N + 127) / 128) * d.batch;
  if (tiles32 <= 1.0 * num_cus()) {             // (tiles32 = a quarter of the 16x16 tiles)
    const int i = find_config("f32small_16x16x256");
    if (i >= 0 && applicable(kConfigs[i], d)) return i;
  }
  if (tiles32 <= 2.0 * num_cus()) return find_config("simt_32x32x64");
  {                                             // fp32 in float4 groups: 128x128 tiles from two per CU on
    const int i = find_config(tiles128 >= 2.0 * num_cus() ? "f32mfma_128x128x32" : "f32mfma_64x64x32");
    if (i >= 0 && applicable(kConfigs[i], d)) return i;
  }
  return find_config(tiles128 >= 4.0 * num_cus() ? "general_mfma32_128x128x16" : "general_mfma32_64x64x16");
}

int fill_launch_shape(gemm_plan& pl) {
  const gemm_desc_t& d = pl.d;
  const Config& c = *pl.cfg;
  pl.block = dim3(c.threads, 1, 1);
  pl.group_m = 1;
  pl.xcd_remap = 0;
  if (c.kind == KIND_SIMT || c.kind == KIND_F32_VEC) {
    const int64_t gx = (d.N + c.bn - 1) / c.bn, gy = (d.M + c.bm - 1) / c.bm;
    if (gy > 65535) return GEMM_ERR_BAD_DIM;   // grid.y / grid.z limits
    pl.grid = dim3((unsigned)gx, (unsigned)gy, (unsigned)d.batch);
  } else if (c.kind == KIND_MFMA) {
    const int64_t tm = (d.M + c.bm - 1) / c.bm, tn = (d.N + c.bn - 1) / c.bn;
    int64_t wgs = tm * tn;
    if (c.persist) {
      // as many workgroups as run at once; workgroup b takes tiles b, b + wgs, ... of all problems of the batch
      const int64_t at_once = (int64_t)num_cus() * (160 * 1024 / c.lds_bytes);
      wgs *= d.batch;
      if (wgs > at_once) wgs = at_once;
      pl.grid = dim3((unsigned)wgs, 1, 1);
    } else {
      pl.grid = dim3((unsigned)wgs, (unsigned)d.batch, 1);
    }
    pl.group_m = (int)(tm < 8 ? tm : 8);
    pl.xcd_remap = ((tm * tn) % 8 == 0) ? 1 : 0;
    // a batch on persistent workgroups: whole problems per XCD (their tiles share panels)
    if (c.persist && d.batch > 1 && (tm * tn * d.batch) % 8 == 0 && wgs % 8 == 0) pl.xcd_remap = 2;
  } else if (c.kind == KIND_SKINNY_PANEL) {
    pl.grid = dim3((unsigned)((d.N + c.bn - 1) / c.bn), (unsigned)d.batch, 1);
  } else {
    // One row of W per wave at a time, rows dealt round-robin: bn workgroups per CU,
    // more only if a wave would otherwise own more rows than the kernel has slots for.
    const int waves = c.threads / 64;
    int64_t wgs = (d.N + waves - 1) / waves;                       // one row per wave
    const int64_t want = (int64_t)num_cus() * c.bn;
    if (wgs > want) wgs = want;
    const int64_t need = (d.N + (int64_t)waves * kSkinnyMaxRows - 1) / ((int64_t)waves * kSkinnyMaxRows);
    if (wgs < need) wgs = need;
    pl.grid = dim3((unsigned)wgs, (unsigned)d.batch, 1);
  }
  return GEMM_OK;
}

// gfx950 check, once per device.
}  // namespace

// ---- C ABI -------------------------------------------------------------------------------

extern "C" {

// GEMM_LOG=1 in the environment: one line on stderr per plan, saying which kernel and tile it got.
static bool log_enabled() {
  static const bool on = [] {
    const char* e = std::getenv("GEMM_LOG");
    return e && e[0] && std::strcmp(e, "0") != 0;
  }();
  return on;
}

int gemm_config_count(void) { return kNumConfigs; }

const char* gemm_config_name(int config) {
  return (config >= 0 && config < kNumConfigs) ? kConfigs[config].name : nullptr;
}

// Plan for an already resolved descriptor.  allow_two_launches: the built-in choice may
// plan a second launch against wave quantisation.
static int create_resolved(const gemm_desc_t& d, int config, bool allow_two_launches, gemm_plan_t** out_plan) {
  if (config < -1 || config >= kNumConfigs) return GEMM_ERR_BAD_CONFIG;
  const bool auto_choice = config == -1;
  if (config == -1) config = choose(d);
  if (config < 0) return GEMM_ERR_UNSUPPORTED;
  if (!applicable(kConfigs[config], d)) return auto_choice ? GEMM_ERR_UNSUPPORTED : GEMM_ERR_BAD_CONFIG;
  gemm_plan* pl = new (std::nothrow) gemm_plan;
  if (!pl) return GEMM_ERR_NULL;
  pl->d = d;
  pl->cfg = &kConfigs[config];
  pl->cfg_index = config;
  pl->tail = nullptr;
  pl->tail_off_b = pl->tail_off_c = pl->tail_off_bias = 0;
  pl->splits = 0;
  pl->inner = nullptr;
  pl->d_user = d;
  pl->c_cached = 0;
  pl->built_in = auto_choice && allow_two_launches;   // (second launches and split-K inner plans are parts, not plans)
  pl->tune_state = 0;
  pl->tuned = nullptr;
  if (auto_choice && allow_two_launches && kConfigs[config].kind == KIND_MFMA) {
    double single_cost = 0;
    best_mfma(d, &single_cost);
    int big = -1;                                   // the first 256x256 shape of the table
    for (int i = 0; i < kNumConfigs && big < 0; ++i)
      if (kConfigs[i].kind == KIND_MFMA && kConfigs[i].bm == 256 && kConfigs[i].bn == 256 &&
          applicable(kConfigs[i], d))
        big = i;
    const int64_t n_first = split_columns(d, big, single_cost);
    if (n_first > 0) {
      config = big;
      pl->cfg = &kConfigs[config];
      pl->cfg_index = config;
      // second launch: columns n_first .. N-1 (rows of the N x K weight matrix, columns of C)
      gemm_desc_t rest = d;
      rest.N = d.N - n_first;
      gemm_plan_t* tail = nullptr;
      if (create_resolved(rest, best_mfma(rest, nullptr), false, &tail) == GEMM_OK) {
        pl->tail = tail;
        pl->tail_off_b = n_first * d.ldb;
        pl->tail_off_c = n_first;
        pl->tail_off_bias = n_first;
        pl->d.N = n_first;
      }
    }
  }
  const int rc = fill_launch_shape(*pl);
  if (rc != GEMM_OK) { gemm_destroy(pl); return rc; }
  *out_plan = pl;
  if (allow_two_launches && log_enabled()) {     // (second launches and split-K inner plans are reported with their parent)
    char buf[512];
    gemm_plan_info(pl, buf, sizeof(buf));
    std::fprintf(stderr, "[mi355gemm] plan %lld x %lld x %lld batch %d dtype %d -> %d epilogue %d: %s\n", (long long)d.M,
                 (long long)d.N, (long long)d.K, (int)d.batch, (int)d.dtype_a, (int)d.dtype_c, (int)d.epilogue, buf);
  }
  return GEMM_OK;
}

int gemm_create_config(const gemm_desc_t* desc, int config, gemm_plan_t** out_plan) {
  if (out_plan) *out_plan = nullptr;
  if (!desc || !out_plan) return GEMM_ERR_NULL;
  gemm_desc_t d;
  const int rc = resolve(desc, &d);
  if (rc != GEMM_OK) return rc;
  return create_resolved(d, config, true, out_plan);
}

// Slices of K for a split-K plan: the count (up to 64, K a multiple of 8 x slices, whole
// slabs per slice preferred) that minimises the tile cost model of the sliced product plus
// the traffic of the fp32 partials (written once, read once: priced at 2 TB/s; in the model's units
// one microsecond is 2.7e6).  512x512x32768 takes 46 / 31 / 29 / 38 us with 8 / 16 / 32 / 64 slices;
// the model picks 16.
static int choose_splits(const gemm_desc_t& d) {
  int best = 1;
  double best_cost = 0;
  for (int pass = 0; pass < 2 && best_cost == 0; ++pass) {
    const int64_t epc = 16 / esize(d.dtype_a);
    const int64_t unit = pass == 0 ? 8 * epc : epc;          // whole slabs, else whole 16-byte pieces
    for (int64_t s = 1; s <= 64; ++s) {
      if (d.K % (s * unit) != 0) continue;
      gemm_desc_t in = d;
      in.K = d.K / s;
      in.batch = (int32_t)s;
      in.stride_a = in.stride_b = in.K;
      double cost = 0;
      if (best_mfma(in, &cost) < 0) continue;
      cost += 2.0 * (double)s * (double)d.M * (double)d.N * 4.0 * (2.7e6 / 2.0e6);
      if (best_cost == 0 || cost < best_cost) { best = (int)s; best_cost = cost; }
    }
  }
  return best;
}

int gemm_create_splitk(const gemm_desc_t* desc, int splits, gemm_plan_t** out_plan) {
  if (out_plan) *out_plan = nullptr;
  if (!desc || !out_plan) return GEMM_ERR_NULL;
  gemm_desc_t d;
  int rc = resolve(desc, &d);
  if (rc != GEMM_OK) return rc;
  if (splits < 0 || splits > 1024) return GEMM_ERR_BAD_DIM;
  if (d.batch != 1 || d.dtype_a == GEMM_F32) return GEMM_ERR_UNSUPPORTED;
  if (d.layout_a != GEMM_ROW_MAJOR || d.layout_b != GEMM_COL_MAJOR) return GEMM_ERR_UNSUPPORTED;
  if (splits == 0) splits = choose_splits(d);
  if (d.K % ((int64_t)splits * (16 / esize(d.dtype_a))) != 0) return GEMM_ERR_UNSUPPORTED;
  if ((double)splits * (double)d.M * (double)d.N * 4.0 >= 9.0e18) return GEMM_ERR_BAD_DIM;
  // the K slices as the batches of a product into packed fp32 partials, no epilogue
  gemm_desc_t in = d;
  in.K = d.K / splits;
  in.batch = splits;
  in.stride_a = in.K;                 // slice s of A starts K/splits columns further on
  in.stride_b = in.K;
  in.dtype_c = GEMM_F32;
  in.layout_c = GEMM_ROW_MAJOR;
  in.ldc = d.N;
  in.stride_c = d.M * d.N;
  in.epilogue = GEMM_EPI_NONE;
  in.stride_bias = 0;
  in.scale = 1.0f;
  const int inner_cfg = best_mfma(in, nullptr);
  if (inner_cfg < 0) return GEMM_ERR_UNSUPPORTED;
  gemm_plan_t* inner = nullptr;
  rc = create_resolved(in, inner_cfg, false, &inner);
  if (rc != GEMM_OK) return rc;
  inner->c_cached = 1;                // the reduction kernel reads the partials next
  if (inner->tail) inner->tail->c_cached = 1;
  gemm_plan* pl = new (std::nothrow) gemm_plan(*inner);
  if (!pl) { gemm_destroy(inner); return GEMM_ERR_NULL; }
  pl->d = d;
  pl->d_user = d;
  pl->built_in = 0;
  pl->splits = splits;
  pl->inner = inner;
  *out_plan = pl;
  return GEMM_OK;
}

size_t gemm_workspace_bytes(const gemm_plan_t* plan) {
  if (!plan || !plan->inner) return 0;
  return (size_t)plan->splits * (size_t)plan->d.M * (size_t)plan->d.N * 4;
}

int gemm_run_workspace(const gemm_plan_t* plan, const void* A, const void* B, void* C,
                       const void* bias, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!plan) return GEMM_ERR_NULL;
  if (!plan->inner) return gemm_run(plan, A, B, C, bias, hip_stream);
  if (!A || !B || !C) return GEMM_ERR_NULL;
  const gemm_desc_t& d = plan->d;
  if (epilogue_has_bias(d.epilogue) != (bias != nullptr)) return GEMM_ERR_NULL;
  if (!workspace || workspace_bytes < gemm_workspace_bytes(plan) || ((uintptr_t)workspace & 15))
    return GEMM_ERR_WORKSPACE;
  if (((uintptr_t)C & ((uintptr_t)esize(d.dtype_c) - 1)) || ((uintptr_t)bias & 3)) return GEMM_ERR_MISALIGNED;
  int rc = gemm_run(plan->inner, A, B, workspace, nullptr, hip_stream);
  if (rc != GEMM_OK) return rc;
  SplitKReduceArgs r;
  r.ws = (const float*)workspace; r.C = C; r.bias = (const float*)bias;
  r.M = d.M; r.N = d.N;
  r.c_si = d.layout_c == GEMM_ROW_MAJOR ? d.ldc : 1;
  r.c_sj = d.layout_c == GEMM_ROW_MAJOR ? 1 : d.ldc;
  r.splits = plan->splits;
  r.has_bias = epilogue_has_bias(d.epilogue);
  r.act = epilogue_activation(d.epilogue);
  r.scale = d.scale;
  const int64_t quads = d.M * ((d.N + 3) / 4);
  const int64_t blocks = (quads + 255) / 256;
  if (blocks >= ((int64_t)1 << 31)) return GEMM_ERR_BAD_DIM;
  hipStream_t s = (hipStream_t)hip_stream;
  switch (d.dtype_c) {
    case GEMM_F32: splitk_reduce_kernel<float><<<(unsigned)blocks, 256, 0, s>>>(r); break;
    case GEMM_BF16: splitk_reduce_kernel<bf16_t><<<(unsigned)blocks, 256, 0, s>>>(r); break;
    default: splitk_reduce_kernel<f16_t><<<(unsigned)blocks, 256, 0, s>>>(r); break;
  }
  return hipGetLastError() == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}

// ---- the fixed scratch buffer -----------------------------------------------------------------
// Device memory inside the code object: each GPU the library is loaded on has its own copy at
// its own address.  In host code the array's name is only a handle for hipGetSymbolAddress;
// the address it returns (per device, looked up once with that device current) is what kernels
// and launches are given.
static __device__ __align__(256) unsigned char g_fixed_scratch[GEMM_FIXED_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of the buffer, or nullptr.
void* fixed_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_fixed_scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

int gemm_run_fixed_scratch(const gemm_plan_t* plan, const void* A, const void* B, void* C,
                           const void* bias, void* hip_stream) {
  if (!plan) return GEMM_ERR_NULL;
  if (!plan->inner) return gemm_run(plan, A, B, C, bias, hip_stream);
  const size_t need = gemm_workspace_bytes(plan);
  if (need > GEMM_FIXED_SCRATCH_BYTES) return GEMM_ERR_FIXED_SCRATCH;
  int rc = check_device_gfx950();
  if (rc != GEMM_OK) return rc;
  void* ws = fixed_scratch_of_current_device();
  if (!ws) return GEMM_ERR_LAUNCH;
  return gemm_run_workspace(plan, A, B, C, bias, ws, GEMM_FIXED_SCRATCH_BYTES, hip_stream);
}

int gemm_create(const gemm_desc_t* desc, gemm_plan_t** out_plan) {
  return gemm_create_config(desc, -1, out_plan);
}

// The launches of one plan, arguments checked; no tuning logic.
static int run_plan(const gemm_plan_t* plan, const void* A, const void* B, void* C, const void* bias,
                    void* hip_stream) {
  if (!plan || !A || !B || !C) return GEMM_ERR_NULL;
  if (plan->inner) return GEMM_ERR_WORKSPACE;
  const gemm_desc_t& d = plan->d;
  if (epilogue_has_bias(d.epilogue) != (bias != nullptr)) return GEMM_ERR_NULL;
  // The tiled 16-bit kernels move 16-byte pieces; the general kernel only needs
  // element alignment.
  const uintptr_t in_mask = plan->cfg->kind == KIND_SIMT || plan->cfg->kind == KIND_F32_VEC ? (uintptr_t)esize(d.dtype_a) - 1 : 15;
  if (((uintptr_t)A & in_mask) || ((uintptr_t)B & in_mask) ||
      ((uintptr_t)C & ((uintptr_t)esize(d.dtype_c) - 1)) || ((uintptr_t)bias & 3))
    return GEMM_ERR_MISALIGNED;
  int rc = check_device_gfx950();
  if (rc != GEMM_OK) return rc;
  hipError_t e = plan->cfg->launch[d.dtype_a](*plan, A, B, C, bias, (hipStream_t)hip_stream);
  if (e != hipSuccess) return GEMM_ERR_LAUNCH;
  if (plan->tail) {
    const gemm_plan* t = plan->tail;
    const char* B2 = (const char*)B + plan->tail_off_b * esize(d.dtype_b);
    char* C2 = (char*)C + plan->tail_off_c * esize(d.dtype_c);
    const float* bias2 = bias ? (const float*)bias + plan->tail_off_bias : nullptr;
    e = t->cfg->launch[d.dtype_a](*t, A, B2, C2, bias2, (hipStream_t)hip_stream);
    if (e != hipSuccess) return GEMM_ERR_LAUNCH;
  }
  return GEMM_OK;
}

// Mean microseconds per launch of one plan under the paper's timing protocol (App.
// "Benchmarking kernel runtime"): a few initial trials size the loops, a warm-up of at least
// min_seconds and 10 launches, then inner loops of >= min(0.01 s, min_seconds) between two
// event synchronisations until at least min_seconds and 10 launches have been measured.
static int time_plan(const gemm_plan_t* pl, const void* A, const void* B, void* C, const void* bias,
                     void* hip_stream, hipEvent_t e0, hipEvent_t e1, double min_seconds, double* us) {
  hipStream_t stream = (hipStream_t)hip_stream;
  int status = GEMM_OK;
  // n launches between two events; returns elapsed seconds (< 0 on failure)
  auto timed = [&](long n) -> double {
    if (hipEventRecord(e0, stream) != hipSuccess) return -1.0;
    for (long i = 0; i < n; ++i) {
      int r = run_plan(pl, A, B, C, bias, hip_stream);
      if (r != GEMM_OK) { status = r; return -1.0; }
    }
    if (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1.0;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.0;
    return (double)ms * 1e-3;
  };
  auto failed = [&]() { return status != GEMM_OK ? status : GEMM_ERR_LAUNCH; };
  const double inner_s = min_seconds < 0.01 ? min_seconds : 0.01;
  double t = timed(3);                                   // initial trials: rough runtime
  if (t < 0) return failed();
  const double per = t / 3 > 1e-7 ? t / 3 : 1e-7;
  const long inner = (long)(inner_s / per) + 1;
  long warm = (long)(min_seconds / per) + 1;             // warm-up: at least min_seconds and 10 launches
  if (warm < 10) warm = 10;
  if (timed(warm) < 0) return failed();
  double total = 0.0;
  long launches = 0;
  while (total < min_seconds || launches < 10) {
    const double dt = timed(inner);
    if (dt < 0) return failed();
    total += dt;
    launches += inner;
  }
  *us = total / (double)launches * 1e6;
  return GEMM_OK;
}

int gemm_tune(const gemm_desc_t* desc, const void* A, const void* B, void* C, const void* bias,
              void* hip_stream, double min_seconds, int* best_config, float* us_per_config) {
  if (!desc || !A || !B || !C || !best_config) return GEMM_ERR_NULL;
  *best_config = -1;
  gemm_desc_t d;
  int rc = resolve(desc, &d);
  if (rc != GEMM_OK) return rc;
  if (!(min_seconds >= 0.0)) min_seconds = 0.0;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) { (void)hipGetLastError(); return GEMM_ERR_LAUNCH; }
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipGetLastError(); (void)hipEventDestroy(e0); return GEMM_ERR_LAUNCH; }
  double best_us = 0.0;
  int status = GEMM_OK;
  for (int i = 0; i < kNumConfigs && status == GEMM_OK; ++i) {
    if (us_per_config) us_per_config[i] = -1.0f;
    if (!applicable(kConfigs[i], d)) continue;
    gemm_plan_t* pl = nullptr;
    if (create_resolved(d, i, true, &pl) != GEMM_OK) continue;
    double us = 0.0;
    status = time_plan(pl, A, B, C, bias, hip_stream, e0, e1, min_seconds, &us);
    gemm_destroy(pl);
    if (status != GEMM_OK) break;
    if (us_per_config) us_per_config[i] = (float)us;
    if (*best_config < 0 || us < best_us) { *best_config = i; best_us = us; }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (status != GEMM_OK) { (void)hipGetLastError(); return status; }
  return *best_config >= 0 ? GEMM_OK : GEMM_ERR_UNSUPPORTED;
}

// ---- tuning mode --------------------------------------------------------------------------
// The paper's parameter optimisation (Sec. 3.4) as a switch: with it on, the first gemm_run of
// a problem times every applicable instantiation and the built-in plan on the caller's own
// buffers and remembers the winner per problem for the rest of the process.
namespace {

struct TuneKey {
  int64_t v[17];
  bool operator<(const TuneKey& o) const { return std::memcmp(v, o.v, sizeof(v)) < 0; }
};
TuneKey tune_key(const gemm_desc_t& d) {                 // everything but the epilogue's scalar
  TuneKey k;
  const int64_t f[17] = {d.M, d.N, d.K, d.batch, d.layout_a, d.layout_b, d.layout_c, d.dtype_a, d.dtype_b,
                         d.dtype_c, d.epilogue, d.lda, d.ldb, d.ldc, d.stride_a, d.stride_b, d.stride_c};
  std::memcpy(k.v, f, sizeof(f));
  return k;
}
std::mutex g_tune_mutex;
std::map<TuneKey, int> g_tune_cache;                     // problem -> fastest configuration, -1 = the built-in plan
std::atomic<int> g_autotune{-1};                         // -1: not yet read from the environment
constexpr double kAutotuneSeconds = 0.02;                // per configuration: warm-up and measurement each

bool autotune_on() {
  int v = g_autotune.load();
  if (v < 0) {
    const char* e = std::getenv("GEMM_TUNE");
    int from_env = (e && e[0] && std::strcmp(e, "0") != 0) ? 1 : 0;
    int expected = -1;
    g_autotune.compare_exchange_strong(expected, from_env);
    v = g_autotune.load();
  }
  return v == 1;
}

// Decide how `plan` runs from now on (tune_state 1: as it is; 2: through plan->tuned).
int autotune_plan(const gemm_plan_t* plan, const void* A, const void* B, void* C, const void* bias,
                  void* hip_stream) {
  gemm_plan_t* self = const_cast<gemm_plan_t*>(plan);    // only the two set-once tuning fields are written
  const gemm_desc_t& d = plan->d_user;
  std::lock_guard<std::mutex> lock(g_tune_mutex);         // one tuning run at a time; later callers find the entry
  if (__atomic_load_n(&self->tune_state, __ATOMIC_ACQUIRE) != 0) return GEMM_OK;
  int cfg = -1;
  const TuneKey key = tune_key(d);
  auto it = g_tune_cache.find(key);
  if (it != g_tune_cache.end()) {
    cfg = it->second;
  } else {
    int best = -1;
    std::vector<float> us(kNumConfigs, -1.0f);
    int rc = gemm_tune(&d, A, B, C, bias, hip_stream, kAutotuneSeconds, &best, us.data());
    if (rc != GEMM_OK) return rc;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) { (void)hipGetLastError(); return GEMM_ERR_LAUNCH; }
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipGetLastError(); (void)hipEventDestroy(e0); return GEMM_ERR_LAUNCH; }
    double own = 0.0;
    rc = time_plan(plan, A, B, C, bias, hip_stream, e0, e1, kAutotuneSeconds, &own);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != GEMM_OK) { (void)hipGetLastError(); return rc; }
    // a configuration replaces the built-in plan only for a clear win
    const bool same = best == plan->cfg_index && !plan->tail;
    cfg = (!same && (double)us[best] < 0.98 * own) ? best : -1;
    g_tune_cache[key] = cfg;
  }
  if (cfg >= 0 && !(cfg == plan->cfg_index && !plan->tail)) {
    gemm_plan_t* tp = nullptr;
    const int rc = create_resolved(d, cfg, true, &tp);
    if (rc != GEMM_OK) return rc;
    tp->built_in = 0;
    self->tuned = tp;
    __atomic_store_n(&self->tune_state, 2, __ATOMIC_RELEASE);
  } else {
    __atomic_store_n(&self->tune_state, 1, __ATOMIC_RELEASE);
  }
  return GEMM_OK;
}

}  // namespace

int gemm_set_autotune(int enabled) {
  const int before = autotune_on() ? 1 : 0;
  g_autotune.store(enabled ? 1 : 0);
  return before;
}

int gemm_autotune_entries(void) {
  std::lock_guard<std::mutex> lock(g_tune_mutex);
  return (int)g_tune_cache.size();
}

int gemm_autotune_clear(void) {
  std::lock_guard<std::mutex> lock(g_tune_mutex);
  g_tune_cache.clear();
  return GEMM_OK;
}

int gemm_run(const gemm_plan_t* plan, const void* A, const void* B, void* C, const void* bias,
             void* hip_stream) {
  if (plan && plan->built_in && !plan->inner && autotune_on()) {
    int state = __atomic_load_n(&plan->tune_state, __ATOMIC_ACQUIRE);
    if (state == 0) {
      // arguments are checked before anything is timed with them
      if (!A || !B || !C) return GEMM_ERR_NULL;
      if (epilogue_has_bias(plan->d.epilogue) != (bias != nullptr)) return GEMM_ERR_NULL;
      if (((uintptr_t)A & 15) || ((uintptr_t)B & 15) || ((uintptr_t)C & 15) || ((uintptr_t)bias & 3))
        return run_plan(plan, A, B, C, bias, hip_stream);   // (unusual alignment: no tuning, the plan's own checks decide)
      const int rc = autotune_plan(plan, A, B, C, bias, hip_stream);
      if (rc != GEMM_OK) return rc;
      state = __atomic_load_n(&plan->tune_state, __ATOMIC_ACQUIRE);
    }
    if (state == 2) return run_plan(plan->tuned, A, B, C, bias, hip_stream);
  }
  return run_plan(plan, A, B, C, bias, hip_stream);
}

int gemm_destroy(gemm_plan_t* plan) {
  if (plan) {
    if (plan->inner) {                 // a split-K plan is a copy of its inner plan's launch data
      gemm_destroy(plan->inner);
    } else {
      delete plan->tail;
      if (plan->built_in && plan->tuned) gemm_destroy(plan->tuned);
    }
  }
  delete plan;
  return GEMM_OK;
}

const char* gemm_status_string(int status) {
  switch (status) {
    case GEMM_OK: return "ok";
    case GEMM_ERR_NULL: return "null pointer (or bias does not match the epilogue)";
    case GEMM_ERR_BAD_DIM: return "bad dimension";
    case GEMM_ERR_BAD_LD: return "bad leading dimension or batch stride";
    case GEMM_ERR_UNSUPPORTED: return "unsupported dtype / layout / epilogue combination";
    case GEMM_ERR_MISALIGNED: return "misaligned pointer";
    case GEMM_ERR_NO_DEVICE: return "current device is not a gfx950 GPU";
    case GEMM_ERR_LAUNCH: return "kernel launch failed";
    case GEMM_ERR_BAD_ENUM: return "enum value out of range";
    case GEMM_ERR_BAD_CONFIG: return "tile configuration unknown or not applicable";
    case GEMM_ERR_BAD_SCALE: return "epilogue scale is not finite";
    case GEMM_ERR_WORKSPACE: return "plan needs a workspace (gemm_run_workspace), or the workspace is too small or misaligned";
    case GEMM_ERR_FIXED_SCRATCH: return "plan needs more workspace than the library's fixed scratch buffer of 32 MiB (use gemm_run_workspace)";
    default: return "unknown status";
  }
}

int gemm_plan_info(const gemm_plan_t* plan, char* buf, size_t n) {
  if (!plan || (!buf && n)) return GEMM_ERR_NULL;
  if (plan->built_in && __atomic_load_n(&plan->tune_state, __ATOMIC_ACQUIRE) == 2) {
    // timed in tuning mode and replaced: report what runs
    const int len = gemm_plan_info(plan->tuned, buf, n);
    if (len < 0) return len;
    const char* tag = " (tuned)";
    if (buf && (size_t)len < n) std::snprintf(buf + len, n - (size_t)len, "%s", tag);
    return len + (int)std::strlen(tag);
  }
  const Config& c = *plan->cfg;
  if (plan->inner) {
    return std::snprintf(buf, n, "kernel=splitk_%d+%s tile=%dx%dx%d grid=%u,%u,%u block=%u lds=%d workspace=%zu",
                         plan->splits, c.name, c.bm, c.bn, c.bk, plan->grid.x, plan->grid.y, plan->grid.z,
                         plan->block.x, c.lds_bytes, gemm_workspace_bytes(plan));
  }
  if (plan->tail) {
    const Config& t = *plan->tail->cfg;
    return std::snprintf(buf, n, "kernel=%s tile=%dx%dx%d grid=%u,%u,%u block=%u lds=%d columns=0..%lld "
                         "+ kernel=%s grid=%u,%u,%u columns=%lld..", c.name, c.bm, c.bn, c.bk,
                         plan->grid.x, plan->grid.y, plan->grid.z, plan->block.x, c.lds_bytes,
                         (long long)plan->d.N - 1, t.name, plan->tail->grid.x, plan->tail->grid.y,
                         plan->tail->grid.z, (long long)plan->d.N);
  }
  return std::snprintf(buf, n, "kernel=%s tile=%dx%dx%d grid=%u,%u,%u block=%u lds=%d", c.name,
                       c.bm, c.bn, c.bk, plan->grid.x, plan->grid.y, plan->grid.z, plan->block.x,
                       c.lds_bytes);
}

}  // extern "C"
