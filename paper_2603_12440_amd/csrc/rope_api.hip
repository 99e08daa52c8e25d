// C ABI of the rotary positional embedding: argument checks, choice between the 16-byte
// and the element-wise kernel, one launch.  gfx950 only.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "../../include/rope.h"
#include "common.hpp"
#include "device_check.hpp"
#include "rope_kernel.hpp"

using namespace mi355gemm;

namespace {

int esize_of(int dtype) { return dtype == GEMM_F32 ? 4 : 2; }

// group = lanes per position of the fast kernels (32 or 64; negative: the exchange kernel),
// or 0 for the general kernel
template <typename T, typename TT>
hipError_t launch_rope(const RopeArgs& a, bool vec, int group, unsigned grid, hipStream_t s) {
  if (group == -32) rope_exchange_kernel<T, TT, 32><<<grid, 256, 0, s>>>(a);
  else if (group == -64) rope_exchange_kernel<T, TT, 64><<<grid, 256, 0, s>>>(a);
  else if (group == 32) rope_group_kernel<T, TT, 32><<<grid, 256, 0, s>>>(a);
  else if (group == 64) rope_group_kernel<T, TT, 64><<<grid, 256, 0, s>>>(a);
  else if (vec) rope_kernel<T, TT, 8><<<grid, 256, 0, s>>>(a);
  else rope_kernel<T, TT, 1><<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_rope_tables(const RopeArgs& a, bool f32_tables, bool vec, int group, unsigned grid,
                              hipStream_t s) {
  if constexpr (std::is_same<T, float>::value) {
    return launch_rope<float, float>(a, vec, group, grid, s);
  } else {
    return f32_tables ? launch_rope<T, float>(a, vec, group, grid, s)
                      : launch_rope<T, T>(a, vec, group, grid, s);
  }
}

}  // namespace

extern "C" int rope_apply(const rope_desc_t* desc, const rope_tensor_t* tensors, int n_tensors,
                          const void* cos_table, const void* sin_table, void* hip_stream) {
  if (!desc || !tensors || !cos_table || !sin_table) return GEMM_ERR_NULL;
  if (n_tensors < 1 || n_tensors > 2) return GEMM_ERR_BAD_DIM;
  const rope_desc_t& d = *desc;
  if (d.dtype < GEMM_F32 || d.dtype > GEMM_F16 || d.table_dtype < GEMM_F32 || d.table_dtype > GEMM_F16)
    return GEMM_ERR_BAD_ENUM;
  if (d.table_dtype != GEMM_F32 && d.table_dtype != d.dtype) return GEMM_ERR_UNSUPPORTED;
  const int64_t kMax = (int64_t)1 << 30;
  if (d.batch < 1 || d.seq < 1 || d.head_dim < 2 || (d.head_dim & 1) || d.batch > kMax || d.seq > kMax ||
      d.head_dim > 65536 || d.batch * d.seq >= ((int64_t)1 << 31))
    return GEMM_ERR_BAD_DIM;
  if (d.table_stride_b < 0 || (d.table_stride_b != 0 && d.table_stride_b < d.seq * d.head_dim))
    return GEMM_ERR_BAD_LD;

  const int es = esize_of(d.dtype), ts = esize_of(d.table_dtype);
  const int64_t D = d.head_dim;
  RopeArgs a{};
  a.cos = cos_table; a.sin = sin_table;
  a.table_stride_b = d.table_stride_b;
  a.positions = d.batch * d.seq;
  a.seq = (int)d.seq; a.head_dim = (int)D;
  a.n_tensors = n_tensors;
  if (((uintptr_t)cos_table % ts) || ((uintptr_t)sin_table % ts)) return GEMM_ERR_MISALIGNED;

  // 16-byte path: whole 8-element chunks in each half, every row start on a 16-byte boundary
  const int vec_elems = 16 / es;                              // storage elements per 16 bytes
  bool vec = (D % 16 == 0) && ((uintptr_t)cos_table % 16 == 0) && ((uintptr_t)sin_table % 16 == 0) &&
             (d.table_stride_b % (16 / ts) == 0);
  int64_t heads_total = 0;
  for (int i = 0; i < n_tensors; ++i) {
    const rope_tensor_t& t = tensors[i];
    if (!t.x || !t.y) return GEMM_ERR_NULL;
    if (t.heads < 1 || t.heads > 65536) return GEMM_ERR_BAD_DIM;
    int64_t xs[3] = {t.x_stride_b, t.x_stride_h, t.x_stride_s};
    int64_t ys[3] = {t.y_stride_b, t.y_stride_h, t.y_stride_s};
    for (int64_t* st : {xs, ys}) {
      if (st[0] < 0 || st[1] < 0 || st[2] < 0) return GEMM_ERR_BAD_LD;
      const int given = (st[0] != 0) + (st[1] != 0) + (st[2] != 0);
      if (given == 0) {                                       // packed [batch, heads, seq, D]
        st[2] = D; st[1] = d.seq * D; st[0] = t.heads * d.seq * D;
      } else if (st[1] == 0 || st[2] == 0 || (st[0] == 0 && d.batch > 1)) {
        return GEMM_ERR_BAD_LD;                               // all of them, or none
      }
      if (st[1] < D && t.heads > 1) return GEMM_ERR_BAD_LD;   // head vectors must not overlap
      if (st[2] < D && d.seq > 1) return GEMM_ERR_BAD_LD;
    }
    if (((uintptr_t)t.x % es) || ((uintptr_t)t.y % es)) return GEMM_ERR_MISALIGNED;
    RopeTensorArgs& o = a.t[i];
    o.x = t.x; o.y = t.y; o.heads = (int)t.heads;
    o.xb = xs[0]; o.xh = xs[1]; o.xs = xs[2];
    o.yb = ys[0]; o.yh = ys[1]; o.ys = ys[2];
    for (int q = 0; q < 3; ++q) vec = vec && (xs[q] % vec_elems == 0) && (ys[q] % vec_elems == 0);
    vec = vec && ((uintptr_t)t.x % 16 == 0) && ((uintptr_t)t.y % 16 == 0);
    heads_total += t.heads;
  }
  a.chunks = vec ? (int)(D / 16) : (int)(D / 2);
  a.items0 = a.t[0].heads * a.chunks;
  const int64_t items_pos = heads_total * a.chunks;
  if (items_pos >= ((int64_t)1 << 24)) return GEMM_ERR_BAD_DIM;
  a.items_pos = (int)items_pos;
  // a workgroup takes enough consecutive positions for about four passes of its 256 lanes
  int ppb = (int)(1024 / items_pos);
  if (ppb < 1) ppb = 1;
  a.pos_per_block = ppb;
  int64_t grid = (a.positions + ppb - 1) / ppb;
  // fast kernel: a group of 32 (or 64) lanes per position, when a head vector's chunks divide it
  // A half of at least 128 bytes already gives whole-line accesses with one lane per pair of
  // chunks; shorter halves (power-of-two chunk counts) go to the exchange kernel, where a lane
  // owns one chunk of the whole head vector.
  int group = 0;
  if (vec) {
    const bool pow2 = (a.chunks & (a.chunks - 1)) == 0;
    const bool long_half = (D / 2) * es >= 128;
    if (long_half && 32 % a.chunks == 0) group = 32;
    else if (long_half && 64 % a.chunks == 0) group = 64;
    else if (pow2 && 2 * a.chunks <= 32) group = -32;
    else if (pow2 && 2 * a.chunks <= 64) group = -64;
  }
  if (group) {
    const int lanes = group < 0 ? -group : group;
    grid = (a.positions * lanes + 255) / 256;
    if (grid >= ((int64_t)1 << 31)) group = 0, grid = (a.positions + ppb - 1) / ppb;
  }

  int rc = check_device_gfx950();
  if (rc != GEMM_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  const bool f32_tables = d.table_dtype == GEMM_F32;
  hipError_t e;
  switch (d.dtype) {
    case GEMM_F32: e = launch_rope_tables<float>(a, true, vec, group, (unsigned)grid, s); break;
    case GEMM_BF16: e = launch_rope_tables<bf16_t>(a, f32_tables, vec, group, (unsigned)grid, s); break;
    default: e = launch_rope_tables<f16_t>(a, f32_tables, vec, group, (unsigned)grid, s); break;
  }
  return e == hipSuccess ? GEMM_OK : GEMM_ERR_LAUNCH;
}
