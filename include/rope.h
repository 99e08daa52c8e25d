/*
 * Rotary positional embedding (rotate-half form) for AMD MI355X (gfx950), in the same
 * shared library as the GEMM entry points (include/gemm.h; its dtype enum and status
 * codes are used here).
 *
 * The operation is the rotary embedding of the paper's language-model case study (Sec. 4,
 * case study on a Llama-style model): the rotate-half form, with per-position tables that
 * are broadcast over the heads.  For every head vector x (even length D) at position s of
 * batch b, with per-position tables cos, sin of length D that are shared by all heads:
 *
 *     rot(x)[i] = -x[i + D/2]  (i < D/2),    rot(x)[i] = x[i - D/2]  (i >= D/2)
 *     y[i]      = x[i] * cos[i] + rot(x)[i] * sin[i]
 *
 * Every index uses its own table entry.  Arithmetic is fp32 (one fused multiply-add per
 * output on top of one product), rounded once, to nearest even, to the storage type.
 *
 * Plain C ABI; all tensor and table pointers are DEVICE pointers, descriptors live on the
 * HOST.  Nothing is allocated and no state is kept; the call enqueues one kernel and
 * returns without waiting.
 */
#ifndef MI355GEMM_ROPE_H
#define MI355GEMM_ROPE_H

#include "gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* What all tensors of one call share. */
typedef struct {
  int64_t batch, seq, head_dim;      /* >= 1; head_dim even */
  int32_t dtype;                     /* gemm_dtype_t: storage type of x and y */
  int32_t table_dtype;               /* GEMM_F32, or the same as dtype */
  int64_t table_stride_b;            /* elements between the tables of consecutive batches;
                                        0 = one [seq, head_dim] table for every batch */
} rope_desc_t;

/*
 * One tensor to rotate: logical shape [batch, heads, seq, head_dim], element (b,h,s,i) at
 *   b*stride_b + h*stride_h + s*stride_s + i     (elements of the storage type).
 * All three strides 0 means packed in that order.  A query tensor as a projection leaves
 * it ([batch, seq, heads, head_dim] in memory) is stride_b = seq*heads*D, stride_h = D,
 * stride_s = heads*D.  y may be x itself (same strides: in place) or must not overlap it.
 * x is only read, y only written; both stay owned by the caller.
 */
typedef struct {
  const void* x;
  void* y;
  int64_t heads;
  int64_t x_stride_b, x_stride_h, x_stride_s;
  int64_t y_stride_b, y_stride_h, y_stride_s;
} rope_tensor_t;

/*
 * rope_apply - rotate n_tensors (1 or 2: e.g. the query and the key tensor of a layer,
 * which share positions and tables) in ONE kernel launch on `hip_stream` (a hipStream_t
 * cast to void*; NULL = the default stream) of the current device.
 * cos, sin: [seq, head_dim] (or [batch, seq, head_dim] with table_stride_b), row s at
 * b*table_stride_b + s*head_dim, of type table_dtype.
 * Returns GEMM_OK or a negative status of gemm.h: GEMM_ERR_NULL, GEMM_ERR_BAD_DIM (sizes
 * out of range, odd head_dim, n_tensors not 1 or 2), GEMM_ERR_BAD_LD (negative strides, or
 * only some of a tensor's strides given), GEMM_ERR_BAD_ENUM, GEMM_ERR_UNSUPPORTED (table
 * type neither fp32 nor the tensors' type), GEMM_ERR_MISALIGNED (a pointer not aligned to
 * its element size), GEMM_ERR_NO_DEVICE, GEMM_ERR_LAUNCH.
 */
int rope_apply(const rope_desc_t* desc, const rope_tensor_t* tensors, int n_tensors,
               const void* cos_table, const void* sin_table, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MI355GEMM_ROPE_H */
