/*
 * Reference (oracle) rotary positional embedding, on the CPU, in fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  The slow, plain definition that the GPU kernel is
 * checked against.  It shares no code with the GPU library and must never be
 * called from it.
 *
 * The operation is the one of the paper's language-model case study (Sec. 4,
 * "Case study": the rotary positional embedding function of a Llama model, with
 * the PyTorch implementation "apply_rotary_pos_emb, combining unsqueeze +
 * rotate-half" as the reference).  The paper prints no formula; the rotate-half
 * form is, for a head vector x of even length D and per-position tables cos, sin
 * of length D (broadcast over the heads: the "unsqueeze"):
 *
 *   rot(x)[i] = -x[i + D/2]   for i <  D/2
 *   rot(x)[i] =  x[i - D/2]   for i >= D/2
 *   y[i]      = x[i] * cos[i] + rot(x)[i] * sin[i]
 *
 * Every index uses its own table entry (tables whose two halves repeat, as a
 * language model builds them, make this a plane rotation of each pair
 * (x[i], x[i + D/2]) by the angle of position s).
 *
 * x, y: logical shape [batch, heads, seq, D], element (b,h,s,i) at
 *   b*stride_b + h*stride_h + s*stride_s + i   (in elements of the storage type).
 * cos, sin: [seq, D] shared by all batches (table_stride_b == 0) or [batch, seq, D]
 *   (table_stride_b = elements between batches), entry (b,s,i) at b*table_stride_b + s*D + i.
 * Stored elements (fp32, bf16 or fp16 bit patterns) are converted exactly to fp64;
 * the result stays in fp64.
 */
#ifndef ORACLE_REF_ROPE_H
#define ORACLE_REF_ROPE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t batch, heads, seq, head_dim;       /* head_dim even */
  int32_t dtype_x;                           /* 0 fp32, 1 bf16, 2 fp16 (as in ref_gemm.h) */
  int32_t dtype_table;
  int64_t stride_b, stride_h, stride_s;      /* of x, in elements (never 0 here) */
  int64_t table_stride_b;                    /* 0 = one table for all batches */
} ref_rope_t;

/* y: room for batch*heads*seq*head_dim doubles, packed [batch, heads, seq, D].
 * Returns 0, or -1 on a bad argument. */
int ref_rope(const ref_rope_t* p, const void* x, const void* cos_t, const void* sin_t, double* y);

#ifdef __cplusplus
}
#endif
#endif
