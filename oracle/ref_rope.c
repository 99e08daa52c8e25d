/* Rotary positional embedding, rotate-half form, in fp64.  See ref_rope.h.
 * TEST INFRASTRUCTURE ONLY. */
#include "ref_rope.h"
#include "ref_gemm.h"   /* the storage decoders */

#include <stddef.h>

static double load_elem(const void* base, int32_t dtype, int64_t idx) {
  switch (dtype) {
    case REF_F32: return (double)((const float*)base)[idx];
    case REF_BF16: return ref_bf16_bits_to_double(((const uint16_t*)base)[idx]);
    default: return ref_f16_bits_to_double(((const uint16_t*)base)[idx]);
  }
}

int ref_rope(const ref_rope_t* p, const void* x, const void* cos_t, const void* sin_t, double* y) {
  if (!p || !x || !cos_t || !sin_t || !y) return -1;
  if (p->batch < 1 || p->heads < 1 || p->seq < 1 || p->head_dim < 2 || (p->head_dim & 1)) return -1;
  if (p->dtype_x < REF_F32 || p->dtype_x > REF_F16 || p->dtype_table < REF_F32 || p->dtype_table > REF_F16)
    return -1;
  const int64_t D = p->head_dim, half = D / 2;
  for (int64_t b = 0; b < p->batch; ++b)
    for (int64_t h = 0; h < p->heads; ++h)
      for (int64_t s = 0; s < p->seq; ++s) {
        const int64_t xo = b * p->stride_b + h * p->stride_h + s * p->stride_s;
        const int64_t to = b * p->table_stride_b + s * D;
        double* out = y + ((b * p->heads + h) * p->seq + s) * D;
        for (int64_t i = 0; i < D; ++i) {
          const double xi = load_elem(x, p->dtype_x, xo + i);
          const double rot = i < half ? -load_elem(x, p->dtype_x, xo + i + half)
                                      : load_elem(x, p->dtype_x, xo + i - half);
          const double c = load_elem(cos_t, p->dtype_table, to + i);
          const double sn = load_elem(sin_t, p->dtype_table, to + i);
          out[i] = xi * c + rot * sn;
        }
      }
  return 0;
}
