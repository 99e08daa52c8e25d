/*
 * Reference (oracle) dense matrix product with epilogue: see ref_gemm.h.
 *
 * TEST INFRASTRUCTURE ONLY; shares nothing with the GPU library.
 *
 * Written as the plain definition: one output element = one k-ascending fp64
 * dot product, followed by the epilogue in fp64.  No tiling, no blocking, no
 * reordering.  OpenMP only distributes independent output rows over cores.
 */
#include "ref_gemm.h"

#include <math.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- storage formats -> fp64 (all exact) -------------------------------- */

/* bf16 is the upper half of an IEEE binary32. */
double ref_bf16_bits_to_double(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double ref_f16_bits_to_double(uint16_t bits) {
  int sign = (bits >> 15) & 1;
  int e = (bits >> 10) & 0x1f;
  int f = bits & 0x3ff;
  double v;
  if (e == 0)
    v = ldexp((double)f, -24);                 /* zero and subnormals */
  else if (e == 31)
    v = f ? NAN : INFINITY;
  else
    v = ldexp(1.0 + (double)f / 1024.0, e - 15);
  return sign ? -v : v;
}

/* OCP 8-bit floating point E4M3: 1 sign bit, 4 exponent bits (bias 7), 3 significand bits.
 * No infinities; S.1111.111 is NaN; exponent field 15 otherwise encodes ordinary numbers
 * (largest: 1.75 * 2^8 = 448); exponent field 0 holds zero and the subnormals f/8 * 2^-6. */
double ref_f8e4m3_bits_to_double(uint8_t bits) {
  int sign = (bits >> 7) & 1;
  int e = (bits >> 3) & 0xf;
  int f = bits & 0x7;
  double v;
  if (e == 0)
    v = ldexp((double)f, -9);
  else if (e == 15 && f == 7)
    v = NAN;
  else
    v = ldexp(1.0 + (double)f / 8.0, e - 7);
  return sign ? -v : v;
}

/* fp32 -> bf16, round to nearest, ties to even, on the bit pattern. */
uint16_t ref_f32_to_bf16_rne(float x) {
  uint32_t u;
  memcpy(&u, &x, sizeof u);
  if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep it a quiet NaN */
    return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return (uint16_t)(u >> 16);
}

/* fp32 -> fp16, round to nearest, ties to even (default fenv rounding mode). */
uint16_t ref_f32_to_f16_rne(float x) {
  uint16_t sign = signbit(x) ? 0x8000u : 0;
  double a = fabs((double)x);
  if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* max + half ulp */
  if (a < ldexp(1.0, -14)) {                              /* subnormal range */
    uint16_t q = (uint16_t)nearbyint(ldexp(a, 24));
    return (uint16_t)(sign | q);                          /* q==1024 -> min normal */
  }
  int e2;
  (void)frexp(a, &e2);                                    /* a = m * 2^e2, m in [0.5,1) */
  int e = e2 - 1;
  int mant = (int)nearbyint((ldexp(a, -e) - 1.0) * 1024.0);
  if (mant == 1024) { mant = 0; e += 1; }
  if (e + 15 >= 31) return (uint16_t)(sign | 0x7c00u);
  return (uint16_t)(sign | ((e + 15) << 10) | mant);
}

static inline double load_elem(const void* base, int dtype, int64_t idx) {
  switch (dtype) {
    case REF_F32:  return (double)((const float*)base)[idx];
    case REF_BF16: return ref_bf16_bits_to_double(((const uint16_t*)base)[idx]);
    case REF_F8E4M3: return ref_f8e4m3_bits_to_double(((const uint8_t*)base)[idx]);
    default:       return ref_f16_bits_to_double(((const uint16_t*)base)[idx]);
  }
}

/* ---- epilogue ------------------------------------------------------------ */

static int epilogue_has_bias(int e) {
  return e == REF_EPI_BIAS || e == REF_EPI_BIAS_RELU ||
         e == REF_EPI_BIAS_GELU_ERF || e == REF_EPI_BIAS_GELU_TANH ||
         e == REF_EPI_BIAS_SWISH_SCALE || e == REF_EPI_BIAS_SIGMOID_SCALE_RESIDUAL;
}

/* act(t).  GELU (erf form) = t * Phi(t) = t/2 * (1 + erf(t/sqrt 2));
 * GELU (tanh form) = t/2 * (1 + tanh(sqrt(2/pi) * (t + 0.044715 t^3))). */
double ref_activation(int epilogue, double t) {
  switch (epilogue) {
    case REF_EPI_BIAS_RELU:
    case REF_EPI_RELU:
      return t > 0.0 ? t : 0.0;
    case REF_EPI_BIAS_GELU_ERF:
    case REF_EPI_GELU_ERF:
      return 0.5 * t * (1.0 + erf(t / sqrt(2.0)));
    case REF_EPI_BIAS_GELU_TANH: {
      const double pi = 3.14159265358979323846;
      double u = sqrt(2.0 / pi) * (t + 0.044715 * t * t * t);
      return 0.5 * t * (1.0 + tanh(u));
    }
    default:
      return t;
  }
}

/* sigma(t) = 1 / (1 + exp(-t)); written so that exp never sees a large positive argument. */
double ref_sigmoid(double t) {
  if (t >= 0.0) return 1.0 / (1.0 + exp(-t));
  const double e = exp(t);
  return e / (1.0 + e);
}

/* Every epilogue: the ones above, and the two with a scalar scale c. */
double ref_epilogue(int epilogue, double t, double scale) {
  switch (epilogue) {
    case REF_EPI_BIAS_SWISH_SCALE:
    case REF_EPI_SWISH_SCALE:
      return scale * (t * ref_sigmoid(t));
    case REF_EPI_BIAS_SIGMOID_SCALE_RESIDUAL:
    case REF_EPI_SIGMOID_SCALE_RESIDUAL:
      return scale * ref_sigmoid(t) + t;
    default:
      return ref_activation(epilogue, t);
  }
}

/* ---- one output element -------------------------------------------------- */

static int check_problem(const ref_problem_t* p, const void* A, const void* B,
                         const float* bias) {
  if (!p || !A || !B) return -1;
  if (p->M <= 0 || p->N <= 0 || p->K <= 0 || p->batch < 1) return -1;
  if (p->epilogue < REF_EPI_NONE || p->epilogue > REF_EPI_SIGMOID_SCALE_RESIDUAL) return -1;
  if (epilogue_has_bias(p->epilogue) != (bias != NULL)) return -1;
  if (p->lda < (p->layout_a == REF_ROW_MAJOR ? p->K : p->M)) return -1;
  if (p->ldb < (p->layout_b == REF_ROW_MAJOR ? p->N : p->K)) return -1;
  return 0;
}

static void one_element(const ref_problem_t* p, const void* A, const void* B,
                        const float* bias, int64_t b, int64_t i, int64_t j,
                        double* y, double* t, double* s) {
  /* strides of the k index and of the free index in each operand */
  const int64_t a_i = p->layout_a == REF_ROW_MAJOR ? p->lda : 1;
  const int64_t a_k = p->layout_a == REF_ROW_MAJOR ? 1 : p->lda;
  const int64_t b_k = p->layout_b == REF_ROW_MAJOR ? p->ldb : 1;
  const int64_t b_j = p->layout_b == REF_ROW_MAJOR ? 1 : p->ldb;
  const int64_t a0 = b * p->stride_a + i * a_i;
  const int64_t b0 = b * p->stride_b + j * b_j;
  double z = 0.0, sabs = 0.0;
  for (int64_t k = 0; k < p->K; ++k) {
    double prod = load_elem(A, p->dtype_a, a0 + k * a_k) *
                  load_elem(B, p->dtype_b, b0 + k * b_k);
    z += prod;
    sabs += fabs(prod);
  }
  double tt = z;
  if (bias) tt += (double)bias[b * p->stride_bias + j];
  if (y) *y = ref_epilogue(p->epilogue, tt, p->scale);
  if (t) *t = tt;
  if (s) *s = sabs;
}

int ref_gemm(const ref_problem_t* p, const void* A, const void* B,
             const float* bias, double* y, double* t, double* s) {
  if (check_problem(p, A, B, bias)) return -1;
  const int64_t rows = (int64_t)p->batch * p->M;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    const int64_t b = r / p->M, i = r % p->M;
    for (int64_t j = 0; j < p->N; ++j) {
      const int64_t o = r * p->N + j;
      one_element(p, A, B, bias, b, i, j, y ? y + o : NULL, t ? t + o : NULL,
                  s ? s + o : NULL);
    }
  }
  return 0;
}

int ref_gemm_points(const ref_problem_t* p, const void* A, const void* B,
                    const float* bias, int64_t npts, const int64_t* pb,
                    const int64_t* pi, const int64_t* pj,
                    double* y, double* t, double* s) {
  if (check_problem(p, A, B, bias)) return -1;
  if (npts < 0 || !pb || !pi || !pj) return -1;
  for (int64_t q = 0; q < npts; ++q)
    if (pb[q] < 0 || pb[q] >= p->batch || pi[q] < 0 || pi[q] >= p->M ||
        pj[q] < 0 || pj[q] >= p->N)
      return -1;
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < npts; ++q)
    one_element(p, A, B, bias, pb[q], pi[q], pj[q], y ? y + q : NULL,
                t ? t + q : NULL, s ? s + q : NULL);
  return 0;
}

int ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
