/*
 * Sanitizer run of the CPU oracle (test infrastructure): built by tests/test_oracle_sanitized.py
 * with -fsanitize=address,undefined and linked with oracle/ref_gemm.c and oracle/ref_rope.c.
 * Every buffer is allocated at exactly the size the oracle's addressing rules give, so that a
 * read or write one element too far, or any undefined arithmetic, aborts the run; the values
 * are small integers and are checked against plain 64-bit integer sums written out here.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/ref_gemm.h"
#include "../oracle/ref_rope.h"

static uint32_t rng_state = 12345u;
static int small_int(void) {                       /* -2 .. 2 */
  rng_state = rng_state * 1664525u + 1013904223u;
  return (int)((rng_state >> 16) % 5u) - 2;
}
static size_t esize(int dt) { return dt == REF_F32 ? 4 : (dt == REF_F8E4M3 ? 1 : 2); }
/* exact encodings of -2 .. 2 */
static void put(void* buf, size_t idx, int dt, int v) {
  static const uint16_t bf[5] = {0xC000, 0xBF80, 0x0000, 0x3F80, 0x4000};
  static const uint16_t hf[5] = {0xC000, 0xBC00, 0x0000, 0x3C00, 0x4000};
  static const uint8_t f8[5] = {0xC0, 0xB8, 0x00, 0x38, 0x40};
  if (dt == REF_F32) ((float*)buf)[idx] = (float)v;
  else if (dt == REF_BF16) ((uint16_t*)buf)[idx] = bf[v + 2];
  else if (dt == REF_F16) ((uint16_t*)buf)[idx] = hf[v + 2];
  else ((uint8_t*)buf)[idx] = f8[v + 2];
}

static int check_gemm(int64_t M, int64_t N, int64_t K, int la, int lb, int dt, int batch, int pad, int epi) {
  ref_problem_t p;
  memset(&p, 0, sizeof(p));
  p.M = M; p.N = N; p.K = K; p.layout_a = la; p.layout_b = lb; p.dtype_a = p.dtype_b = dt;
  p.epilogue = epi; p.batch = batch; p.scale = 1.0;
  const int64_t a_major = la == REF_ROW_MAJOR ? M : K, a_minor = la == REF_ROW_MAJOR ? K : M;
  const int64_t b_major = lb == REF_ROW_MAJOR ? K : N, b_minor = lb == REF_ROW_MAJOR ? N : K;
  p.lda = a_minor + pad; p.ldb = b_minor + pad;
  p.stride_a = a_major * p.lda + pad; p.stride_b = b_major * p.ldb + pad;
  const int has_bias = epi == REF_EPI_BIAS || epi == REF_EPI_BIAS_RELU;
  p.stride_bias = has_bias && batch > 1 ? N : 0;
  /* exact extents: the last batch ends with the last valid element */
  const size_t na = (size_t)((batch - 1) * p.stride_a + (a_major - 1) * p.lda + a_minor);
  const size_t nb = (size_t)((batch - 1) * p.stride_b + (b_major - 1) * p.ldb + b_minor);
  void* A = malloc(na * esize(dt));
  void* B = malloc(nb * esize(dt));
  float* bias = has_bias ? (float*)malloc(sizeof(float) * (size_t)(N + (batch - 1) * p.stride_bias)) : NULL;
  int* av = (int*)calloc((size_t)(batch * M * K), sizeof(int));
  int* bv = (int*)calloc((size_t)(batch * K * N), sizeof(int));
  memset(A, 0, na * esize(dt)); memset(B, 0, nb * esize(dt));
  for (int b = 0; b < batch; ++b)
    for (int64_t i = 0; i < M; ++i)
      for (int64_t k = 0; k < K; ++k) {
        const int v = small_int();
        av[(b * M + i) * K + k] = v;
        put(A, (size_t)(b * p.stride_a + (la == REF_ROW_MAJOR ? i * p.lda + k : k * p.lda + i)), dt, v);
      }
  for (int b = 0; b < batch; ++b)
    for (int64_t k = 0; k < K; ++k)
      for (int64_t j = 0; j < N; ++j) {
        const int v = small_int();
        bv[(b * K + k) * N + j] = v;
        put(B, (size_t)(b * p.stride_b + (lb == REF_ROW_MAJOR ? k * p.ldb + j : j * p.ldb + k)), dt, v);
      }
  if (bias) for (int64_t q = 0; q < N + (batch - 1) * p.stride_bias; ++q) bias[q] = (float)small_int();
  const size_t nout = (size_t)(batch * M * N);
  double* y = (double*)malloc(sizeof(double) * nout);
  double* t = (double*)malloc(sizeof(double) * nout);
  double* s = (double*)malloc(sizeof(double) * nout);
  int bad = ref_gemm(&p, A, B, bias, y, t, s) != 0;
  /* the same at every position through the points entry */
  int64_t* pb = (int64_t*)malloc(sizeof(int64_t) * nout);
  int64_t* pi = (int64_t*)malloc(sizeof(int64_t) * nout);
  int64_t* pj = (int64_t*)malloc(sizeof(int64_t) * nout);
  double* yp = (double*)malloc(sizeof(double) * nout);
  size_t q = 0;
  for (int b = 0; b < batch; ++b)
    for (int64_t i = 0; i < M; ++i)
      for (int64_t j = 0; j < N; ++j, ++q) { pb[q] = b; pi[q] = i; pj[q] = j; }
  bad |= ref_gemm_points(&p, A, B, bias, (int64_t)nout, pb, pi, pj, yp, NULL, NULL) != 0;
  q = 0;
  for (int b = 0; b < batch && !bad; ++b)
    for (int64_t i = 0; i < M; ++i)
      for (int64_t j = 0; j < N; ++j, ++q) {
        int64_t z = 0, sa = 0;
        for (int64_t k = 0; k < K; ++k) {
          const int64_t pr = (int64_t)av[(b * M + i) * K + k] * bv[(b * K + k) * N + j];
          z += pr; sa += pr < 0 ? -pr : pr;
        }
        double want = (double)z + (bias ? (double)bias[b * p.stride_bias + j] : 0.0);
        if (epi == REF_EPI_BIAS_RELU || epi == REF_EPI_RELU) want = want > 0 ? want : 0.0;
        if (y[q] != want || yp[q] != want || s[q] != (double)sa) bad = 1;
      }
  free(A); free(B); free(bias); free(av); free(bv); free(y); free(t); free(s); free(pb); free(pi); free(pj); free(yp);
  if (bad) fprintf(stderr, "gemm mismatch M=%lld N=%lld K=%lld la=%d lb=%d dt=%d batch=%d pad=%d epi=%d\n",
                   (long long)M, (long long)N, (long long)K, la, lb, dt, batch, pad, epi);
  return bad;
}

static int check_rope(int64_t batch, int64_t heads, int64_t seq, int64_t D, int per_batch_tables) {
  ref_rope_t p;
  memset(&p, 0, sizeof(p));
  p.batch = batch; p.heads = heads; p.seq = seq; p.head_dim = D; p.dtype_x = REF_F32; p.dtype_table = REF_F32;
  /* [batch, seq, heads, D] memory, exact extent */
  p.stride_h = D; p.stride_s = heads * D; p.stride_b = seq * heads * D;
  p.table_stride_b = per_batch_tables ? seq * D : 0;
  const size_t nx = (size_t)(batch * seq * heads * D);
  const size_t nt = (size_t)((per_batch_tables ? batch : 1) * seq * D);
  float* x = (float*)malloc(sizeof(float) * nx);
  float* c = (float*)malloc(sizeof(float) * nt);
  float* sn = (float*)malloc(sizeof(float) * nt);
  double* y = (double*)malloc(sizeof(double) * nx);
  for (size_t i = 0; i < nx; ++i) x[i] = (float)small_int();
  for (size_t i = 0; i < nt; ++i) { c[i] = (float)small_int(); sn[i] = (float)small_int(); }
  int bad = ref_rope(&p, x, c, sn, y) != 0;
  for (int64_t b = 0; b < batch && !bad; ++b)
    for (int64_t h = 0; h < heads; ++h)
      for (int64_t s = 0; s < seq; ++s)
        for (int64_t i = 0; i < D; ++i) {
          const float* xv = x + b * p.stride_b + h * p.stride_h + s * p.stride_s;
          const size_t ti = (size_t)((per_batch_tables ? b * seq * D : 0) + s * D + i);
          const double rot = i < D / 2 ? -(double)xv[i + D / 2] : (double)xv[i - D / 2];
          const double want = (double)xv[i] * c[ti] + rot * sn[ti];
          if (y[((b * heads + h) * seq + s) * D + i] != want) bad = 1;
        }
  free(x); free(c); free(sn); free(y);
  if (bad) fprintf(stderr, "rope mismatch b=%lld h=%lld s=%lld D=%lld\n", (long long)batch, (long long)heads, (long long)seq, (long long)D);
  return bad;
}

int main(void) {
  int bad = 0, cases = 0;
  const int dts[4] = {REF_F32, REF_BF16, REF_F16, REF_F8E4M3};
  const int epis[4] = {REF_EPI_NONE, REF_EPI_BIAS, REF_EPI_BIAS_RELU, REF_EPI_RELU};
  for (int la = 0; la < 2; ++la)
    for (int lb = 0; lb < 2; ++lb)
      for (int d = 0; d < 4; ++d)
        for (int pad = 0; pad < 2; ++pad) {
          bad |= check_gemm(5, 7, 9, la, lb, dts[d], 1, pad * 3, epis[(la + lb + d) & 3]); ++cases;
          bad |= check_gemm(1, 1, 1, la, lb, dts[d], 3, pad, epis[(d + pad) & 3]); ++cases;
          bad |= check_gemm(4, 3, 17, la, lb, dts[d], 2, pad * 2, epis[(la + d + 1) & 3]); ++cases;
        }
  /* the scalar helpers over their whole domain */
  double acc = 0.0;
  for (uint32_t b = 0; b < 65536; ++b) {
    const double v = ref_bf16_bits_to_double((uint16_t)b), h = ref_f16_bits_to_double((uint16_t)b);
    if (!isnan(v) && !isinf(v)) acc += v * 1e-300;
    if (!isnan(h) && !isinf(h)) acc += h * 1e-300;
  }
  for (uint32_t b = 0; b < 256; ++b) { const double v = ref_f8e4m3_bits_to_double((uint8_t)b); if (!isnan(v)) acc += v; }
  const float probes[8] = {0.0f, -0.0f, 1.0f, 3.3895314e38f, 1e-45f, 65504.0f, 65520.0f, -1e-8f};
  for (int i = 0; i < 8; ++i) { acc += ref_f32_to_bf16_rne(probes[i]); acc += ref_f32_to_f16_rne(probes[i]); }
  for (int e = 0; e <= REF_EPI_SIGMOID_SCALE_RESIDUAL; ++e)
    for (double t = -800.0; t <= 800.0; t += 37.5) acc += ref_epilogue(e, t, 1.5) * 1e-300;
  bad |= check_rope(2, 3, 4, 8, 0); ++cases;
  bad |= check_rope(1, 1, 1, 2, 1); ++cases;
  bad |= check_rope(2, 2, 3, 6, 1); ++cases;
  printf("sanitized oracle run: %d cases, %s (checksum %.3g)\n", cases, bad ? "MISMATCH" : "ok", acc);
  return bad;
}
