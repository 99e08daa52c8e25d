/*
 * Reference (oracle) dense matrix product with epilogue, on the CPU, in fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition that the GPU
 * library is checked against.  It shares no code with the GPU library and must
 * never be called from it.
 *
 * What it computes (textbook definition; the paper states no GEMM problem of
 * its own, it only lists matmul(+post-op) workloads, Sec. 4 / Tab. "operations"):
 *
 *   z[b,i,j] = sum_{k=0}^{K-1} a[b,i,k] * w[b,k,j]          (fp64, k ascending)
 *   s[b,i,j] = sum_k |a[b,i,k] * w[b,k,j]|                   (for error bounds)
 *   t[b,i,j] = z[b,i,j] + bias[b,j]        (if the epilogue has a bias)
 *   y[b,i,j] = act(t[b,i,j])               act in {id, relu, gelu_erf, gelu_tanh,
 *                                                  swish_scale, sigmoid_scale_residual}
 *
 * The last two are the post-ops of two of the paper's tasks: matmul followed by Swish and a
 * scaling, GEMM followed by sigmoid, scaling and a residual add (App. "Per-task results").  The paper gives
 * only the names; they are read here as the element-wise formulas the names spell out,
 * with sigma(t) = 1 / (1 + exp(-t)) and a scalar scale c:
 *   swish_scale(t)            = c * t * sigma(t)
 *   sigmoid_scale_residual(t) = c * sigma(t) + t     (the residual is the GEMM output itself)
 *
 * Every stored operand element (fp32, bf16, fp16 or 8-bit E4M3) is converted exactly to
 * fp64 first; products of two such values are exact in fp64.  Outputs stay in
 * fp64, never rounded to a storage type.
 *
 * Addressing: element (i,k) of A lives at A[b*stride_a + i*lda + k] when A is
 * row-major and at A[b*stride_a + k*lda + i] when column-major; the same rule
 * holds for B (K x N, ldb).  Outputs are packed row-major: y[(b*M + i)*N + j].
 */
#ifndef ORACLE_REF_GEMM_H
#define ORACLE_REF_GEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { REF_F32 = 0, REF_BF16 = 1, REF_F16 = 2, REF_F8E4M3 = 3 };   /* F8E4M3: OCP 8-bit float, operands only */
enum { REF_ROW_MAJOR = 0, REF_COL_MAJOR = 1 };
enum {
  REF_EPI_NONE = 0,
  REF_EPI_BIAS = 1,
  REF_EPI_BIAS_RELU = 2,
  REF_EPI_BIAS_GELU_ERF = 3,
  REF_EPI_BIAS_GELU_TANH = 4,
  REF_EPI_RELU = 5,
  REF_EPI_GELU_ERF = 6,
  REF_EPI_BIAS_SWISH_SCALE = 7,
  REF_EPI_BIAS_SIGMOID_SCALE_RESIDUAL = 8,
  REF_EPI_SWISH_SCALE = 9,
  REF_EPI_SIGMOID_SCALE_RESIDUAL = 10
};

typedef struct {
  int64_t M, N, K;
  int32_t layout_a, layout_b;      /* REF_ROW_MAJOR / REF_COL_MAJOR */
  int64_t lda, ldb;                /* leading dimensions in elements (never 0 here) */
  int32_t dtype_a, dtype_b;        /* REF_F32 / REF_BF16 / REF_F16 / REF_F8E4M3 */
  int32_t epilogue;                /* REF_EPI_* */
  int32_t batch;                   /* >= 1 */
  int64_t stride_a, stride_b;      /* elements between consecutive batches */
  int64_t stride_bias;             /* 0 = one bias shared by all batches */
  double scale;                    /* the scalar c of the *_SCALE epilogues; ignored by the others */
} ref_problem_t;

/* Full product.  y, t, s: each either NULL or room for batch*M*N doubles.
 * bias: fp32, length N (+ stride_bias per batch), NULL iff the epilogue has none.
 * Returns 0, or -1 on a bad argument. Uses OpenMP over output rows only. */
int ref_gemm(const ref_problem_t* p, const void* A, const void* B,
             const float* bias, double* y, double* t, double* s);

/* The same quantities at npts chosen output positions (pb[q], pi[q], pj[q]). */
int ref_gemm_points(const ref_problem_t* p, const void* A, const void* B,
                    const float* bias, int64_t npts, const int64_t* pb,
                    const int64_t* pi, const int64_t* pj,
                    double* y, double* t, double* s);

/* Scalar helpers (exposed so the tests can pin them one by one). */
double   ref_bf16_bits_to_double(uint16_t bits);
double   ref_f16_bits_to_double(uint16_t bits);
double   ref_f8e4m3_bits_to_double(uint8_t bits);
uint16_t ref_f32_to_bf16_rne(float x);   /* round to nearest, ties to even */
uint16_t ref_f32_to_f16_rne(float x);
double   ref_activation(int epilogue, double t);                 /* the epilogues without a scale */
double   ref_epilogue(int epilogue, double t, double scale);     /* every epilogue */
double   ref_sigmoid(double t);
int      ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
