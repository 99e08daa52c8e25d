/*
 * mi355gemm - dense matrix product with a fused epilogue for AMD MI355X (gfx950).
 *
 *     C[b] = act( A[b] . B[b] + bias )        b = 0 .. batch-1
 *
 * A is M x K, B is K x N, C is M x N (logical shapes).  Products are
 * accumulated in fp32 whatever the storage type; the epilogue runs in fp32 on
 * the accumulators and the result is rounded once (to nearest even) to C's
 * storage type.  The operation is the matmul-with-post-op workload class of
 * the paper's evaluation (Sec. 4, Tab. "operations": the matmul row with a ReLU post-op;
 * App. "Per-task results": the matmul-with-activation tasks,
 * matrix-vector product, FFN-shaped layers).  The paper fixes no GEMM problem
 * statement; the definition above is the textbook one.
 *
 * Plain C ABI: no exceptions, no C++ or torch types cross this boundary.
 * All matrix pointers are DEVICE pointers; descriptors and plans live on the
 * HOST.  The library never allocates device memory and keeps no state between
 * calls besides the plans it hands out; only gemm_tune waits for the device.
 */
#ifndef MI355GEMM_GEMM_H
#define MI355GEMM_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gemm_plan gemm_plan_t;          /* opaque, owned by the library */

/* GEMM_F8E4M3: 8-bit floating point, OCP E4M3 (bias 7, no infinities, S.1111.111 = NaN, max 448);
 * operands only (the "reduced precision" direction of the paper's case study, Sec. 4): C is then
 * GEMM_BF16 or GEMM_F32.  Products of two such values are exact in fp32; accumulation is fp32. */
typedef enum { GEMM_F32 = 0, GEMM_BF16 = 1, GEMM_F16 = 2, GEMM_F8E4M3 = 3 } gemm_dtype_t;
typedef enum { GEMM_ROW_MAJOR = 0, GEMM_COL_MAJOR = 1 } gemm_layout_t;

/* Epilogues.  bias is a length-N fp32 vector added to every row (one value per
 * output column), before the activation.
 *   GELU_ERF (t) = t/2 * (1 + erf(t / sqrt 2))
 *   GELU_TANH(t) = t/2 * (1 + tanh(sqrt(2/pi) * (t + 0.044715 t^3)))
 * The last four are the post-ops of two of the paper's tasks, the matmul followed by Swish and a
 * scaling and the GEMM followed by sigmoid, scaling and a residual add (App. "Per-task results"), read as the
 * element-wise formulas their names spell out, with sigma(t) = 1 / (1 + exp(-t)) and
 * c = gemm_desc_t.scale:
 *   SWISH_SCALE(t)            = c * t * sigma(t)
 *   SIGMOID_SCALE_RESIDUAL(t) = c * sigma(t) + t     (the residual is the GEMM output itself) */
typedef enum {
  GEMM_EPI_NONE = 0,
  GEMM_EPI_BIAS = 1,
  GEMM_EPI_BIAS_RELU = 2,
  GEMM_EPI_BIAS_GELU_ERF = 3,
  GEMM_EPI_BIAS_GELU_TANH = 4,
  GEMM_EPI_RELU = 5,
  GEMM_EPI_GELU_ERF = 6,
  GEMM_EPI_BIAS_SWISH_SCALE = 7,
  GEMM_EPI_BIAS_SIGMOID_SCALE_RESIDUAL = 8,
  GEMM_EPI_SWISH_SCALE = 9,
  GEMM_EPI_SIGMOID_SCALE_RESIDUAL = 10
} gemm_epilogue_t;

/* Status codes: 0 is success, every failure is negative. */
enum {
  GEMM_OK = 0,
  GEMM_ERR_NULL = -1,         /* a required pointer is NULL (or bias given/absent against the epilogue) */
  GEMM_ERR_BAD_DIM = -2,      /* M, N or K <= 0, batch < 1, or sizes beyond the supported range */
  GEMM_ERR_BAD_LD = -3,       /* leading dimension below the extent, or batch stride overlapping */
  GEMM_ERR_UNSUPPORTED = -4,  /* no kernel for this dtype / layout / epilogue combination */
  GEMM_ERR_MISALIGNED = -5,   /* pointer not aligned to the element size */
  GEMM_ERR_NO_DEVICE = -6,    /* current device is not a gfx950 GPU */
  GEMM_ERR_LAUNCH = -7,       /* the HIP runtime refused the launch */
  GEMM_ERR_BAD_ENUM = -8,     /* an enum field holds a value outside its range */
  GEMM_ERR_BAD_CONFIG = -9,   /* tile configuration index unknown or not applicable */
  GEMM_ERR_BAD_SCALE = -10,   /* a *_SCALE epilogue with a scale that is not finite */
  GEMM_ERR_WORKSPACE = -11,   /* the plan needs a workspace (gemm_run_workspace), or the one given is too small / misaligned */
  GEMM_ERR_FIXED_SCRATCH = -12 /* gemm_run_fixed_scratch: the plan needs more than GEMM_FIXED_SCRATCH_BYTES of workspace */
};

/*
 * Problem descriptor (host memory, read only during gemm_create).
 *
 * Addressing, in elements of the operand's storage type:
 *   A(i,k) = A[b*stride_a + i*lda + k]   row-major,   A[b*stride_a + k*lda + i]   column-major
 *   B(k,j) = B[b*stride_b + k*ldb + j]   row-major,   B[b*stride_b + j*ldb + k]   column-major
 *   C(i,j) = C[b*stride_c + i*ldc + j]   row-major,   C[b*stride_c + j*ldc + i]   column-major
 *   bias(j) = bias[b*stride_bias + j]
 * A leading dimension of 0 means packed (the minor extent); a batch stride of 0
 * means packed for A, B and C (ld * major extent) and "shared by all batches"
 * for the bias.  Elements of the padding between rows are neither read into
 * results nor written.
 */
typedef struct {
  int64_t M, N, K;
  int32_t layout_a, layout_b, layout_c;          /* gemm_layout_t */
  int64_t lda, ldb, ldc;
  int32_t dtype_a, dtype_b, dtype_c, dtype_bias; /* gemm_dtype_t; dtype_a == dtype_b; dtype_c is dtype_a or F32
                                                    (BF16 or F32 for F8E4M3 operands); bias F32 */
  int32_t epilogue;                              /* gemm_epilogue_t */
  int32_t batch;                                 /* >= 1 */
  int64_t stride_a, stride_b, stride_c, stride_bias;
  float scale;                                   /* c of the *_SCALE epilogues (finite); ignored by the others */
} gemm_desc_t;

/*
 * Which kernel serves a problem.  The matrix-core and skinny kernels take 16-bit (or fp8)
 * operands with K contiguous in both (A row-major, B column-major: the weight matrix stored
 * N x K), row-major C, and move 16-byte pieces: K, lda, ldb and the batch strides of A and B
 * must be multiples of 16 bytes' worth of elements (8 for bf16 / fp16, 16 for fp8), and at
 * gemm_run A and B must be 16-byte aligned (GEMM_ERR_MISALIGNED otherwise).  M <= 16 goes to
 * the HBM-bound skinny kernels, everything else to the tiled MFMA kernel.  Every other
 * combination (fp32 operands, other layouts, odd leading dimensions) is served by the general
 * true-fp32 kernels (vector-ALU FMA for small problems, the fp32 matrix-core instruction
 * otherwise), which need element alignment only; fp8 operands have no such fallback
 * (GEMM_ERR_UNSUPPORTED).
 */

/*
 * gemm_create - validate a descriptor and choose kernel, tile shape and grid.
 * Runs entirely on the host and touches no device.  On success *out_plan
 * receives a new plan (release with gemm_destroy); on failure it is set to NULL
 * and nothing is allocated.  The kernel is picked from a fixed table of
 * compiled tile instantiations, in the manner of the paper's templated kernels
 * with a dispatch function (Sec. 3.4, App. "Templated kernel" listing).
 */
int gemm_create(const gemm_desc_t* desc, gemm_plan_t** out_plan);

/*
 * gemm_create_config - as gemm_create, but with tile configuration `config`
 * (0 .. gemm_config_count()-1) instead of the built-in choice; -1 = built-in
 * choice.  Returns GEMM_ERR_BAD_CONFIG if that instantiation cannot run this
 * problem.  This is the hook for parameter tuning (Sec. 3.4): time every
 * applicable configuration, keep the best.
 */
int gemm_create_config(const gemm_desc_t* desc, int config, gemm_plan_t** out_plan);
int gemm_config_count(void);
const char* gemm_config_name(int config);      /* NULL if out of range; static storage */

/*
 * gemm_run - enqueue one product on `hip_stream` (a hipStream_t cast to void*;
 * NULL = the default stream) of the current device and return without waiting.
 * A, B, C, bias: device pointers laid out as the plan's descriptor says, owned
 * by the caller; A, B and bias are only read, C is only written and must not
 * overlap A or B.  bias must be non-NULL exactly when the epilogue has a bias.
 * Every call recomputes everything; no result is cached between calls.  A plan
 * may be shared by threads and streams.  (In tuning mode, see gemm_set_autotune, the
 * first call for a problem also times the alternatives.)
 */
int gemm_run(const gemm_plan_t* plan, const void* A, const void* B, void* C,
             const void* bias, void* hip_stream);

/*
 * gemm_tune - parameter tuning over the compiled tile instantiations (the paper's templated
 * kernels, Sec. 3.4: every valid instantiation is evaluated, the best one wins, all results
 * are reported back).  Runs the problem `desc` on the caller's device buffers with every
 * configuration that can take it and times each one with the paper's protocol (App.
 * "Benchmarking kernel runtime"): a few initial trials size the loops, then a warm-up of at
 * least `min_seconds` and 10 launches, then a measurement of at least `min_seconds` and 10
 * launches made of inner loops of >= min(0.01 s, min_seconds) between two synchronisations.
 *   best_config   receives the index of the fastest configuration (pass it to gemm_create_config);
 *   us_per_config NULL, or room for gemm_config_count() floats: mean microseconds per launch,
 *                 negative for configurations that cannot run this problem.
 * C is overwritten (with correct results).  Blocks until done: it synchronises `hip_stream`.
 * Creates HIP events and nothing else; no device memory is allocated.
 */
int gemm_tune(const gemm_desc_t* desc, const void* A, const void* B, void* C, const void* bias,
              void* hip_stream, double min_seconds, int* best_config, float* us_per_config);

/*
 * Tuning mode - the paper's parameter optimisation over templated kernels (Sec. 3.4) as a
 * switch.  Off by default; on when the environment variable GEMM_TUNE is set to anything but
 * "" or "0" at the library's first use, or after gemm_set_autotune(1).  While it is on, the
 * first gemm_run of a plan from gemm_create (or gemm_create_config(-1)) times every
 * applicable instantiation (as gemm_tune does, 0.02 s each) and the plan as built on the
 * caller's own buffers, keeps the fastest for that plan, and remembers it per problem (sizes,
 * layouts, dtypes, epilogue, leading dimensions, batch strides) for the rest of the process:
 * later plans of the same problem skip the timing.  That first call blocks (it synchronises
 * the stream, so it must not be made under stream capture), overwrites C several times with
 * the correct result, and needs A, B and C 16-byte aligned (otherwise the plan runs untuned).
 * Plans of gemm_create_config(config >= 0) and gemm_create_splitk are never re-planned.  The
 * table lives in host memory; no device memory is allocated.  Thread-safe.
 *   gemm_set_autotune      switch the mode (non-zero = on); returns the previous setting (0 / 1)
 *   gemm_autotune_entries  number of problems remembered
 *   gemm_autotune_clear    forget them (plans already timed keep their choice)
 */
int gemm_set_autotune(int enabled);
int gemm_autotune_entries(void);
int gemm_autotune_clear(void);

/*
 * Split-K: for products with few output tiles and a long K (too few tiles to occupy the 256
 * CUs), K is cut into `splits` equal slices that are multiplied side by side into fp32
 * partial results in a caller-provided workspace, and a second kernel adds the slices (in
 * a fixed order), applies the epilogue and writes C.  This is the highest synchronisation level of the paper's taxonomy (Sec. 3.2, d_sync = 3:
 * several passes with a device-wide synchronisation between them).
 *
 * gemm_create_splitk - as gemm_create, for batch == 1 problems the matrix-core kernels can
 *   take (16-bit or fp8 operands, K-contiguous A and B, every slice a whole number of 16-byte pieces).  splits >= 1, or
 *   0 for a built-in choice (which may be 1).  GEMM_ERR_UNSUPPORTED if the problem or the
 *   split cannot be served.
 * gemm_workspace_bytes - bytes of device memory the plan needs as workspace (0 for plans of
 *   gemm_create / gemm_create_config): splits * M * N * 4.
 * gemm_run_workspace - as gemm_run; `workspace` is a DEVICE pointer, 16-byte aligned, of at
 *   least gemm_workspace_bytes(plan) bytes, owned by the caller, overwritten by the call and
 *   free to re-use once the work enqueued here has finished.  Two launches on `hip_stream`.
 *   Also runs plans that need no workspace (workspace may then be NULL).
 * gemm_run on a split-K plan returns GEMM_ERR_WORKSPACE.
 */
int gemm_create_splitk(const gemm_desc_t* desc, int splits, gemm_plan_t** out_plan);
size_t gemm_workspace_bytes(const gemm_plan_t* plan);
int gemm_run_workspace(const gemm_plan_t* plan, const void* A, const void* B, void* C,
                       const void* bias, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * gemm_run_fixed_scratch - gemm_run_workspace for callers that cannot allocate device memory
 * or pass a workspace along: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The split-K partial results go to a fixed buffer of
 * GEMM_FIXED_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs
 * on holds its own copy until the process ends); nothing is allocated or freed, here or in any
 * call it makes.  A, B, C, bias and hip_stream as for gemm_run.
 *   - A plan whose gemm_workspace_bytes exceeds GEMM_FIXED_SCRATCH_BYTES is refused with
 *     GEMM_ERR_FIXED_SCRATCH and nothing is enqueued (use gemm_run_workspace).  Plans that need
 *     no workspace run as with gemm_run.
 *   - All calls on one GPU share that GPU's buffer, on every stream and for every plan: calls
 *     whose work overlaps in time on one GPU race on it (the results of both are undefined).
 *     Calls on one stream, or otherwise ordered, are safe: every partial result is written
 *     before it is read, nothing carries over from one call to the next, nothing needs
 *     clearing.
 *   - The first call on a device looks up that device's copy of the buffer (no allocation);
 *     GEMM_ERR_LAUNCH if the runtime cannot provide it.
 */
#define GEMM_FIXED_SCRATCH_BYTES ((size_t)32 << 20)
int gemm_run_fixed_scratch(const gemm_plan_t* plan, const void* A, const void* B, void* C,
                           const void* bias, void* hip_stream);

/* gemm_destroy - release a plan.  NULL is a no-op that returns GEMM_OK. */
int gemm_destroy(gemm_plan_t* plan);

/*
 * Logging (the paper's profiler feedback reports which kernel variant ran, App. "Profiler
 * Feedback"): with GEMM_LOG=1 in the environment every gemm_create* writes one line to stderr
 * with the problem and the text gemm_plan_info gives for the plan it made.
 */

/* Static, human-readable text for a status code (never NULL). */
const char* gemm_status_string(int status);

/* Writes "kernel=<name> tile=<BM>x<BN>x<BK> grid=<x>,<y>,<z> block=<t> lds=<bytes>"
 * (NUL-terminated, truncated to n bytes) into buf; returns the untruncated length
 * or a negative status. */
int gemm_plan_info(const gemm_plan_t* plan, char* buf, size_t n);

#ifdef __cplusplus
}
#endif
#endif /* MI355GEMM_GEMM_H */
