// Internal to the library: the plan object behind gemm_plan_t, the table entry type of the
// compiled kernel instantiations, and the signature every launcher has.  Shared by the
// translation units the kernel instantiations are spread over (one per operand type of the
// matrix-core kernel, so that they compile side by side).
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/gemm.h"
#include "common.hpp"

namespace mi355gemm {

enum Kind { KIND_SIMT = 0, KIND_MFMA = 1, KIND_SKINNY = 2, KIND_SKINNY_PANEL = 3, KIND_F32_VEC = 4 };
// (KIND_F32_VEC: the general kernels' grid, fp32 operands in 16-byte pieces; KIND_SKINNY: vector ALUs, a wave per row of W; KIND_SKINNY_PANEL: matrix cores, a workgroup per
// 32-row panel of W)

struct Config;

}  // namespace mi355gemm

struct gemm_plan {
  gemm_desc_t d;          // fully resolved (no zero ld / stride left)
  const mi355gemm::Config* cfg;
  int cfg_index;
  dim3 grid, block;
  int group_m, xcd_remap; // MFMA scheduling
  // Optional second launch for the columns past d.N (a different tile shape for the part of
  // the problem that does not fill whole rounds of the CUs): its own plan, and the element
  // offsets of its B, C and bias.
  gemm_plan* tail;
  int64_t tail_off_b, tail_off_c, tail_off_bias;
  // Split-K: `d` is the caller's problem, `inner` the batched product of the K slices into
  // the fp32 workspace (cfg, grid, ... above are then those of the inner plan, for reporting).
  int splits;
  gemm_plan* inner;
  // Tuning mode (gemm_set_autotune / GEMM_TUNE=1): `d_user` is the caller's resolved problem
  // (d may have been narrowed to the first launch's columns), `built_in` says the kernel was
  // the library's choice, and once the problem has been timed `tune_state` is 1 (this plan
  // is the fastest) or 2 (`tuned`, a plan of the fastest configuration, runs instead).
  // Both are set once, with atomic operations; a plan stays shareable between threads.
  gemm_desc_t d_user;
  int c_cached;           // fp32 C of this plan is re-read right away (the inner plan of a split-K plan)
  int built_in;
  int tune_state;
  gemm_plan* tuned;
};

namespace mi355gemm {

typedef hipError_t (*launch_fn)(const gemm_plan&, const void*, const void*, void*, const void*,
                                hipStream_t);

struct Config {
  const char* name;
  Kind kind;
  int bm, bn, bk;         // tile (skinny: bm = padded M, bn = workgroups per CU, bk = K per pass)
  int threads;
  int lds_bytes;
  launch_fn launch[4];    // per operand dtype (GEMM_F32 / BF16 / F16 / F8E4M3); NULL = not compiled
  int persist;            // 1: workgroups walk over several tiles (grid = workgroups resident at once)
};

inline int esize(int dt) { return dt == GEMM_F32 ? 4 : (dt == GEMM_F8E4M3 ? 1 : 2); }

}  // namespace mi355gemm
