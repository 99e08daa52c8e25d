// Instantiations of the 16x16x32 matrix-core kernel for one operand type, one tile per workgroup
// (a translation unit of its own, so that the operand types compile side by side).
#include "mfma16_launch.hpp"

namespace mi355gemm {
#define X(BM, BN, WM, WN, G, P) MI355GEMM_MFMA16_DEFINE(bf16_t, bf16_t, BM, BN, WM, WN, G, P)
MI355GEMM_MFMA16_TILES(X)
#undef X
}  // namespace mi355gemm
