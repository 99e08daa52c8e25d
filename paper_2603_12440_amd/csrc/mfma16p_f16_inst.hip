// Instantiations of the 16x16x32 matrix-core kernel for one operand type, persistent workgroups
// (a translation unit of its own, so that the operand types compile side by side).
#include "mfma16_launch.hpp"

namespace mi355gemm {
#define X(BM, BN, WM, WN, G, P) MI355GEMM_MFMA16_DEFINE(f16_t, f16_t, BM, BN, WM, WN, G, P)
MI355GEMM_MFMA16P_TILES(X)
#undef X
}  // namespace mi355gemm
