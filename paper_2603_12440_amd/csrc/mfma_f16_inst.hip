// Instantiations of the matrix-core kernel for one operand type (a translation unit of its own,
// so that the operand types compile side by side).
#include "mfma_launch.hpp"

namespace mi355gemm {
#define X(BM, BN, BK, WM, WN, NS) MI355GEMM_MFMA_DEFINE(f16_t, f16_t, BM, BN, BK, WM, WN, NS)
MI355GEMM_MFMA_TILES(X)
#undef X
}  // namespace mi355gemm
