"""CPU oracle for C = epilogue(A.B) and for the rotary positional embedding.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's CPU-baseline leg may import this
package.  It shares no code with the GPU library and does not import it.
"""
from .ref import (  # noqa: F401
    DTYPE_F32, DTYPE_BF16, DTYPE_F16, DTYPE_F8E4M3, ROW_MAJOR, COL_MAJOR,
    EPI_NONE, EPI_BIAS, EPI_BIAS_RELU, EPI_BIAS_GELU_ERF, EPI_BIAS_GELU_TANH,
    EPI_RELU, EPI_GELU_ERF, EPI_BIAS_SWISH_SCALE, EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
    EPI_SWISH_SCALE, EPI_SIGMOID_SCALE_RESIDUAL,
    Problem, build, ref_gemm, ref_gemm_points, ref_rope, activation, epilogue, sigmoid, num_threads,
    bf16_bits_to_double, f16_bits_to_double, f8e4m3_bits_to_double, f32_to_bf16_rne, f32_to_f16_rne,
)
