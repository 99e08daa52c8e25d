"""MI355X-native GEMM with fused epilogue (and the rotary positional embedding): thin
Python binding of the C ABI in include/gemm.h and include/rope.h.  All arithmetic happens in the HIP kernels of libmi355gemm.so;
this package only marshals arguments."""
from .binding import (  # noqa: F401
    F32, BF16, F16, F8E4M3, ROW_MAJOR, COL_MAJOR,
    EPI_NONE, EPI_BIAS, EPI_BIAS_RELU, EPI_BIAS_GELU_ERF, EPI_BIAS_GELU_TANH,
    EPI_RELU, EPI_GELU_ERF, EPI_BIAS_SWISH_SCALE, EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
    EPI_SWISH_SCALE, EPI_SIGMOID_SCALE_RESIDUAL, EPILOGUES,
    GemmError, GemmDesc, Plan, RopeDesc, RopeTensor, rope_apply, probe_mfma_peak, probe_mfma16_peak, probe_read_peak,
    gemm_create, gemm_create_config, gemm_create_splitk, gemm_workspace_bytes, gemm_run,
    gemm_run_workspace, gemm_run_fixed_scratch, FIXED_SCRATCH_BYTES, gemm_tune, gemm_destroy, gemm_status_string,
    gemm_set_autotune, gemm_autotune_entries, gemm_autotune_clear,
    gemm_plan_info, gemm_config_count, gemm_config_name, config_names, library_path, load_library,
)
