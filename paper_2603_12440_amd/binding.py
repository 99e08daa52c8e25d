"""ctypes binding of include/gemm.h: same names, argument marshalling only.

There is no fallback: if libmi355gemm.so is missing or does not load, every
entry point raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libmi355gemm.so")

F32, BF16, F16, F8E4M3 = 0, 1, 2, 3
ROW_MAJOR, COL_MAJOR = 0, 1
(EPI_NONE, EPI_BIAS, EPI_BIAS_RELU, EPI_BIAS_GELU_ERF, EPI_BIAS_GELU_TANH,
 EPI_RELU, EPI_GELU_ERF, EPI_BIAS_SWISH_SCALE, EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
 EPI_SWISH_SCALE, EPI_SIGMOID_SCALE_RESIDUAL) = range(11)
EPILOGUES = {"none": EPI_NONE, "bias": EPI_BIAS, "bias_relu": EPI_BIAS_RELU,
             "bias_gelu_erf": EPI_BIAS_GELU_ERF, "bias_gelu_tanh": EPI_BIAS_GELU_TANH,
             "relu": EPI_RELU, "gelu_erf": EPI_GELU_ERF,
             "bias_swish_scale": EPI_BIAS_SWISH_SCALE,
             "bias_sigmoid_scale_residual": EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
             "swish_scale": EPI_SWISH_SCALE,
             "sigmoid_scale_residual": EPI_SIGMOID_SCALE_RESIDUAL}

GEMM_OK = 0


class GemmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"gemm status {status}: {text}")
        self.status = status


class GemmDesc(ctypes.Structure):
    """Mirror of gemm_desc_t."""
    _fields_ = [
        ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("layout_a", ctypes.c_int32), ("layout_b", ctypes.c_int32), ("layout_c", ctypes.c_int32),
        ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("ldc", ctypes.c_int64),
        ("dtype_a", ctypes.c_int32), ("dtype_b", ctypes.c_int32), ("dtype_c", ctypes.c_int32),
        ("dtype_bias", ctypes.c_int32),
        ("epilogue", ctypes.c_int32), ("batch", ctypes.c_int32),
        ("stride_a", ctypes.c_int64), ("stride_b", ctypes.c_int64), ("stride_c", ctypes.c_int64),
        ("stride_bias", ctypes.c_int64),
        ("scale", ctypes.c_float),
    ]

    def __init__(self, M=0, N=0, K=0, dtype=BF16, layout_a=ROW_MAJOR, layout_b=COL_MAJOR,
                 layout_c=ROW_MAJOR, lda=0, ldb=0, ldc=0, dtype_c=None, epilogue=EPI_NONE,
                 batch=1, stride_a=0, stride_b=0, stride_c=0, stride_bias=0,
                 dtype_b=None, dtype_bias=F32, scale=1.0):
        super().__init__(M, N, K, layout_a, layout_b, layout_c, lda, ldb, ldc,
                         dtype, dtype if dtype_b is None else dtype_b,
                         (BF16 if dtype == F8E4M3 else dtype) if dtype_c is None else dtype_c, dtype_bias,
                         epilogue, batch, stride_a, stride_b, stride_c, stride_bias, scale)


class RopeDesc(ctypes.Structure):
    """Mirror of rope_desc_t."""
    _fields_ = [
        ("batch", ctypes.c_int64), ("seq", ctypes.c_int64), ("head_dim", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("table_dtype", ctypes.c_int32),
        ("table_stride_b", ctypes.c_int64),
    ]

    def __init__(self, batch=0, seq=0, head_dim=0, dtype=BF16, table_dtype=F32, table_stride_b=0):
        super().__init__(batch, seq, head_dim, dtype, table_dtype, table_stride_b)


class RopeTensor(ctypes.Structure):
    """Mirror of rope_tensor_t; x and y are torch device tensors or raw addresses."""
    _fields_ = [
        ("x", ctypes.c_void_p), ("y", ctypes.c_void_p), ("heads", ctypes.c_int64),
        ("x_stride_b", ctypes.c_int64), ("x_stride_h", ctypes.c_int64), ("x_stride_s", ctypes.c_int64),
        ("y_stride_b", ctypes.c_int64), ("y_stride_h", ctypes.c_int64), ("y_stride_s", ctypes.c_int64),
    ]

    def __init__(self, x=None, y=None, heads=0, x_strides=(0, 0, 0), y_strides=(0, 0, 0)):
        super().__init__(_dev_ptr(x), _dev_ptr(y), heads, *x_strides, *y_strides)


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libmi355gemm.so (built by paper_2603_12440_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it first "
                           "(python -m paper_2603_12440_amd.build); there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    pp = ctypes.POINTER(ctypes.c_void_p)
    lib.gemm_create.restype = ctypes.c_int
    lib.gemm_create.argtypes = [ctypes.POINTER(GemmDesc), pp]
    lib.gemm_create_config.restype = ctypes.c_int
    lib.gemm_create_config.argtypes = [ctypes.POINTER(GemmDesc), ctypes.c_int, pp]
    lib.gemm_config_count.restype = ctypes.c_int
    lib.gemm_config_name.restype = ctypes.c_char_p
    lib.gemm_config_name.argtypes = [ctypes.c_int]
    lib.gemm_run.restype = ctypes.c_int
    lib.gemm_run.argtypes = [ctypes.c_void_p] * 6
    lib.gemm_tune.restype = ctypes.c_int
    lib.gemm_tune.argtypes = [ctypes.POINTER(GemmDesc), ctypes.c_void_p, ctypes.c_void_p,
                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double,
                              ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)]
    lib.gemm_destroy.restype = ctypes.c_int
    lib.gemm_destroy.argtypes = [ctypes.c_void_p]
    lib.gemm_set_autotune.restype = ctypes.c_int
    lib.gemm_set_autotune.argtypes = [ctypes.c_int]
    lib.gemm_autotune_entries.restype = ctypes.c_int
    lib.gemm_autotune_entries.argtypes = []
    lib.gemm_autotune_clear.restype = ctypes.c_int
    lib.gemm_autotune_clear.argtypes = []
    lib.gemm_status_string.restype = ctypes.c_char_p
    lib.gemm_status_string.argtypes = [ctypes.c_int]
    lib.gemm_plan_info.restype = ctypes.c_int
    lib.gemm_plan_info.argtypes = [ctypes.c_void_p, ctypes.c_char_p, ctypes.c_size_t]
    lib.gemm_create_splitk.restype = ctypes.c_int
    lib.gemm_create_splitk.argtypes = [ctypes.POINTER(GemmDesc), ctypes.c_int, pp]
    lib.gemm_workspace_bytes.restype = ctypes.c_size_t
    lib.gemm_workspace_bytes.argtypes = [ctypes.c_void_p]
    lib.gemm_run_workspace.restype = ctypes.c_int
    lib.gemm_run_workspace.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_size_t, ctypes.c_void_p]
    lib.gemm_run_fixed_scratch.restype = ctypes.c_int
    lib.gemm_run_fixed_scratch.argtypes = [ctypes.c_void_p] * 6
    lib.probe_mfma_peak.restype = ctypes.c_int
    lib.probe_mfma_peak.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double,
                                    ctypes.POINTER(ctypes.c_double)]
    lib.probe_mfma16_peak.restype = ctypes.c_int
    lib.probe_mfma16_peak.argtypes = lib.probe_mfma_peak.argtypes
    lib.probe_read_peak.restype = ctypes.c_int
    lib.probe_read_peak.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
    lib.rope_apply.restype = ctypes.c_int
    lib.rope_apply.argtypes = [ctypes.POINTER(RopeDesc), ctypes.POINTER(RopeTensor), ctypes.c_int,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    _lib = lib
    return lib


def gemm_status_string(status: int) -> str:
    return load_library().gemm_status_string(status).decode()


def _check(status: int):
    if status != GEMM_OK:
        raise GemmError(status, gemm_status_string(status))


class Plan:
    """Owns one gemm_plan_t*; destroyed with the object (or by gemm_destroy)."""

    def __init__(self, handle: int, desc: GemmDesc):
        self.handle = handle
        self.desc = desc

    def info(self) -> str:
        return gemm_plan_info(self)

    def close(self):
        if self.handle:
            load_library().gemm_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gemm_create_config(desc: GemmDesc, config: int = -1) -> Plan:
    lib = load_library()
    out = ctypes.c_void_p()
    _check(lib.gemm_create_config(ctypes.byref(desc), config, ctypes.byref(out)))
    return Plan(out.value, desc)


def gemm_create(desc: GemmDesc) -> Plan:
    lib = load_library()
    out = ctypes.c_void_p()
    _check(lib.gemm_create(ctypes.byref(desc), ctypes.byref(out)))
    return Plan(out.value, desc)


def gemm_create_splitk(desc: GemmDesc, splits: int = 0) -> Plan:
    """A split-K plan (splits = 0: built-in choice); run it with gemm_run_workspace."""
    lib = load_library()
    out = ctypes.c_void_p()
    _check(lib.gemm_create_splitk(ctypes.byref(desc), splits, ctypes.byref(out)))
    return Plan(out.value, desc)


def gemm_workspace_bytes(plan: Plan) -> int:
    return int(load_library().gemm_workspace_bytes(plan.handle))


def _dev_ptr(x) -> Optional[int]:
    """Device address of a torch tensor (or a raw integer address, or None)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def gemm_run(plan: Plan, A, B, C, bias=None, stream: Optional[int] = None) -> None:
    """Enqueue C = epilogue(A.B) on `stream` (a raw hipStream_t value; default:
    torch's current stream).  A, B, C, bias: torch device tensors or raw addresses."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(load_library().gemm_run(plan.handle, _dev_ptr(A), _dev_ptr(B), _dev_ptr(C),
                                   _dev_ptr(bias), stream or None))


def gemm_run_workspace(plan: Plan, A, B, C, bias=None, workspace=None, workspace_bytes: Optional[int] = None,
                       stream: Optional[int] = None) -> None:
    """As gemm_run, with a caller-provided device workspace (a torch tensor or a raw address
    plus workspace_bytes) for plans that need one."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().gemm_run_workspace(plan.handle, _dev_ptr(A), _dev_ptr(B), _dev_ptr(C), _dev_ptr(bias),
                                             _dev_ptr(workspace), workspace_bytes, stream or None))


FIXED_SCRATCH_BYTES = 32 << 20


def gemm_run_fixed_scratch(plan: Plan, A, B, C, bias=None, stream: Optional[int] = None) -> None:
    """As gemm_run_workspace, with the library's own fixed scratch buffer (no allocation anywhere;
    plans that need more than FIXED_SCRATCH_BYTES are refused)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(load_library().gemm_run_fixed_scratch(plan.handle, _dev_ptr(A), _dev_ptr(B), _dev_ptr(C),
                                                 _dev_ptr(bias), stream or None))


def gemm_tune(desc: GemmDesc, A, B, C, bias=None, stream: Optional[int] = None,
              min_seconds: float = 1.0):
    """Time every applicable tile configuration on the given device buffers; returns
    (best_config_index, {config_name: microseconds per launch})."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    lib = load_library()
    n = lib.gemm_config_count()
    best = ctypes.c_int(-1)
    us = (ctypes.c_float * n)()
    _check(lib.gemm_tune(ctypes.byref(desc), _dev_ptr(A), _dev_ptr(B), _dev_ptr(C), _dev_ptr(bias),
                         stream or None, float(min_seconds), ctypes.byref(best), us))
    return best.value, {gemm_config_name(i): float(us[i]) for i in range(n) if us[i] >= 0}


def gemm_set_autotune(enabled: bool) -> bool:
    """Switches tuning mode (include/gemm.h); returns the previous setting."""
    return bool(load_library().gemm_set_autotune(1 if enabled else 0))


def gemm_autotune_entries() -> int:
    return int(load_library().gemm_autotune_entries())


def gemm_autotune_clear() -> None:
    _check(load_library().gemm_autotune_clear())


def gemm_destroy(plan: Optional[Plan]) -> None:
    if plan is not None:
        plan.close()


def gemm_plan_info(plan: Plan) -> str:
    buf = ctypes.create_string_buffer(256)
    n = load_library().gemm_plan_info(plan.handle, buf, len(buf))
    if n < 0:
        _check(n)
    return buf.value.decode()


def gemm_config_count() -> int:
    return load_library().gemm_config_count()


def gemm_config_name(config: int) -> Optional[str]:
    s = load_library().gemm_config_name(config)
    return s.decode() if s is not None else None


def config_names() -> List[str]:
    return [gemm_config_name(i) for i in range(gemm_config_count())]


def rope_apply(desc: RopeDesc, tensors, cos, sin, stream: Optional[int] = None) -> None:
    """Enqueue the rotary embedding of one or two tensors (a list of RopeTensor) that share
    positions and tables, in one launch.  cos, sin: torch device tensors or raw addresses."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    arr = (RopeTensor * len(tensors))(*tensors)
    _check(load_library().rope_apply(ctypes.byref(desc), arr, len(tensors), _dev_ptr(cos), _dev_ptr(sin),
                                     stream or None))


def probe_mfma_peak(dtype: int, sink, stream: Optional[int] = None, min_seconds: float = 0.3,
                    refresh_operands: bool = False) -> float:
    """TFLOP/s of an MFMA-only register loop on the current device (blocks until done)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    out = ctypes.c_double(0.0)
    _check(load_library().probe_mfma_peak(dtype, int(refresh_operands), _dev_ptr(sink), stream or None,
                                          min_seconds, ctypes.byref(out)))
    return out.value


def probe_mfma16_peak(dtype: int, sink, stream: Optional[int] = None, min_seconds: float = 0.3,
                    refresh_operands: bool = False) -> float:
    """TFLOP/s of an MFMA-only register loop on the 16x16x32 shape on the current device (blocks until done)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    out = ctypes.c_double(0.0)
    _check(load_library().probe_mfma16_peak(dtype, int(refresh_operands), _dev_ptr(sink), stream or None,
                                          min_seconds, ctypes.byref(out)))
    return out.value


def probe_read_peak(src, nbytes: int, sink, stream: Optional[int] = None, min_seconds: float = 0.3) -> float:
    """GB/s of a streaming read of `nbytes` (>= 1 GiB) of the device buffer `src` (blocks until done)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    out = ctypes.c_double(0.0)
    _check(load_library().probe_read_peak(_dev_ptr(src), nbytes, _dev_ptr(sink), stream or None, min_seconds,
                                          ctypes.byref(out)))
    return out.value
