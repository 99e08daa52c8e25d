"""ctypes front end of the C oracle (ref_gemm.c).  TEST INFRASTRUCTURE ONLY.

Operands are passed as flat numpy storage buffers: float32 for fp32, uint16 bit
patterns for bf16 / fp16, uint8 bit patterns for 8-bit E4M3.  Results come back as float64 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ref_gemm.c")
_SRC_ROPE = os.path.join(_HERE, "ref_rope.c")
_LIB = os.path.join(_HERE, "libref_gemm.so")

DTYPE_F32, DTYPE_BF16, DTYPE_F16, DTYPE_F8E4M3 = 0, 1, 2, 3
ROW_MAJOR, COL_MAJOR = 0, 1
(EPI_NONE, EPI_BIAS, EPI_BIAS_RELU, EPI_BIAS_GELU_ERF, EPI_BIAS_GELU_TANH,
 EPI_RELU, EPI_GELU_ERF, EPI_BIAS_SWISH_SCALE, EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
 EPI_SWISH_SCALE, EPI_SIGMOID_SCALE_RESIDUAL) = range(11)
_BIAS_EPILOGUES = (EPI_BIAS, EPI_BIAS_RELU, EPI_BIAS_GELU_ERF, EPI_BIAS_GELU_TANH,
                   EPI_BIAS_SWISH_SCALE, EPI_BIAS_SIGMOID_SCALE_RESIDUAL)


class _CProblem(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("layout_a", ctypes.c_int32), ("layout_b", ctypes.c_int32),
        ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64),
        ("dtype_a", ctypes.c_int32), ("dtype_b", ctypes.c_int32),
        ("epilogue", ctypes.c_int32), ("batch", ctypes.c_int32),
        ("stride_a", ctypes.c_int64), ("stride_b", ctypes.c_int64),
        ("stride_bias", ctypes.c_int64),
        ("scale", ctypes.c_double),
    ]


class _CRope(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int64), ("heads", ctypes.c_int64), ("seq", ctypes.c_int64),
        ("head_dim", ctypes.c_int64),
        ("dtype_x", ctypes.c_int32), ("dtype_table", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_s", ctypes.c_int64),
        ("table_stride_b", ctypes.c_int64),
    ]


@dataclass
class Problem:
    """One (batched) product.  Leading dimensions / strides of 0 mean packed."""
    M: int
    N: int
    K: int
    dtype_a: int = DTYPE_BF16
    dtype_b: int = DTYPE_BF16
    layout_a: int = ROW_MAJOR
    layout_b: int = COL_MAJOR
    lda: int = 0
    ldb: int = 0
    epilogue: int = EPI_NONE
    batch: int = 1
    stride_a: int = 0
    stride_b: int = 0
    stride_bias: int = 0
    scale: float = 1.0

    def resolved(self) -> "Problem":
        lda = self.lda or (self.K if self.layout_a == ROW_MAJOR else self.M)
        ldb = self.ldb or (self.N if self.layout_b == ROW_MAJOR else self.K)
        sa = self.stride_a or lda * (self.M if self.layout_a == ROW_MAJOR else self.K)
        sb = self.stride_b or ldb * (self.K if self.layout_b == ROW_MAJOR else self.N)
        return Problem(self.M, self.N, self.K, self.dtype_a, self.dtype_b,
                       self.layout_a, self.layout_b, lda, ldb, self.epilogue,
                       self.batch, sa, sb, self.stride_bias, self.scale)

    def _c(self) -> _CProblem:
        r = self.resolved()
        return _CProblem(r.M, r.N, r.K, r.layout_a, r.layout_b, r.lda, r.ldb,
                         r.dtype_a, r.dtype_b, r.epilogue, r.batch,
                         r.stride_a, r.stride_b, r.stride_bias, r.scale)


def build(force: bool = False) -> str:
    """Compile ref_gemm.c with gcc (plain -O2, OpenMP, no fast-math)."""
    deps = [_SRC, _SRC_ROPE, os.path.join(_HERE, "ref_gemm.h"), os.path.join(_HERE, "ref_rope.h")]
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < max(os.path.getmtime(d) for d in deps):
        cmd = ["gcc", "-std=c11", "-O2", "-fno-fast-math", "-ffp-contract=off",
               "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, _SRC_ROPE, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.ref_gemm.restype = ctypes.c_int
        lib.ref_gemm.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p,
                                 ctypes.c_void_p, ctypes.c_void_p, dp, dp, dp]
        lib.ref_gemm_points.restype = ctypes.c_int
        lib.ref_gemm_points.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ip, ip, ip, dp, dp, dp]
        lib.ref_bf16_bits_to_double.restype = ctypes.c_double
        lib.ref_bf16_bits_to_double.argtypes = [ctypes.c_uint16]
        lib.ref_f16_bits_to_double.restype = ctypes.c_double
        lib.ref_f16_bits_to_double.argtypes = [ctypes.c_uint16]
        lib.ref_f8e4m3_bits_to_double.restype = ctypes.c_double
        lib.ref_f8e4m3_bits_to_double.argtypes = [ctypes.c_uint8]
        lib.ref_f32_to_bf16_rne.restype = ctypes.c_uint16
        lib.ref_f32_to_bf16_rne.argtypes = [ctypes.c_float]
        lib.ref_f32_to_f16_rne.restype = ctypes.c_uint16
        lib.ref_f32_to_f16_rne.argtypes = [ctypes.c_float]
        lib.ref_activation.restype = ctypes.c_double
        lib.ref_activation.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.ref_epilogue.restype = ctypes.c_double
        lib.ref_epilogue.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_double]
        lib.ref_sigmoid.restype = ctypes.c_double
        lib.ref_sigmoid.argtypes = [ctypes.c_double]
        lib.ref_num_threads.restype = ctypes.c_int
        lib.ref_rope.restype = ctypes.c_int
        lib.ref_rope.argtypes = [ctypes.POINTER(_CRope), ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.c_void_p, dp]
        _lib = lib
    return _lib


def _np_dtype(code: int):
    return np.float32 if code == DTYPE_F32 else (np.uint8 if code == DTYPE_F8E4M3 else np.uint16)


def _operand(x, code: int, need: int, name: str) -> np.ndarray:
    x = np.ascontiguousarray(x).reshape(-1)
    if x.dtype != _np_dtype(code):
        raise TypeError(f"{name}: expected storage dtype {_np_dtype(code)}, got {x.dtype}")
    if x.size < need:
        raise ValueError(f"{name}: buffer of {x.size} elements, problem addresses {need}")
    return x


def _extent(rows_major: int, ld: int, inner: int, stride: int, batch: int) -> int:
    return (batch - 1) * stride + (rows_major - 1) * ld + inner


def _prepare(p: Problem, A, B, bias):
    r = p.resolved()
    a_major, a_inner = (r.M, r.K) if r.layout_a == ROW_MAJOR else (r.K, r.M)
    b_major, b_inner = (r.K, r.N) if r.layout_b == ROW_MAJOR else (r.N, r.K)
    A = _operand(A, r.dtype_a, _extent(a_major, r.lda, a_inner, r.stride_a, r.batch), "A")
    B = _operand(B, r.dtype_b, _extent(b_major, r.ldb, b_inner, r.stride_b, r.batch), "B")
    has_bias = r.epilogue in _BIAS_EPILOGUES
    if has_bias != (bias is not None):
        raise ValueError("bias must be given exactly when the epilogue has one")
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32).reshape(-1)
        if bias.size < (r.batch - 1) * r.stride_bias + r.N:
            raise ValueError("bias too short")
    return r, A, B, bias


def _ptr(x):
    return None if x is None else x.ctypes.data_as(ctypes.c_void_p)


def _dptr(x):
    return None if x is None else x.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def ref_gemm(p: Problem, A, B, bias=None, want=("y",)):
    """Full product; returns a dict with the requested ones of 'y', 't', 's',
    each a float64 array of shape (batch, M, N)."""
    lib = _load()
    r, A, B, bias = _prepare(p, A, B, bias)
    out = {k: np.empty((r.batch, r.M, r.N), dtype=np.float64) for k in want}
    cp = r._c()
    rc = lib.ref_gemm(ctypes.byref(cp), _ptr(A), _ptr(B), _ptr(bias),
                      _dptr(out.get("y")), _dptr(out.get("t")), _dptr(out.get("s")))
    if rc != 0:
        raise ValueError("ref_gemm rejected the problem")
    return out


def ref_gemm_points(p: Problem, A, B, bias, pb, pi, pj, want=("y",)):
    """The same quantities at chosen (batch, row, col) positions."""
    lib = _load()
    r, A, B, bias = _prepare(p, A, B, bias)
    pb = np.ascontiguousarray(pb, dtype=np.int64)
    pi = np.ascontiguousarray(pi, dtype=np.int64)
    pj = np.ascontiguousarray(pj, dtype=np.int64)
    n = pb.size
    if pi.size != n or pj.size != n:
        raise ValueError("index arrays differ in length")
    out = {k: np.empty(n, dtype=np.float64) for k in want}
    ip = ctypes.POINTER(ctypes.c_int64)
    cp = r._c()
    rc = lib.ref_gemm_points(ctypes.byref(cp), _ptr(A), _ptr(B), _ptr(bias), n,
                             pb.ctypes.data_as(ip), pi.ctypes.data_as(ip),
                             pj.ctypes.data_as(ip),
                             _dptr(out.get("y")), _dptr(out.get("t")), _dptr(out.get("s")))
    if rc != 0:
        raise ValueError("ref_gemm_points rejected the problem")
    return out


def ref_rope(batch, heads, seq, head_dim, x, cos, sin, dtype_x=DTYPE_BF16, dtype_table=DTYPE_F32,
             stride_b=0, stride_h=0, stride_s=0, table_stride_b=0):
    """Rotary embedding (rotate-half form) of x, logical shape [batch, heads, seq, head_dim]
    with element strides (0 = packed in that order); cos, sin: [seq, head_dim] or, with
    table_stride_b, [batch, seq, head_dim].  Returns float64 [batch, heads, seq, head_dim]."""
    lib = _load()
    ss = stride_s or head_dim
    sh = stride_h or seq * head_dim
    sb = stride_b or heads * seq * head_dim
    need = (batch - 1) * sb + (heads - 1) * sh + (seq - 1) * ss + head_dim
    x = _operand(x, dtype_x, need, "x")
    tneed = (batch - 1) * table_stride_b + seq * head_dim
    cos = _operand(cos, dtype_table, tneed, "cos")
    sin = _operand(sin, dtype_table, tneed, "sin")
    y = np.empty((batch, heads, seq, head_dim), dtype=np.float64)
    cp = _CRope(batch, heads, seq, head_dim, dtype_x, dtype_table, sb, sh, ss, table_stride_b)
    rc = lib.ref_rope(ctypes.byref(cp), _ptr(x), _ptr(cos), _ptr(sin), _dptr(y))
    if rc != 0:
        raise ValueError("ref_rope rejected the problem")
    return y


def activation(epilogue: int, t: float) -> float:
    return _load().ref_activation(epilogue, t)


def epilogue(code: int, t: float, scale: float) -> float:
    return _load().ref_epilogue(code, t, scale)


def sigmoid(t: float) -> float:
    return _load().ref_sigmoid(t)


def num_threads() -> int:
    return _load().ref_num_threads()


def f8e4m3_bits_to_double(bits: int) -> float:
    return _load().ref_f8e4m3_bits_to_double(bits)


def bf16_bits_to_double(bits: int) -> float:
    return _load().ref_bf16_bits_to_double(bits)


def f16_bits_to_double(bits: int) -> float:
    return _load().ref_f16_bits_to_double(bits)


def f32_to_bf16_rne(x: float) -> int:
    return _load().ref_f32_to_bf16_rne(x)


def f32_to_f16_rne(x: float) -> int:
    return _load().ref_f32_to_f16_rne(x)
