"""Shared plumbing for the parity tests: run one problem through the GPU
library (C ABI via the Python binding) and through the CPU oracle, and compare.

Error measures:
  E1  max|C - y| / (K max|A| max|B| [+ max|bias|])     the stated tolerance
  E2  per-element a-priori bound: any-order fp32 accumulation of exact products
      (K u32 S), fp32 epilogue slack, one rounding to the output type
  E3  the paper's criterion (Sec. 4, "Metrics"): nu = |y - c| / (|y| + eps) < 0.01
      on >= 99 % of the outputs, and cosine similarity of the flattened outputs
"""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl

U32 = 2.0 ** -24
OUT_ROUNDOFF = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24}
E1_TOL = {"bf16": 2e-3, "f16": 2e-3, "f32": 1e-6, "f8": 2e-3}


def oracle_codes(o):
    return ({"f32": o.DTYPE_F32, "bf16": o.DTYPE_BF16, "f16": o.DTYPE_F16, "f8": o.DTYPE_F8E4M3},
            {"row": o.ROW_MAJOR, "col": o.COL_MAJOR},
            {"none": o.EPI_NONE, "bias": o.EPI_BIAS, "bias_relu": o.EPI_BIAS_RELU,
             "bias_gelu_erf": o.EPI_BIAS_GELU_ERF, "bias_gelu_tanh": o.EPI_BIAS_GELU_TANH,
             "relu": o.EPI_RELU, "gelu_erf": o.EPI_GELU_ERF,
             "bias_swish_scale": o.EPI_BIAS_SWISH_SCALE,
             "bias_sigmoid_scale_residual": o.EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
             "swish_scale": o.EPI_SWISH_SCALE,
             "sigmoid_scale_residual": o.EPI_SIGMOID_SCALE_RESIDUAL})


def oracle_problem(o, w: wl.Workload, lda=0, ldb=0, stride_a=0, stride_b=0, stride_bias=0):
    dt, lay, epi = oracle_codes(o)
    return o.Problem(w.M, w.N, w.K, dt[w.dtype], dt[w.dtype], lay[w.layout_a], lay[w.layout_b],
                     lda, ldb, epi[w.epilogue], w.batch, stride_a, stride_b, stride_bias, w.scale)


def gpu_desc(g, w: wl.Workload, out_dtype=None, layout_c="row", lda=0, ldb=0, ldc=0,
             stride_a=0, stride_b=0, stride_c=0, stride_bias=0):
    dt = {"f32": g.F32, "bf16": g.BF16, "f16": g.F16, "f8": g.F8E4M3}
    lay = {"row": g.ROW_MAJOR, "col": g.COL_MAJOR}
    return g.GemmDesc(w.M, w.N, w.K, dtype=dt[w.dtype], layout_a=lay[w.layout_a],
                      layout_b=lay[w.layout_b], layout_c=lay[layout_c], lda=lda, ldb=ldb, ldc=ldc,
                      dtype_c=dt[out_dtype or w.out_dtype or w.dtype], epilogue=g.EPILOGUES[w.epilogue],
                      batch=w.batch, stride_a=stride_a, stride_b=stride_b, stride_c=stride_c,
                      stride_bias=stride_bias, scale=w.scale)


def pad_minor(t: torch.Tensor, pad: int, fill=float("nan")) -> torch.Tensor:
    """(batch, major, minor) -> (batch, major, minor + pad) with `fill` in the padding."""
    if pad == 0:
        return t
    b, major, minor = t.shape
    if t.dtype == torch.float8_e4m3fn:          # no fill / slice assignment for 8-bit floats: go through fp32
        out = torch.full((b, major, minor + pad), fill, dtype=torch.float32)
        out[:, :, :minor] = t.float()
        return out.to(t.dtype)
    out = torch.full((b, major, minor + pad), fill, dtype=t.dtype)
    out[:, :, :minor] = t
    return out


def run_gpu(g, w: wl.Workload, A: torch.Tensor, B: torch.Tensor, bias, config=-1,
            out_dtype=None, layout_c="row", pad_a=0, pad_b=0, pad_c=0, stride_bias=0,
            return_plan_info=False, offset_a=0, offset_b=0):
    """A, B: host tensors (batch, major, minor) in storage order.  Returns C as a host
    tensor of logical shape (batch, M, N).  Padding is poisoned with NaN on the inputs
    and checked to be untouched on the output.  offset_a / offset_b: elements by which the
    operand's first element is displaced from its (256-byte aligned) allocation."""
    dev = torch.device("cuda:0")
    Ap, Bp = pad_minor(A, pad_a), pad_minor(B, pad_b)
    lda, ldb = Ap.shape[2], Bp.shape[2]
    c_major, c_minor = (w.M, w.N) if layout_c == "row" else (w.N, w.M)
    ldc = c_minor + pad_c
    odt = wl.TORCH_DTYPE[out_dtype or w.out_dtype or w.dtype]
    sentinel = -777.0
    Cd = torch.full((w.batch, c_major, ldc), sentinel, dtype=odt, device=dev)
    def displaced(X, off):
        if not off:
            return X.to(dev)
        buf = torch.zeros(X.numel() + off, dtype=X.dtype, device=dev)
        buf[off:] = X.to(dev).reshape(-1)
        return buf[off:].view(X.shape)
    Ad, Bd = displaced(Ap, offset_a), displaced(Bp, offset_b)
    biasd = bias.to(dev) if bias is not None else None
    desc = gpu_desc(g, w, out_dtype, layout_c, lda, ldb, ldc, stride_bias=stride_bias)
    plan = g.gemm_create_config(desc, config)
    info = plan.info()
    g.gemm_run(plan, Ad, Bd, Cd, biasd)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    Ch = Cd.cpu()
    if pad_c:
        assert torch.all(Ch[:, :, c_minor:] == sentinel), "padding of C was written"
    Ch = Ch[:, :, :c_minor]
    if layout_c == "col":
        Ch = Ch.transpose(1, 2)
    Ch = Ch.contiguous()
    return (Ch, info) if return_plan_info else Ch


def run_oracle(o, w: wl.Workload, A, B, bias, want=("y", "t", "s"), stride_bias=0):
    p = oracle_problem(o, w, stride_bias=stride_bias)
    return o.ref_gemm(p, wl.storage_numpy(A), wl.storage_numpy(B),
                      None if bias is None else bias.numpy(), want=want)


def e2_bound(w: wl.Workload, ref, out_dtype=None):
    """Per-element bound on |C - y| that any summation order in fp32 satisfies."""
    y, t, s = ref["y"], ref["t"], ref["s"]
    # Lipschitz constant of the activation (how an error of t shows in y) and the size of
    # the terms its fp32 evaluation rounds: |d/dt c t sigma(t)| <= 1.1 |c|,
    # |d/dt (c sigma(t) + t)| <= 1 + |c|/4.
    c = abs(w.scale)
    if "gelu" in w.epilogue:
        lip, mag = 1.13, 1.0
    elif "swish_scale" in w.epilogue:
        lip, mag = 1.1 * c, max(c, 1.0)
    elif "sigmoid_scale_residual" in w.epilogue:
        lip, mag = 1.0 + 0.25 * c, max(c, 1.0)
    else:
        lip, mag = 1.0, 1.0
    acc = w.K * U32 * s
    epi = 16 * U32 * mag * (np.abs(t) + 1.0) if w.epilogue != "none" else 0.0
    rnd = OUT_ROUNDOFF[out_dtype or w.out_dtype or w.dtype] * (np.abs(y) + lip * acc + epi) * 1.001
    return lip * acc + epi + rnd + 1e-30


def compare(w: wl.Workload, C: torch.Tensor, ref, A, B, bias, out_dtype=None):
    """All three error measures; returns a dict and asserts nothing."""
    c = wl.to_float64(C)
    y = ref["y"].reshape(c.shape)
    err = np.abs(c - y)
    scale = w.K * float(A.abs().max()) * float(B.abs().max())
    if bias is not None:
        scale += float(bias.abs().max())
    if "scale" in w.epilogue:
        scale = scale * max(abs(w.scale), 1.0) + abs(w.scale)
    res = {"e1": float(err.max() / scale), "finite": bool(np.isfinite(c).all())}
    if "s" in ref:
        bound = e2_bound(w, {k: v.reshape(c.shape) for k, v in ref.items()}, out_dtype)
        res["e2_worst"] = float((err / bound).max())
    eps = 1e-3 * float(np.sqrt(np.mean(y * y))) + 1e-30
    nu = err / (np.abs(y) + eps)
    res["e3_frac"] = float(np.mean(nu < 0.01))
    denom = float(np.linalg.norm(c.ravel()) * np.linalg.norm(y.ravel()))
    res["cosine"] = float(np.dot(c.ravel(), y.ravel()) / denom) if denom > 0 else 1.0
    return res


def assert_parity(w: wl.Workload, C, ref, A, B, bias, out_dtype=None):
    r = compare(w, C, ref, A, B, bias, out_dtype)
    assert r["finite"], r
    assert r["e1"] <= E1_TOL[w.dtype], r
    assert r["e2_worst"] <= 1.0, r
    assert r["e3_frac"] >= 0.99, r
    assert r["cosine"] >= 0.9999, r
    return r
