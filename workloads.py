"""Seeded synthetic inputs for C = epilogue(A.B) and for the rotary embedding, shared by the CPU oracle's
tests and the GPU library's tests / bench.

This module holds no GEMM arithmetic: it only draws random (or structured)
operand values, rounds them to their storage type with the library cast
(round to nearest even) and describes the benchmark shapes.  Neither the
oracle nor the GPU library is imported here.

The paper evaluates on public kernel-benchmark suites whose matmul-family tasks
(matrix-vector product, matmul with a small K, matmul + activation, FFN-shaped
layers; App. "Per-task results") are not reproduced here; the shapes below are
synthetic stand-ins for that workload class.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16,
               "f8": torch.float8_e4m3fn}     # OCP E4M3: operands only, results are bf16 or fp32


@dataclass(frozen=True)
class Workload:
    """A named problem: logical shape, storage, value distributions, seeds.

    layout 'row' / 'col' refers to the logical matrices A (M x K), B (K x N).
    dist = (kind, scale): kind 'normal' -> scale * N(0,1); 'uniform' -> U[-scale, scale].
    """
    name: str
    M: int
    N: int
    K: int
    dtype: str = "bf16"            # storage type of A, B and C ("f8": A and B only, C is out_dtype)
    out_dtype: Optional[str] = None   # storage type of C when it differs from dtype
    layout_a: str = "row"
    layout_b: str = "col"
    dist_a: Tuple[str, float] = ("normal", 1.0)
    dist_b: Tuple[str, float] = ("normal", 1.0)
    epilogue: str = "none"         # 'none' | 'bias' | 'bias_relu' | 'bias_gelu_erf' | 'bias_gelu_tanh' | 'relu' | 'gelu_erf'
                                   # | '[bias_]swish_scale' | '[bias_]sigmoid_scale_residual'
    scale: float = 1.0             # the scalar of the *_scale epilogues
    dist_bias: Tuple[str, float] = ("uniform", 0.1)
    batch: int = 1
    seed_a: int = 1
    seed_b: int = 2
    seed_bias: int = 3
    bound: str = "mfma"            # roofline that bounds it: 'mfma' | 'hbm' | 'latency'

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K * self.batch

    @property
    def bytes(self) -> float:
        """Compulsory traffic: read A and B once, write C once (bias ignored)."""
        e = torch.empty((), dtype=TORCH_DTYPE[self.dtype]).element_size()
        ec = torch.empty((), dtype=TORCH_DTYPE[self.out_dtype or self.dtype]).element_size()
        return float(self.batch * (e * (self.M * self.K + self.K * self.N) + ec * self.M * self.N))

    @property
    def has_bias(self) -> bool:
        return self.epilogue.startswith("bias")


def _k(n):  # 1/sqrt(K) scaling used by the square and epilogue shapes
    return 1.0 / float(np.sqrt(n))


WORKLOADS = {w.name: w for w in [
    # small fp32 case the oracle finishes in well under a second
    Workload("f32_256", 256, 256, 256, dtype="f32", layout_b="row",
             dist_a=("uniform", 1.0), dist_b=("uniform", 1.0),
             seed_a=1001, seed_b=1002, bound="latency"),
    # square bf16, the headline shape
    Workload("square_8192", 8192, 8192, 8192, dist_a=("normal", _k(8192)),
             dist_b=("normal", _k(8192)), seed_a=2001, seed_b=2002),
    # LLM-layer shapes: activations N(0,1), weights N(0, 0.02)
    Workload("llm_4096x14336x4096", 4096, 14336, 4096, dist_b=("normal", 0.02),
             seed_a=3001, seed_b=3002),
    Workload("llm_4096x4096x14336", 4096, 4096, 14336, dist_b=("normal", 0.02),
             seed_a=3003, seed_b=3004),
    Workload("llm_4096x6144x4096", 4096, 6144, 4096, dist_b=("normal", 0.02),
             seed_a=3005, seed_b=3006),
    # decode-shaped skinny products (HBM-bound)
    *[Workload(f"skinny_m{m}_n{n}", m, n, 8192, dist_b=("normal", 0.02),
               seed_a=4001 + 10 * q + r, seed_b=4002 + 10 * q + r, bound="hbm")
      for q, n in enumerate((8192, 28672)) for r, m in enumerate((1, 4, 16))],
    # fused bias + GELU epilogue, and the strided-batched variant
    Workload("gelu_8192x16384x4096", 8192, 16384, 4096, dist_a=("normal", _k(4096)),
             dist_b=("normal", _k(4096)), epilogue="bias_gelu_erf",
             seed_a=5001, seed_b=5002, seed_bias=5003),
    # the two scaled post-ops on the same shape
    Workload("swish_8192x16384x4096", 8192, 16384, 4096, dist_a=("normal", _k(4096)),
             dist_b=("normal", 1.5 * _k(4096)), epilogue="bias_swish_scale", scale=2.0,
             dist_bias=("uniform", 1.0), seed_a=5011, seed_b=5012, seed_bias=5013),
    Workload("sigres_8192x16384x4096", 8192, 16384, 4096, dist_a=("normal", _k(4096)),
             dist_b=("normal", 1.5 * _k(4096)), epilogue="bias_sigmoid_scale_residual", scale=0.5,
             dist_bias=("uniform", 1.0), seed_a=5021, seed_b=5022, seed_bias=5023),
    # 8-bit floating-point operands (E4M3), bf16 result: the square shape and an LLM layer shape
    Workload("f8_square_8192", 8192, 8192, 8192, dtype="f8", out_dtype="bf16", dist_a=("normal", 1.0),
             dist_b=("normal", 1.0), seed_a=8001, seed_b=8002),
    Workload("f8_llm_4096x14336x4096", 4096, 14336, 4096, dtype="f8", out_dtype="bf16", dist_a=("normal", 1.0),
             dist_b=("normal", 0.25), seed_a=8003, seed_b=8004),
    # few output tiles, long K: the split-K case
    Workload("smallmn_512x512x32768", 512, 512, 32768, dist_a=("normal", 1.0),
             dist_b=("normal", _k(32768)), seed_a=6001, seed_b=6002),
    Workload("batched_64x512x512x128", 512, 512, 128, dist_a=("normal", _k(128)),
             dist_b=("normal", _k(128)), batch=64, seed_a=5004, seed_b=5005,
             seed_bias=5006, bound="hbm"),
]}


@dataclass(frozen=True)
class RopeWorkload:
    """One rotary-embedding problem: query and key tensors of a decoder layer, logical
    shape [batch, heads, seq, head_dim], stored as the projection leaves them
    ([batch, seq, heads, head_dim] in memory, i.e. the heads axis is a strided view), and
    per-position cos / sin tables [seq, head_dim] shared by all batches and heads."""
    name: str
    batch: int
    heads_q: int
    heads_k: int
    seq: int
    head_dim: int
    dtype: str = "bf16"
    table_dtype: str = "f32"
    theta: float = 500000.0        # frequency base of the tables
    seed_q: int = 7001
    seed_k: int = 7002

    @property
    def elements(self) -> int:
        return self.batch * (self.heads_q + self.heads_k) * self.seq * self.head_dim

    @property
    def bytes(self) -> float:
        """Compulsory traffic: every element of q and k read once and written once, the tables once."""
        e = torch.empty((), dtype=TORCH_DTYPE[self.dtype]).element_size()
        t = torch.empty((), dtype=TORCH_DTYPE[self.table_dtype]).element_size()
        return float(2 * e * self.elements + 2 * t * self.seq * self.head_dim)


ROPE_WORKLOADS = {w.name: w for w in [
    # small case the oracle finishes at once
    RopeWorkload("rope_small", 2, 8, 2, 96, 64),
    # the layer shape of a 1B-parameter Llama-style decoder (32 query heads, 8 key heads of 64), long batch
    RopeWorkload("rope_llama1b_b8_s4096", 8, 32, 8, 4096, 64),
    # 128-wide heads (8B-class layer)
    RopeWorkload("rope_h32_d128_b4_s4096", 4, 32, 8, 4096, 128),
]}


def rope_tables(seq: int, head_dim: int, theta: float = 500000.0, dtype: str = "f32", offset: int = 0):
    """cos / sin tables [seq, head_dim] as a language model builds them: angle of position p and
    pair j is p * theta^(-2j / head_dim), the two halves of a row repeat.  Computed in fp64,
    stored in `dtype`."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    inv = theta ** (-2.0 * j / head_dim)
    ang = (np.arange(seq, dtype=np.float64)[:, None] + offset) * inv[None, :]
    ang = np.concatenate([ang, ang], axis=1)
    dt = TORCH_DTYPE[dtype]
    return torch.from_numpy(np.cos(ang)).to(dt), torch.from_numpy(np.sin(ang)).to(dt)


def make_rope_inputs(w: RopeWorkload):
    """q, k as host tensors of MEMORY shape [batch, seq, heads, head_dim] (logical [b, h, s, d]
    is their transpose(1, 2)), N(0,1) entries; cos, sin tables [seq, head_dim]."""
    dt = TORCH_DTYPE[w.dtype]
    q = _draw(("normal", 1.0), (w.batch, w.seq, w.heads_q, w.head_dim), w.seed_q).to(dt)
    k = _draw(("normal", 1.0), (w.batch, w.seq, w.heads_k, w.head_dim), w.seed_k).to(dt)
    cos, sin = rope_tables(w.seq, w.head_dim, w.theta, w.table_dtype)
    return q, k, cos, sin


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (e.g. a smaller shape with
    the same distributions, for parity tests the oracle finishes in seconds)."""
    return replace(w, **changes)


def _draw(dist: Tuple[str, float], shape, seed: int) -> torch.Tensor:
    rng = np.random.Generator(np.random.Philox(key=seed))
    kind, scale = dist
    if kind == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
        x *= np.float32(scale)
    elif kind == "uniform":
        x = rng.random(shape, dtype=np.float32)
        x = (x * np.float32(2.0) - np.float32(1.0)) * np.float32(scale)
    else:
        raise ValueError(kind)
    return torch.from_numpy(x)


def operand_shapes(w: Workload):
    """Storage shapes (batch, major, minor) of A and B for the workload's layouts."""
    a = (w.batch, w.M, w.K) if w.layout_a == "row" else (w.batch, w.K, w.M)
    b = (w.batch, w.K, w.N) if w.layout_b == "row" else (w.batch, w.N, w.K)
    return a, b


def make_inputs(w: Workload):
    """Host tensors in storage order and storage dtype: A, B and bias (fp32 or None)."""
    sa, sb = operand_shapes(w)
    dt = TORCH_DTYPE[w.dtype]
    A = _draw(w.dist_a, sa, w.seed_a).to(dt)
    B = _draw(w.dist_b, sb, w.seed_b).to(dt)
    bias = _draw(w.dist_bias, (w.N,), w.seed_bias) if w.has_bias else None
    return A, B, bias


def storage_numpy(t: Optional[torch.Tensor]):
    """A host tensor as the flat numpy storage buffer the oracle reads:
    float32 values, or uint16 bit patterns for bf16 / fp16."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy().reshape(-1)
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16).reshape(-1)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy().reshape(-1)
    raise TypeError(t.dtype)


def to_float64(t: torch.Tensor) -> np.ndarray:
    """Exact fp64 values of a result tensor of any supported storage type."""
    return t.detach().cpu().to(torch.float64).numpy()


# ---- structured operands (closed-form tests) --------------------------------

def small_integers(shape, seed: int, lo: int = -2, hi: int = 2, dtype: str = "bf16") -> torch.Tensor:
    """Integers in [lo, hi]: exact in every storage type, and so are their
    products and (for moderate K) sums in fp32."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    x = rng.integers(lo, hi + 1, size=shape).astype(np.float32)
    return torch.from_numpy(x).to(TORCH_DTYPE[dtype])


def one_hot_columns(rows: int, K: int, ks, dtype: str = "bf16") -> torch.Tensor:
    """rows x K matrix (K contiguous) whose row r has a single 1 at k = ks[r % len(ks)]."""
    x = torch.zeros((rows, K), dtype=torch.float32)
    ks = list(ks)
    for r in range(rows):
        x[r, ks[r % len(ks)]] = 1.0
    return x.to(TORCH_DTYPE[dtype])


def sample_points(w: Workload, n_random: int, seed: int, tile: int = 256):
    """Output positions for sampled checks at full size: every corner of the
    tile lattice (first/last row and column of each tile, clipped to a few
    thousand points) plus n_random uniformly drawn positions."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    edges_i = sorted({i for t in range(0, w.M, tile) for i in (t, min(t + tile, w.M) - 1)})
    edges_j = sorted({j for t in range(0, w.N, tile) for j in (t, min(t + tile, w.N) - 1)})
    ii, jj = np.meshgrid(np.array(edges_i), np.array(edges_j), indexing="ij")
    ii, jj = ii.reshape(-1), jj.reshape(-1)
    if ii.size > 4096:
        keep = rng.choice(ii.size, 4096, replace=False)
        ii, jj = ii[keep], jj[keep]
    ri = rng.integers(0, w.M, n_random)
    rj = rng.integers(0, w.N, n_random)
    pi = np.concatenate([ii, ri]).astype(np.int64)
    pj = np.concatenate([jj, rj]).astype(np.int64)
    pb = rng.integers(0, w.batch, pi.size).astype(np.int64)
    return pb, pi, pj
