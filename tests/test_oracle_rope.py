"""Pins for the rotary-embedding oracle (oracle/ref_rope.c): things the definition and the
mathematics fix, chosen so that a wrong sign, a swapped half, a table index taken from the
partner element, or a stride mix-up fails at least one of them.  No GPU."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import workloads as wl


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def test_worked_example(oracle):
    """D = 4, x = (1, 2, 3, 4), cos = 0.6, sin = 0.8 everywhere:
    y = (1*0.6 - 3*0.8, 2*0.6 - 4*0.8, 3*0.6 + 1*0.8, 4*0.6 + 2*0.8) = (-1.8, -2.0, 2.6, 4.0)."""
    x = _f32([1, 2, 3, 4]); c = _f32([0.6] * 4); s = _f32([0.8] * 4)
    y = oracle.ref_rope(1, 1, 1, 4, x, c, s, dtype_x=oracle.DTYPE_F32)[0, 0, 0]
    c64, s64 = float(np.float32(0.6)), float(np.float32(0.8))      # the stored fp32 values, exactly
    want = [1 * c64 - 3 * s64, 2 * c64 - 4 * s64, 3 * c64 + 1 * s64, 4 * c64 + 2 * s64]
    assert np.array_equal(y, np.array(want))
    assert np.allclose(y, [-1.8, -2.0, 2.6, 4.0], atol=1e-7)


def test_every_index_uses_its_own_table_entry(oracle):
    """Tables whose halves differ: y[i] = x[i] cos[i] + rot[i] sin[i] with index i's own entries
    (the PyTorch reference multiplies element-wise), exact in small integers."""
    x = _f32([1, 2, 3, 4, 5, 6])
    c = _f32([2, 3, 5, 7, 11, 13]); s = _f32([1, -1, 2, -2, 3, -3])
    y = oracle.ref_rope(1, 1, 1, 6, x, c, s, dtype_x=oracle.DTYPE_F32)[0, 0, 0]
    rot = np.array([-4, -5, -6, 1, 2, 3], dtype=np.float64)
    assert np.array_equal(y, x * c.astype(np.float64) + rot * s)


def test_identity_and_quarter_turn(oracle):
    """cos = 1, sin = 0 leaves x alone; cos = 0, sin = 1 gives rotate_half(x) = (-x2, x1);
    cos = -1, sin = 0 negates.  Exact for every storage type."""
    rng = np.random.default_rng(5)
    B, H, S, D = 2, 3, 5, 8
    for dt, code in (("bf16", oracle.DTYPE_BF16), ("f16", oracle.DTYPE_F16), ("f32", oracle.DTYPE_F32)):
        xt = torch.from_numpy(rng.standard_normal((B, H, S, D)).astype(np.float32)).to(wl.TORCH_DTYPE[dt])
        x64 = wl.to_float64(xt)
        one, zero = _f32(np.ones((S, D))), _f32(np.zeros((S, D)))
        y = oracle.ref_rope(B, H, S, D, wl.storage_numpy(xt), one, zero, dtype_x=code)
        assert np.array_equal(y, x64)
        y = oracle.ref_rope(B, H, S, D, wl.storage_numpy(xt), zero, one, dtype_x=code)
        assert np.array_equal(y, np.concatenate([-x64[..., D // 2:], x64[..., :D // 2]], axis=-1))
        y = oracle.ref_rope(B, H, S, D, wl.storage_numpy(xt), -one, zero, dtype_x=code)
        assert np.array_equal(y, -x64)


def test_pair_norms_and_composition(oracle):
    """With repeated halves (cos t, sin t) each pair (x[i], x[i+D/2]) is turned by the angle t:
    its norm is kept, turning by a then by b equals turning by a + b, and turning by -a undoes it."""
    rng = np.random.default_rng(6)
    S, D = 7, 16
    x = _f32(rng.standard_normal((1, 1, S, D)))
    a = rng.uniform(-3, 3, (S, D // 2)); b = rng.uniform(-3, 3, (S, D // 2))
    def tables(t):
        t2 = np.concatenate([t, t], axis=1)
        return np.cos(t2), np.sin(t2)
    def rope(v, t):
        c, s = tables(t)
        # fp64 tables handed over as two fp32 pieces would lose the point; use fp32 tables and
        # loosen the tolerance to their rounding instead
        return oracle.ref_rope(1, 1, S, D, _f32(v), _f32(c), _f32(s), dtype_x=oracle.DTYPE_F32)
    ya = rope(x, a)
    n_in = x[0, 0, :, :D // 2].astype(np.float64) ** 2 + x[0, 0, :, D // 2:].astype(np.float64) ** 2
    n_out = ya[0, 0, :, :D // 2] ** 2 + ya[0, 0, :, D // 2:] ** 2
    assert np.allclose(n_out, n_in, rtol=1e-6, atol=0)
    yab = rope(ya, b)
    assert np.allclose(yab, rope(x, a + b), rtol=0, atol=2e-6)
    assert np.allclose(rope(ya, -a), x.astype(np.float64), rtol=0, atol=2e-6)
    # direction of the turn: the pair (1, 0) at angle t goes to (cos t, sin t)
    e = np.zeros((1, 1, S, D), dtype=np.float32); e[..., :D // 2] = 1.0
    ye = rope(e, a)
    assert np.allclose(ye[0, 0, :, :D // 2], np.cos(a), atol=1e-7)
    assert np.allclose(ye[0, 0, :, D // 2:], np.sin(a), atol=1e-7)


def test_relative_position_property(oracle):
    """The reason the method exists: with a language model's tables, <rope_m(q), rope_n(k)>
    depends on m - n only."""
    D, S = 32, 40
    rng = np.random.default_rng(7)
    q = _f32(rng.standard_normal(D)); k = _f32(rng.standard_normal(D))
    cos, sin = wl.rope_tables(S, D, theta=10000.0)
    Q = oracle.ref_rope(1, 1, S, D, _f32(np.tile(q, (S, 1))), cos.numpy(), sin.numpy(), dtype_x=oracle.DTYPE_F32)[0, 0]
    K = oracle.ref_rope(1, 1, S, D, _f32(np.tile(k, (S, 1))), cos.numpy(), sin.numpy(), dtype_x=oracle.DTYPE_F32)[0, 0]
    G = Q @ K.T                      # G[m, n] must be a function of m - n
    for d in (-5, 0, 1, 13):
        diag = np.array([G[m, m - d] for m in range(max(d, 0), min(S, S + d))])
        assert np.ptp(diag) < 2e-5 * (np.linalg.norm(q) * np.linalg.norm(k)), d
    assert abs(G[0, 0] - float(q.astype(np.float64) @ k.astype(np.float64))) < 1e-5


def test_strides_batches_and_table_batches(oracle):
    """[batch, seq, heads, D] memory read as a strided [batch, heads, seq, D] view equals the packed
    computation; a per-batch table is used by its own batch only; heads share the table row of
    their position."""
    rng = np.random.default_rng(8)
    B, H, S, D = 2, 3, 4, 8
    x_bshd = _f32(rng.standard_normal((B, S, H, D)))
    cos = _f32(rng.standard_normal((B, S, D))); sin = _f32(rng.standard_normal((B, S, D)))
    y = oracle.ref_rope(B, H, S, D, x_bshd, cos, sin, dtype_x=oracle.DTYPE_F32,
                        stride_b=S * H * D, stride_h=D, stride_s=H * D, table_stride_b=S * D)
    x_bhsd = np.ascontiguousarray(x_bshd.transpose(0, 2, 1, 3))
    y2 = oracle.ref_rope(B, H, S, D, x_bhsd, cos, sin, dtype_x=oracle.DTYPE_F32, table_stride_b=S * D)
    assert np.array_equal(y, y2)
    # brute force, element by element, straight from the definition
    for b in range(B):
        for h in range(H):
            for s in range(S):
                v = x_bhsd[b, h, s].astype(np.float64)
                rot = np.concatenate([-v[D // 2:], v[:D // 2]])
                assert np.array_equal(y[b, h, s], v * cos[b, s].astype(np.float64) + rot * sin[b, s].astype(np.float64))
    # shared table = batch 0's table for everyone
    y3 = oracle.ref_rope(B, H, S, D, x_bhsd, cos[0], sin[0], dtype_x=oracle.DTYPE_F32)
    assert np.array_equal(y3[0], y2[0]) and not np.array_equal(y3[1], y2[1])


def test_16bit_tables_and_argument_checks(oracle):
    B, H, S, D = 1, 2, 3, 4
    x = torch.arange(B * H * S * D, dtype=torch.float32).reshape(B, H, S, D).to(torch.bfloat16)
    cos = torch.full((S, D), 0.5, dtype=torch.bfloat16); sin = torch.full((S, D), -0.25, dtype=torch.bfloat16)
    y = oracle.ref_rope(B, H, S, D, wl.storage_numpy(x), wl.storage_numpy(cos), wl.storage_numpy(sin),
                        dtype_x=oracle.DTYPE_BF16, dtype_table=oracle.DTYPE_BF16)
    x64 = wl.to_float64(x)
    rot = np.concatenate([-x64[..., 2:], x64[..., :2]], axis=-1)
    assert np.array_equal(y, 0.5 * x64 - 0.25 * rot)
    with pytest.raises(ValueError):
        oracle.ref_rope(1, 1, 1, 3, _f32([1, 2, 3]), _f32([1, 1, 1]), _f32([0, 0, 0]), dtype_x=oracle.DTYPE_F32)
    with pytest.raises(ValueError):
        oracle.ref_rope(1, 1, 2, 4, _f32([1, 2, 3, 4]), _f32([1] * 8), _f32([0] * 8), dtype_x=oracle.DTYPE_F32)
