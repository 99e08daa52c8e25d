"""GPU parity of the rotary embedding (include/rope.h) against the CPU oracle, through the C ABI."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

U_OUT = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24}
# half a unit in the last place below the smallest normal number (fp16 results near zero are
# subnormal: absolute spacing 2^-24)
SUBNORMAL_HALF_ULP = {"bf16": 0.0, "f16": 2.0 ** -25, "f32": 0.0}


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def g():
    import paper_2603_12440_amd as g
    g.load_library()
    assert torch.cuda.is_available()
    return g


def codes(g, oracle):
    return ({"f32": g.F32, "bf16": g.BF16, "f16": g.F16},
            {"f32": oracle.DTYPE_F32, "bf16": oracle.DTYPE_BF16, "f16": oracle.DTYPE_F16})


def bound(x_bhsd: np.ndarray, cos: np.ndarray, sin: np.ndarray, y: np.ndarray, dtype: str) -> np.ndarray:
    """|GPU - oracle| allowed per element: a few fp32 roundings of the two products, then one
    rounding to the storage type.  cos, sin broadcast to x's shape."""
    D = x_bhsd.shape[-1]
    rot = np.concatenate([x_bhsd[..., D // 2:], x_bhsd[..., :D // 2]], axis=-1)
    mag = np.abs(x_bhsd) * np.abs(cos) + np.abs(rot) * np.abs(sin)
    arith = 4 * 2.0 ** -24 * mag
    return arith + U_OUT[dtype] * (np.abs(y) + arith) * 1.001 + SUBNORMAL_HALF_ULP[dtype] + 1e-30


def run_case(g, oracle, B, H, S, D, dtype, table_dtype, layout, per_batch_table=False, in_place=False,
             elem_offset=0, seed=0, heads_k=0):
    """One tensor (or two, with heads_k) through rope_apply and through the oracle."""
    gd, od = codes(g, oracle)
    dev = torch.device("cuda:0")
    dt, tdt = wl.TORCH_DTYPE[dtype], wl.TORCH_DTYPE[table_dtype]
    tb = B if per_batch_table else 1
    cos = wl._draw(("uniform", 1.0), (tb, S, D), 100 + seed).to(tdt)
    sin = wl._draw(("uniform", 1.0), (tb, S, D), 200 + seed).to(tdt)
    desc = g.RopeDesc(B, S, D, dtype=gd[dtype], table_dtype=gd[table_dtype],
                      table_stride_b=S * D if per_batch_table else 0)
    tensors, keep = [], []
    for ti, heads in enumerate([H] + ([heads_k] if heads_k else [])):
        mem_shape = (B, S, heads, D) if layout == "bshd" else (B, heads, S, D)
        xh = wl._draw(("normal", 1.0), mem_shape, 300 + seed + ti).to(dt)
        n = xh.numel()
        # device buffers with `elem_offset` leading elements (misalignment) and a poisoned tail
        xbuf = torch.full((n + elem_offset + 16,), float("nan"), dtype=dt, device=dev)
        xbuf[elem_offset:elem_offset + n] = xh.reshape(-1).to(dev)
        ybuf = xbuf if in_place else torch.full((n + elem_offset + 16,), -768.0, dtype=dt, device=dev)
        strides = (S * heads * D, D, heads * D) if layout == "bshd" else (0, 0, 0)
        es = xbuf.element_size()
        tensors.append(g.RopeTensor(xbuf.data_ptr() + elem_offset * es, ybuf.data_ptr() + elem_offset * es,
                                    heads, strides, strides))
        keep.append((xh, xbuf, ybuf, mem_shape, strides, heads))
    cosd, sind = cos.to(dev), sin.to(dev)
    g.rope_apply(desc, tensors, cosd, sind)
    torch.cuda.synchronize()
    worst = 0.0
    for xh, xbuf, ybuf, mem_shape, strides, heads in keep:
        n = xh.numel()
        got_mem = ybuf[elem_offset:elem_offset + n].cpu().reshape(mem_shape)
        got = wl.to_float64(got_mem.transpose(1, 2) if layout == "bshd" else got_mem)
        ref = oracle.ref_rope(B, heads, S, D, wl.storage_numpy(xh), wl.storage_numpy(cos), wl.storage_numpy(sin),
                              dtype_x=od[dtype], dtype_table=od[table_dtype],
                              stride_b=strides[0], stride_h=strides[1], stride_s=strides[2],
                              table_stride_b=S * D if per_batch_table else 0)
        x64 = wl.to_float64(xh.transpose(1, 2) if layout == "bshd" else xh)
        c64 = wl.to_float64(cos)[:, None, :, :]
        s64 = wl.to_float64(sin)[:, None, :, :]
        lim = bound(x64, c64, s64, ref, dtype)
        err = np.abs(got - ref)
        assert np.isfinite(got).all()
        assert np.all(err <= lim), float((err / lim).max())
        worst = max(worst, float((err / lim).max()))
        # nothing outside the tensor was written
        tail = ybuf[elem_offset + n:].cpu().float()
        head = ybuf[:elem_offset].cpu().float()
        if in_place:
            assert torch.isnan(tail).all() and torch.isnan(head).all()
        else:
            assert torch.all(tail == -768.0) and torch.all(head == -768.0)
    return worst


@pytest.mark.parametrize("dtype,table_dtype", [("bf16", "f32"), ("bf16", "bf16"), ("f16", "f32"), ("f16", "f16"),
                                               ("f32", "f32")])
def test_rope_against_oracle_shapes_and_layouts(g, oracle, dtype, table_dtype):
    cases = [
        # B, H, S, D, layout
        (2, 8, 96, 64, "bshd"), (2, 8, 96, 64, "bhsd"), (1, 32, 37, 128, "bshd"), (3, 5, 19, 96, "bhsd"),
        (2, 3, 11, 40, "bshd"),      # 40 % 16 != 0: element-wise kernel
        (1, 1, 1, 2, "bhsd"), (1, 2, 300, 16, "bshd"), (2, 1, 1, 256, "bhsd"),
        (1, 3, 5, 512, "bshd"),      # a head vector fills a 64-lane group
        (1, 3, 5, 1024, "bshd"),     # half a head vector per 64-lane group: no lane exchange
        (2, 7, 9, 32, "bshd"),       # 4 lanes per head vector, 8 heads per group step, ragged head count
    ]
    for i, (B, H, S, D, layout) in enumerate(cases):
        say(f"rope {dtype}/{table_dtype} B={B} H={H} S={S} D={D} {layout}")
        r = run_case(g, oracle, B, H, S, D, dtype, table_dtype, layout, seed=i)
        say("    worst err/bound", round(r, 3))


def test_rope_two_tensors_in_place_tables_per_batch_and_misalignment(g, oracle):
    say("rope q+k one launch")
    run_case(g, oracle, 2, 8, 50, 64, "bf16", "f32", "bshd", heads_k=2, seed=11)
    run_case(g, oracle, 2, 3, 7, 40, "f16", "f16", "bhsd", heads_k=5, seed=12)
    say("rope in place")
    run_case(g, oracle, 2, 8, 50, 64, "bf16", "f32", "bshd", in_place=True, seed=13)
    run_case(g, oracle, 1, 4, 33, 128, "f32", "f32", "bhsd", in_place=True, heads_k=1, seed=14)
    say("rope per-batch tables")
    run_case(g, oracle, 3, 4, 21, 64, "bf16", "bf16", "bshd", per_batch_table=True, seed=15)
    say("rope rows not 16-byte aligned -> element-wise kernel")
    run_case(g, oracle, 2, 4, 21, 64, "bf16", "f32", "bshd", elem_offset=1, seed=16)
    run_case(g, oracle, 2, 4, 21, 64, "f32", "f32", "bhsd", elem_offset=3, heads_k=2, seed=17)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_rope_exact_special_tables(g, dtype):
    """cos = 1, sin = 0: bit-exact copy; cos = 0, sin = 1: (-x2, x1) bit-exact; and a model's
    tables keep every pair's norm (to the rounding of the output type)."""
    dev = torch.device("cuda:0")
    gd = {"f32": g.F32, "bf16": g.BF16, "f16": g.F16}
    B, H, S, D = 2, 4, 33, 64
    dt = wl.TORCH_DTYPE[dtype]
    x = wl._draw(("normal", 1.0), (B, H, S, D), 5).to(dt).to(dev)
    y = torch.empty_like(x)
    one, zero = torch.ones((S, D), device=dev), torch.zeros((S, D), device=dev)
    desc = g.RopeDesc(B, S, D, dtype=gd[dtype])
    g.rope_apply(desc, [g.RopeTensor(x, y, H)], one, zero)
    torch.cuda.synchronize()
    assert torch.equal(y, x)
    g.rope_apply(desc, [g.RopeTensor(x, y, H)], zero, one)
    torch.cuda.synchronize()
    assert torch.equal(y, torch.cat([-x[..., D // 2:], x[..., :D // 2]], dim=-1))
    cos, sin = wl.rope_tables(S, D)
    g.rope_apply(desc, [g.RopeTensor(x, y, H)], cos.to(dev), sin.to(dev))
    torch.cuda.synchronize()
    xf, yf = x.double().cpu(), y.double().cpu()
    n_in = xf[..., :D // 2] ** 2 + xf[..., D // 2:] ** 2
    n_out = yf[..., :D // 2] ** 2 + yf[..., D // 2:] ** 2
    assert torch.all((n_out - n_in).abs() <= 4 * U_OUT[dtype] * n_in + 1e-12)
    # position 0 has angle 0: untouched
    assert torch.equal(y[:, :, 0], x[:, :, 0])


@pytest.mark.parametrize("name", sorted(wl.ROPE_WORKLOADS))
def test_rope_workloads_full_size_sampled(g, oracle, name):
    """Every benchmark shape at full size, both tensors in one launch as bench.py times it; the
    oracle evaluates a sample of positions (first, last, around the workgroup seams, random)."""
    w = wl.ROPE_WORKLOADS[name]
    gd, od = codes(g, oracle)
    dev = torch.device("cuda:0")
    q, k, cos, sin = wl.make_rope_inputs(w)
    say(f"rope full size {name}: q {tuple(q.shape)} k {tuple(k.shape)}")
    qd, kd = q.to(dev), k.to(dev)
    qy, ky = torch.full_like(qd, -768.0), torch.full_like(kd, -768.0)
    desc = g.RopeDesc(w.batch, w.seq, w.head_dim, dtype=gd[w.dtype], table_dtype=gd[w.table_dtype])
    def tensor(x, y, heads):
        st = (w.seq * heads * w.head_dim, w.head_dim, heads * w.head_dim)
        return g.RopeTensor(x, y, heads, st, st)
    g.rope_apply(desc, [tensor(qd, qy, w.heads_q), tensor(kd, ky, w.heads_k)], cos.to(dev), sin.to(dev))
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.Philox(key=99))
    pos = sorted(set([0, 1, 2, 3, 4, 5, 6, 7, w.seq - 1, w.seq - 2, w.seq // 2] +
                     [int(p) for p in rng.integers(0, w.seq, 40)]))
    for x, y, heads in ((q, qy.cpu(), w.heads_q), (k, ky.cpu(), w.heads_k)):
        assert not torch.any(y == -768.0)                      # everything was written
        xs = x[:, pos].contiguous()                            # [B, P, heads, D] memory
        P = len(pos)
        ref = oracle.ref_rope(w.batch, heads, P, w.head_dim, wl.storage_numpy(xs),
                              wl.storage_numpy(cos[pos].contiguous()), wl.storage_numpy(sin[pos].contiguous()),
                              dtype_x=od[w.dtype], dtype_table=od[w.table_dtype],
                              stride_b=P * heads * w.head_dim, stride_h=w.head_dim, stride_s=heads * w.head_dim)
        got = wl.to_float64(y[:, pos].transpose(1, 2))
        x64 = wl.to_float64(xs.transpose(1, 2))
        c64 = wl.to_float64(cos[pos])[None, None]
        s64 = wl.to_float64(sin[pos])[None, None]
        lim = bound(x64, c64, s64, ref, w.dtype)
        err = np.abs(got - ref)
        assert np.all(err <= lim), float((err / lim).max())
