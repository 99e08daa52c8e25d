"""Maximum-size edge cases: outputs and operands beyond 2^31 elements / 2^32 bytes, so every
index that must be 64-bit is exercised.  Data is drawn on the device (torch's generator, seeded);
the oracle evaluates sampled outputs from the rows it needs, copied to the host."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def g():
    import paper_2603_12440_amd as g
    g.load_library()
    assert torch.cuda.is_available()
    return g


def device_normal(shape, seed, scale, dtype=torch.bfloat16):
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    return (torch.randn(shape, device="cuda:0", generator=gen, dtype=torch.float32) * scale).to(dtype)


def check_points(oracle, A_rows, B_rows, got, K, epilogue_code=None):
    """Point q of the sample is row q of A_rows against row q of B_rows (both host bf16, K contiguous):
    a diagonal of the small product the oracle evaluates."""
    n = A_rows.shape[0]
    p = oracle.Problem(n, n, K, oracle.DTYPE_BF16, oracle.DTYPE_BF16)
    idx = np.arange(n, dtype=np.int64)
    ref = oracle.ref_gemm_points(p, wl.storage_numpy(A_rows), wl.storage_numpy(B_rows), None,
                                 np.zeros(n, dtype=np.int64), idx, idx, want=("y", "s"))
    err = np.abs(got - ref["y"])
    bound = K * 2.0 ** -24 * ref["s"] + 2.0 ** -8 * 1.001 * (np.abs(ref["y"]) + K * 2.0 ** -24 * ref["s"]) + 1e-30
    assert np.all(err <= bound), float((err / bound).max())


def test_output_beyond_2_to_31_elements(g, oracle):
    """C = 66048 x 66048 bf16: 4.36e9 elements, 8.7 GB; K = 64.  Samples include the last row and
    column and positions on both sides of the 2^31-element and 2^32-byte marks of C."""
    M = N = 66048
    K = 64
    A = device_normal((M, K), 11, 1.0)
    B = device_normal((N, K), 12, 0.125)
    C = torch.full((M, N), -768.0, dtype=torch.bfloat16, device="cuda:0")
    plan = g.gemm_create(g.GemmDesc(M, N, K))
    say("large C:", plan.info())
    g.gemm_run(plan, A, B, C)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    assert not bool((C == -768.0).any())                       # every element written
    rng = np.random.Generator(np.random.Philox(key=5))
    flat = [0, M * N - 1, 2 ** 31 - 1, 2 ** 31, 2 ** 31 + 1, 2 ** 32 - 1, 2 ** 32, 2 ** 32 + 7]
    ii = [f // N for f in flat] + [M - 1, 0, M - 1] + [int(v) for v in rng.integers(0, M, 200)]
    jj = [f % N for f in flat] + [0, N - 1, N - 1] + [int(v) for v in rng.integers(0, N, 200)]
    it, jt = torch.tensor(ii, device="cuda:0"), torch.tensor(jj, device="cuda:0")
    got = C[it, jt].double().cpu().numpy()
    check_points(oracle, A[it].cpu(), B[jt].cpu(), got, K)


@pytest.mark.parametrize("M", [1, 4, 16])
def test_skinny_weight_beyond_2_to_32_bytes(g, oracle, M):
    """W = 270336 rows x 8192 bf16 = 4.4 GB: row offsets past 2^32 bytes in every skinny kernel."""
    N, K = 270336, 8192
    x = device_normal((M, K), 21, 1.0)
    W = device_normal((N, K), 22, 0.02)
    y = torch.full((M, N), -768.0, dtype=torch.bfloat16, device="cuda:0")
    plan = g.gemm_create(g.GemmDesc(M, N, K))
    say(f"large W, M={M}:", plan.info())
    assert "kernel=skinny" in plan.info()
    g.gemm_run(plan, x, W, y)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    assert not bool((y == -768.0).any())
    rng = np.random.Generator(np.random.Philox(key=6))
    first_past = 2 ** 32 // (K * 2)                            # first row that starts past 2^32 bytes
    cols = [0, N - 1, first_past - 1, first_past, first_past + 1, N - 32, N - 33] + \
           [int(v) for v in rng.integers(0, N, 120)]
    rows = [int(v) for v in rng.integers(0, M, len(cols))]
    rows[0], rows[1] = 0, M - 1
    it, jt = torch.tensor(rows, device="cuda:0"), torch.tensor(cols, device="cuda:0")
    got = y[it, jt].double().cpu().numpy()
    check_points(oracle, x[it].cpu(), W[jt].cpu(), got, K)


def test_rope_beyond_2_to_31_elements(g, oracle):
    """Query tensor of 2.4e9 elements (4.8 GB) plus a key tensor, rotated in place."""
    B, S, Hq, Hk, D = 18, 16384, 128, 8, 64
    assert B * S * Hq * D > 2 ** 31
    q = device_normal((B, S, Hq, D), 31, 1.0)
    k = device_normal((B, S, Hk, D), 32, 1.0)
    cos, sin = wl.rope_tables(S, D)
    # keep what the oracle needs before the tensors are overwritten
    rng = np.random.Generator(np.random.Philox(key=7))
    bs = [(0, 0), (B - 1, S - 1), (B // 2, S - 1), (B - 1, 0)] + \
         [(int(b), int(s)) for b, s in zip(rng.integers(0, B, 60), rng.integers(0, S, 60))]
    bi = torch.tensor([b for b, _ in bs], device="cuda:0")
    si = torch.tensor([s for _, s in bs], device="cuda:0")
    q_in, k_in = q[bi, si].cpu(), k[bi, si].cpu()               # [P, heads, D]
    desc = g.RopeDesc(B, S, D, dtype=g.BF16, table_dtype=g.F32)
    def tensor(x, heads):
        st = (S * heads * D, D, heads * D)
        return g.RopeTensor(x, x, heads, st, st)
    g.rope_apply(desc, [tensor(q, Hq), tensor(k, Hk)], cos.to("cuda:0"), sin.to("cuda:0"))
    torch.cuda.synchronize()
    P = len(bs)
    ci, sn = cos[si.cpu()].contiguous(), sin[si.cpu()].contiguous()   # [P, D]: one table row per sampled position
    for x_in, x_out, heads in ((q_in, q[bi, si].cpu(), Hq), (k_in, k[bi, si].cpu(), Hk)):
        # the sample as a problem of its own: batch 1, seq P, memory [P, heads, D]
        ref = oracle.ref_rope(1, heads, P, D, wl.storage_numpy(x_in), wl.storage_numpy(ci), wl.storage_numpy(sn),
                              dtype_x=oracle.DTYPE_BF16, dtype_table=oracle.DTYPE_F32,
                              stride_b=P * heads * D, stride_h=D, stride_s=heads * D)[0]     # [heads, P, D]
        got = wl.to_float64(x_out.transpose(0, 1))
        x64 = wl.to_float64(x_in.transpose(0, 1))
        rot = np.concatenate([x64[..., D // 2:], x64[..., :D // 2]], axis=-1)
        mag = np.abs(x64) * np.abs(wl.to_float64(ci))[None] + np.abs(rot) * np.abs(wl.to_float64(sn))[None]
        lim = 4 * 2.0 ** -24 * mag + 2.0 ** -8 * 1.001 * (np.abs(ref) + 4 * 2.0 ** -24 * mag) + 1e-30
        assert np.all(np.abs(got - ref) <= lim)
