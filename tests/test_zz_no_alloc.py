"""gemm_run_fixed_scratch: the entry point that allocates nothing (split-K partials in the
library's own fixed device buffer).  Two calls in a row through the C ABI, the second on a
smaller problem, each compared bit for bit with gemm_run_workspace on the same plan (the entry
point it is a variant of) and with the CPU oracle to the usual bounds; a plan that needs more
than the fixed buffer is refused; a plan without a workspace runs as with gemm_run."""
from __future__ import annotations

import sys

import pytest
import torch

import workloads as wl
from helpers import assert_parity, gpu_desc, run_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2603_12440_amd as g
    g.load_library()          # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available()
    return g


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def one_call(g, oracle, w, splits):
    dev = torch.device("cuda:0")
    A, B, bias = wl.make_inputs(w)
    Ad, Bd = A.to(dev), B.to(dev)
    bd = None if bias is None else bias.to(dev)
    plan = g.gemm_create_splitk(gpu_desc(g, w), splits)
    need = g.gemm_workspace_bytes(plan)
    say(f"fixed scratch: {w.M}x{w.N}x{w.K} {w.epilogue} splits={splits}: {plan.info()}")
    assert 0 < need <= g.FIXED_SCRATCH_BYTES
    odt = wl.TORCH_DTYPE[w.out_dtype or w.dtype]
    C_fixed = torch.full((1, w.M, w.N), -777.0, dtype=odt, device=dev)
    g.gemm_run_fixed_scratch(plan, Ad, Bd, C_fixed, bd)
    torch.cuda.synchronize()
    # the entry point it is a variant of, with a workspace of the caller's
    ws = torch.empty(need // 4, dtype=torch.float32, device=dev)
    C_ws = torch.full((1, w.M, w.N), -777.0, dtype=odt, device=dev)
    g.gemm_run_workspace(plan, Ad, Bd, C_ws, bd, ws)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    assert torch.equal(C_fixed.view(torch.int16), C_ws.view(torch.int16)), "differs from gemm_run_workspace"
    ref = run_oracle(oracle, w, A, B, bias)
    assert_parity(w, C_fixed.cpu(), ref, A, B, bias)


def test_fixed_scratch_two_calls_then_limits(g, oracle):
    big = wl.Workload("t", 520, 392, 8192, dist_b=("normal", 1.0 / 90), epilogue="bias_gelu_erf",
                      dist_bias=("uniform", 0.5), seed_a=41, seed_b=42, seed_bias=43)
    small = wl.Workload("t", 130, 72, 2048, dist_b=("normal", 1.0 / 45), epilogue="none", seed_a=44, seed_b=45)
    one_call(g, oracle, big, 16)          # 16 x 520 x 392 fp32 partials = 13 MB of the buffer
    one_call(g, oracle, small, 4)         # the same buffer again, a smaller problem: nothing stale shows
    one_call(g, oracle, big, 8)

    dev = torch.device("cuda:0")
    # more workspace than the fixed buffer holds: refused, nothing enqueued
    w = wl.Workload("t", 2048, 2048, 4096)
    plan = g.gemm_create_splitk(gpu_desc(g, w), 4)                     # 4 x 2048 x 2048 x 4 B = 64 MiB
    assert g.gemm_workspace_bytes(plan) > g.FIXED_SCRATCH_BYTES
    x = torch.zeros(8, dtype=torch.bfloat16, device=dev)
    with pytest.raises(g.GemmError) as e:
        g.gemm_run_fixed_scratch(plan, x, x, x)                        # (refused before any pointer is used)
    assert e.value.status == -12 and "fixed scratch" in str(e.value)
    g.gemm_destroy(plan)

    # a plan without a workspace runs as with gemm_run
    w = wl.Workload("t", 300, 264, 256, seed_a=46, seed_b=47)
    A, B, _ = wl.make_inputs(w)
    plan = g.gemm_create(gpu_desc(g, w))
    C1 = torch.empty((1, w.M, w.N), dtype=torch.bfloat16, device=dev)
    C2 = torch.empty_like(C1)
    g.gemm_run_fixed_scratch(plan, A.to(dev), B.to(dev), C1)
    g.gemm_run(plan, A.to(dev), B.to(dev), C2)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    assert torch.equal(C1.view(torch.int16), C2.view(torch.int16))
