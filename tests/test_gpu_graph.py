"""The entry points only enqueue kernels: no allocation, no synchronisation, no memset.  A HIP graph
captured around them must therefore replay correctly, replay after replay, with eager work in between."""
from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

import workloads as wl
from helpers import gpu_desc

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def g():
    import paper_2603_12440_amd as g
    g.load_library()
    assert torch.cuda.is_available()
    return g


def test_graph_replays_match_eager_runs(g):
    dev = torch.device("cuda:0")
    big = wl.Workload("t", 300, 520, 264, epilogue="bias_gelu_erf", seed_a=3, seed_b=4, seed_bias=5)   # MFMA kernel
    thin = wl.Workload("t", 4, 520, 264, seed_a=3, seed_b=4)                                           # skinny kernel
    deep = wl.Workload("t", 256, 256, 4096, seed_a=6, seed_b=7)                                        # split-K, two kernels
    cases = []
    for w in (big, thin, deep):
        sa, sb = wl.operand_shapes(w)
        A = [wl.small_integers(sa, 10 + i, -2, 2).to(dev) for i in range(2)]
        B = wl.small_integers(sb, 20, -2, 2).to(dev)
        bias = wl.small_integers((w.N,), 30, -3, 3, "f32").to(dev) if w.has_bias else None
        C = torch.empty((1, w.M, w.N), dtype=wl.TORCH_DTYPE[w.dtype], device=dev)
        if w is deep:
            plan = g.gemm_create_splitk(gpu_desc(g, w), 4)
            ws = torch.empty(g.gemm_workspace_bytes(plan) // 4, dtype=torch.float32, device=dev)
            run = (lambda plan=plan, B=B, C=C, bias=bias, ws=ws: lambda a: g.gemm_run_workspace(plan, a, B, C, bias, ws))()
        else:
            plan = g.gemm_create(gpu_desc(g, w))
            run = (lambda plan=plan, B=B, C=C, bias=bias: lambda a: g.gemm_run(plan, a, B, C, bias))()
        say("graph case: " + plan.info())
        # eager results for both inputs (this also makes the library's one-time device check outside the capture)
        want = []
        for a in A:
            run(a)
            torch.cuda.synchronize()
            want.append(C.clone())
        cases.append((plan, A, C, run, want))

    stream = torch.cuda.Stream()
    for plan, A, C, run, want in cases:
        a_in = A[0].clone()                                     # the graph reads this buffer; its content changes between replays
        graph = torch.cuda.CUDAGraph()
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=stream):
            run(a_in)                                           # the binding enqueues on torch's current (capturing) stream
        for rep in range(4):
            which = rep % 2
            a_in.copy_(A[which])                                # eager work between the replays
            C.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(C, want[which]), (plan.info(), rep)
        del graph
        g.gemm_destroy(plan)
