"""The seeded input recipe: determinism, storage shapes, value distributions."""
import numpy as np
import torch

import workloads as wl


def test_catalogue_matches_the_stated_configs():
    names = set(wl.WORKLOADS)
    assert {"f32_256", "square_8192", "llm_4096x14336x4096", "llm_4096x4096x14336",
            "llm_4096x6144x4096", "gelu_8192x16384x4096", "batched_64x512x512x128"} <= names
    for m in (1, 4, 16):
        for n in (8192, 28672):
            w = wl.WORKLOADS[f"skinny_m{m}_n{n}"]
            assert (w.M, w.N, w.K, w.bound) == (m, n, 8192, "hbm")
    sq = wl.WORKLOADS["square_8192"]
    assert sq.flops == 2 * 8192 ** 3 and sq.bytes == 3 * 8192 * 8192 * 2


def test_generation_is_deterministic_and_in_storage_order():
    w = wl.scaled(wl.WORKLOADS["gelu_8192x16384x4096"], M=48, N=80, K=64)
    A1, B1, b1 = wl.make_inputs(w)
    A2, B2, b2 = wl.make_inputs(w)
    assert A1.dtype == torch.bfloat16 and A1.shape == (1, 48, 64)
    assert B1.shape == (1, 80, 64)                    # column-major K x N = N rows of K
    assert b1.dtype == torch.float32 and b1.shape == (80,)
    assert torch.equal(A1, A2) and torch.equal(B1, B2) and torch.equal(b1, b2)
    assert not torch.equal(A1[0, :, :48], B1[0, :48, :48])
    f = wl.WORKLOADS["f32_256"]
    A, B, bias = wl.make_inputs(f)
    assert A.dtype == torch.float32 and B.shape == (1, 256, 256) and bias is None
    assert A.abs().max() <= 1.0 and abs(float(A.mean())) < 0.02


def test_distributions():
    w = wl.scaled(wl.WORKLOADS["llm_4096x6144x4096"], M=256, N=512, K=1024)
    A, B, _ = wl.make_inputs(w)
    assert abs(float(A.float().std()) - 1.0) < 0.02
    assert abs(float(B.float().std()) - 0.02) < 0.001
    g = wl.scaled(wl.WORKLOADS["gelu_8192x16384x4096"], M=64, N=4096, K=64)
    _, _, bias = wl.make_inputs(g)
    assert bias.abs().max() <= 0.1 and bias.abs().max() > 0.09


def test_storage_numpy_views_bits():
    t = torch.tensor([1.0, -2.0, 0.5], dtype=torch.bfloat16)
    assert wl.storage_numpy(t).tolist() == [0x3F80, 0xC000, 0x3F00]
    t = torch.tensor([1.0, -2.0], dtype=torch.float16)
    assert wl.storage_numpy(t).tolist() == [0x3C00, 0xC000]
    pb, pi, pj = wl.sample_points(wl.WORKLOADS["square_8192"], 100, 5)
    assert pi.max() < 8192 and pj.max() < 8192 and pb.max() == 0 and pi.size == pj.size
