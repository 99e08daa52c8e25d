"""Parity of the HIP kernels (through the C ABI) against the CPU oracle, element
by element on seeded inputs.  Integer-valued inputs must match bit for bit;
random inputs must satisfy the stated tolerance (E1), the a-priori fp32 error
bound (E2) and the paper's relative criterion (E3); see tests/helpers.py."""
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from helpers import assert_parity, compare, gpu_desc, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2603_12440_amd as g
    g.load_library()          # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available()
    return g


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def cfg_index(g, name):
    return g.config_names().index(name)


def mfma_configs(g):
    """The matrix-core tile configurations that take any K (one tile per workgroup)."""
    return [n for n in g.config_names() if n.startswith(("mfma_", "mfma16_")) and not n.endswith("_p")]


def persistent_configs(g):
    """The persistent-workgroup configurations (K a whole number of 64-column slabs, at least two)."""
    return [n for n in g.config_names() if n.startswith("mfma16_") and n.endswith("_p")]


def skinny_configs(g, m):
    """Every skinny-path configuration (vector-ALU or matrix-core) that takes M = m."""
    out = []
    for i, n in enumerate(g.config_names()):
        if not n.startswith("skinny"):
            continue
        try:
            g.gemm_destroy(g.gemm_create_config(g.GemmDesc(m, 64, 64), i))
            out.append(n)
        except g.GemmError:
            pass
    return out


# ---- exact cases: small integers, every kernel family ---------------------------------

def exact_case(g, o, w, config, out_dtype=None, lo=-1, hi=1, **pads):
    sa, sb = wl.operand_shapes(w)
    A = wl.small_integers(sa, w.seed_a, lo, hi, w.dtype)
    B = wl.small_integers(sb, w.seed_b, lo, hi, w.dtype)
    bias = wl.small_integers((w.N,), w.seed_bias, -3, 3, "f32") if w.has_bias else None
    say(f"exact {w.M}x{w.N}x{w.K} b{w.batch} {w.dtype} {w.epilogue} cfg={config} {pads}")
    C = run_gpu(g, w, A, B, bias, config=cfg_index(g, config) if config else -1,
                out_dtype=out_dtype, **pads)
    ref = run_oracle(o, w, A, B, bias, want=("y",))
    assert np.array_equal(wl.to_float64(C), ref["y"]), config


@pytest.mark.parametrize("shape", [(256, 256, 64), (300, 520, 200), (33, 47, 8), (512, 384, 72),
                                   (257, 255, 136), (64, 1000, 1024)])
def test_mfma_exact_small_integers(g, oracle, shape):
    """Multiple tiles, ragged M and N edges, K tails (K % 64 != 0), all tile shapes."""
    M, N, K = shape
    for cfg in mfma_configs(g):
        w = wl.Workload("t", M, N, K, seed_a=M + 1, seed_b=N + 2)
        exact_case(g, oracle, w, cfg)
        exact_case(g, oracle, w, cfg, out_dtype="f32", lo=-2, hi=2)


def test_mfma_exact_padded_and_fp16(g, oracle):
    for cfg in mfma_configs(g):
        w = wl.Workload("t", 200, 264, 328, seed_a=5, seed_b=6)
        exact_case(g, oracle, w, cfg, pad_a=8, pad_b=16, pad_c=3)
        exact_case(g, oracle, wl.scaled(w, dtype="f16"), cfg, pad_a=16, pad_b=8, pad_c=4)
        exact_case(g, oracle, wl.scaled(w, epilogue="bias_relu", seed_bias=9), cfg, out_dtype="f32", pad_c=5)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 13, 16])
def test_skinny_exact_small_integers(g, oracle, M):
    cfgs = skinny_configs(g, M)
    assert cfgs
    for cfg in cfgs:
        for (N, K) in [(1000, 520), (64, 8), (4099, 1024), (8, 4096), (300, 8200), (130, 16904), (2100, 1032)]:
            w = wl.Workload("t", M, N, K, seed_a=M, seed_b=N)
            exact_case(g, oracle, w, cfg, out_dtype="f32")
        w = wl.Workload("t", M, 515, 136, seed_a=7, seed_b=8)
        exact_case(g, oracle, w, cfg, pad_a=8, pad_b=8, pad_c=1)
        exact_case(g, oracle, wl.scaled(w, dtype="f16", epilogue="bias_relu", seed_bias=3), cfg, out_dtype="f32")


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("la,lb,lc", [("row", "row", "row"), ("row", "col", "row"), ("col", "row", "col"),
                                      ("col", "col", "row"), ("row", "row", "col")])
def test_general_kernel_exact_all_layouts(g, oracle, dtype, la, lb, lc):
    for cfg in ("simt_64x64x16", "simt_32x32x16", "general_mfma32_128x128x16", "general_mfma32_64x64x16"):
        w = wl.Workload("t", 70, 130, 45, dtype=dtype, layout_a=la, layout_b=lb, seed_a=3, seed_b=4)
        exact_case(g, oracle, w, cfg, layout_c=lc, pad_a=1, pad_b=2, pad_c=3)
    # several tiles of the matrix-core general kernel in both directions, ragged edges, K tail
    w = wl.Workload("t", 300, 260, 70, dtype=dtype, layout_a=la, layout_b=lb, epilogue="bias_relu",
                    seed_a=8, seed_b=9, seed_bias=10)
    exact_case(g, oracle, w, "general_mfma32_128x128x16", layout_c=lc, pad_a=3, pad_c=1)
    w = wl.Workload("t", 65, 33, 19, dtype=dtype, layout_a=la, layout_b=lb, batch=3,
                    epilogue="bias", seed_a=5, seed_b=6, seed_bias=7)
    exact_case(g, oracle, w, None, layout_c=lc, out_dtype="f32")


# ---- closed forms on the GPU --------------------------------------------------------------

@pytest.mark.parametrize("K", [128, 256, 4096, 8192, 14336])
def test_all_ones_gives_K(g, K):
    """Every k contributes exactly once (K and all partial sums are exact in fp32,
    and these K are exact in bf16)."""
    for (M, N, cfg) in [(256, 256, "mfma_256x256x64_w2x2_s2"), (256, 256, "mfma16_256x256x64_w2x4"),
                        (130, 70, "mfma_128x128x64_w2x2_s2"), (1, 96, "skinny_m1_w4_g1"),
                        (8, 33, "skinny_m8_w4_g1"),
                        (16, 70, "skinnystage_d3_b256"), (3, 33, "skinnystage_d2_b512"),
                        (16, 70, "skinnydirect_d2_b512_w4"), (3, 33, "skinnydirect_d2_b256_w8"),
                        (2, 33, "skinnydirect_d3_b512_w4"), (11, 64, "skinnydirect_d2_b256_w8")]:
        w = wl.Workload("t", M, N, K)
        say(f"all-ones {M}x{N}x{K} {cfg}")
        A = torch.ones((1, M, K), dtype=torch.bfloat16)
        B = torch.ones((1, N, K), dtype=torch.bfloat16)
        C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg))
        assert torch.all(C.float() == float(K)), cfg


def test_one_hot_k_sweep_copies_columns_of_b(g):
    """A[i, k0] = 1 only: C[i, :] = B[k0, :] exactly.  k0 sweeps slab and MFMA-step
    boundaries, so a dropped, duplicated or shifted k-slab cannot hide."""
    K = 328
    ks = [0, 1, 7, 8, 15, 16, 31, 32, 63, 64, 65, 127, 128, 191, 192, 255, 256, 319, 320, 327]
    for cfg, M, N in [(c, 300, 260) for c in mfma_configs(g)] + [("skinny_m4_w4_g1", 4, 260),
                                                                ("skinny_m8_w4_g1", 7, 70),
                                                                ("skinnystage_d2_b512", 16, 100),
                                                                ("skinnystage_d3_b256", 5, 70),
                                                                ("skinnydirect_d2_b512_w4", 16, 100),
                                                                ("skinnydirect_d2_b256_w8", 5, 70),
                                                                ("skinnydirect_d3_b512_w4", 9, 70),
                                                                ("skinnydirect_d2_b512_w4", 3, 33)]:
        w = wl.Workload("t", M, N, K, seed_b=77)
        say(f"one-hot {cfg}")
        A = wl.one_hot_columns(M, K, ks).unsqueeze(0)
        _, B, _ = wl.make_inputs(w)
        C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg))
        for i in range(M):
            assert torch.equal(C[0, i], B[0, :, ks[i % len(ks)]]), (cfg, i)


def test_identity(g):
    n = 512
    w = wl.Workload("t", n, n, n, seed_a=1, seed_b=2)
    A, B, _ = wl.make_inputs(w)
    eye = torch.eye(n, dtype=torch.bfloat16).unsqueeze(0)
    for cfg in mfma_configs(g):
        say(f"identity {cfg}")
        assert torch.equal(run_gpu(g, w, eye, B, None, config=cfg_index(g, cfg))[0], B[0].T)
        assert torch.equal(run_gpu(g, w, A, eye, None, config=cfg_index(g, cfg))[0], A[0])


def test_bias_only_and_applied_once(g):
    """A = 0: C = round(act(bias[j])) per column; all-ones: K + bias."""
    M, N, K = 260, 300, 64
    bias = wl._draw(("uniform", 3.0), (N,), 5)
    for cfg in ["mfma_256x256x64_w2x2_s2", "simt_64x64x16"]:
        w = wl.Workload("t", M, N, K, epilogue="bias")
        C = run_gpu(g, w, torch.zeros((1, M, K), dtype=torch.bfloat16),
                    torch.ones((1, N, K), dtype=torch.bfloat16), bias, config=cfg_index(g, cfg))
        assert torch.equal(C[0], bias.to(torch.bfloat16).expand(M, N)), cfg
        C = run_gpu(g, w, torch.ones((1, M, K), dtype=torch.bfloat16),
                    torch.ones((1, N, K), dtype=torch.bfloat16), bias, config=cfg_index(g, cfg), out_dtype="f32")
        assert torch.equal(C[0], (bias + float(K)).expand(M, N)), cfg
    w = wl.Workload("t", 3, N, K, epilogue="bias_relu")
    C = run_gpu(g, w, torch.zeros((1, 3, K), dtype=torch.bfloat16),
                torch.ones((1, N, K), dtype=torch.bfloat16), bias, out_dtype="f32")
    assert torch.equal(C[0], bias.clamp(min=0).expand(3, N))


# ---- random data against the oracle -----------------------------------------------------------

RANDOM_CASES = [
    # scaled-down versions of the benchmark workloads (same distributions and layouts)
    ("square_8192", dict(M=512, N=768, K=1024)),
    ("llm_4096x14336x4096", dict(M=384, N=896, K=512)),
    ("llm_4096x4096x14336", dict(M=256, N=256, K=3584)),
    ("llm_4096x6144x4096", dict(M=300, N=200, K=520)),
    ("gelu_8192x16384x4096", dict(M=512, N=1024, K=512)),
    ("gelu_8192x16384x4096", dict(M=250, N=1030, K=264)),
    ("batched_64x512x512x128", dict(batch=5)),
]


@pytest.mark.parametrize("name,changes", RANDOM_CASES)
def test_mfma_random_against_oracle(g, oracle, name, changes):
    w = wl.scaled(wl.WORKLOADS[name], **changes)
    A, B, bias = wl.make_inputs(w)
    ref = run_oracle(oracle, w, A, B, bias)
    for cfg in [None] + mfma_configs(g):
        say(f"random {name} {changes} cfg={cfg}")
        C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg) if cfg else -1)
        r = assert_parity(w, C, ref, A, B, bias)
        say("   ", r)


@pytest.mark.parametrize("epilogue", ["none", "bias", "bias_relu", "bias_gelu_erf", "bias_gelu_tanh", "relu", "gelu_erf",
                                      "bias_swish_scale", "bias_sigmoid_scale_residual", "swish_scale",
                                      "sigmoid_scale_residual"])
def test_every_epilogue_on_every_kernel_family(g, oracle, epilogue):
    for (M, N, K, cfg) in [(260, 264, 136, "mfma_256x256x64_w2x2_s2"), (130, 140, 72, "mfma_128x128x64_w2x2_s2"),
                           (3, 515, 264, "skinny_m4_w4_g1"), (8, 100, 1032, "skinny_m8_w4_g1"),
                           (16, 100, 1032, "skinnystage_d3_b256"), (7, 70, 264, "skinnystage_d2_b512"),
                           (16, 100, 1032, "skinnydirect_d2_b512_w4"), (7, 70, 264, "skinnydirect_d2_b256_w8"),
                           (3, 70, 3128, "skinnydirect_d3_b512_w4"), (11, 40, 5192, "skinnydirect_d2_b512_w4"),
                           (70, 90, 50, "simt_64x64x16"), (150, 140, 50, "general_mfma32_128x128x16")]:
        # pre-activations of order 1 so that the activations' curved parts are exercised
        w = wl.Workload("t", M, N, K, dist_a=("normal", 1.0), dist_b=("normal", 1.5 / np.sqrt(K)),
                        epilogue=epilogue, dist_bias=("uniform", 1.0), seed_a=11, seed_b=12, seed_bias=13,
                        scale=-1.75 if "residual" in epilogue else 2.5)
        A, B, bias = wl.make_inputs(w)
        ref = run_oracle(oracle, w, A, B, bias)
        for od in (None, "f32"):
            say(f"epilogue {epilogue} {cfg} out={od}")
            C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg), out_dtype=od)
            assert_parity(w, C, ref, A, B, bias, out_dtype=od)


def test_scaled_epilogues_closed_form_and_tails(g, oracle):
    """A = one-hot (k = 0), B row 0 = chosen pre-activations t_j (exact in bf16): C[i, j] is the
    scalar formula of t_j.  The t_j include 0, +-ln 3 rounded to bf16, and the far tails where
    exp overflows in fp32 (sigma -> 0 or 1), for every kernel family, fp32 output."""
    ts = torch.tensor([0.0, 1.09375, -1.09375, 0.5, -0.5, 8.0, -8.0, 30.0, -30.0, 100.0, -100.0, 200.0,
                       -200.0, 3.0, -3.0, 0.0078125], dtype=torch.float32)
    for (M, cfg) in [(40, "mfma_128x128x64_w2x2_s2"), (300, "mfma_256x256x64_w2x4_s2"), (3, "skinny_m4_w4_g1"),
                     (16, "skinnystage_d2_b512"), (9, "skinnydirect_d2_b512_w4"), (33, "simt_32x32x16")]:
        N, K = 16 * 5, 72
        for epilogue, c in [("swish_scale", 3.0), ("sigmoid_scale_residual", -0.5)]:
            w = wl.Workload("t", M, N, K, epilogue=epilogue, scale=c)
            A = wl.one_hot_columns(M, K, [0]).unsqueeze(0)
            B = torch.zeros((1, N, K), dtype=torch.bfloat16)
            B[0, :, 0] = ts.repeat(5).to(torch.bfloat16)
            say(f"scaled epilogue closed form {epilogue} {cfg}")
            C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg), out_dtype="f32")
            t = ts.repeat(5).double().numpy()
            from scipy.special import expit            # library sigmoid, accurate in both tails
            sig = expit(t)
            want = c * t * sig if epilogue == "swish_scale" else c * sig + t
            got = C[0].double().numpy()
            assert np.isfinite(got).all(), cfg
            # fp32 evaluation: a few units of 2^-24 relative (the exponent's argument carries
            # |t| * 2^-24); tails underflow to exactly 0
            bad = np.abs(got[0] - want) > 8e-6 * np.abs(want) + 1e-30
            assert not bad.any(), (cfg, epilogue, t[bad], got[0][bad], want[bad])
            # rows of a one-hot A are identical
            assert np.array_equal(got, np.tile(got[0], (M, 1)))
            ref = run_oracle(oracle, w, A, B, None)
            assert_parity(w, C, ref, A, B, None, out_dtype="f32")


@pytest.mark.parametrize("M", [1, 4, 16])
def test_skinny_random_against_oracle(g, oracle, M):
    for N, K in [(1024, 8192), (3000, 1032)]:
        w = wl.scaled(wl.WORKLOADS[f"skinny_m{M}_n8192"], N=N, K=K)
        A, B, bias = wl.make_inputs(w)
        ref = run_oracle(oracle, w, A, B, bias)
        say(f"skinny random M={M} N={N} K={K}")
        C, info = run_gpu(g, w, A, B, bias, return_plan_info=True)
        assert "kernel=skinny" in info
        assert_parity(w, C, ref, A, B, bias)
        # the matrix-core path must agree with it on the same data
        C2 = run_gpu(g, w, A, B, bias, config=cfg_index(g, "mfma_128x128x64_w2x2_s2"))
        assert_parity(w, C2, ref, A, B, bias)


@pytest.mark.parametrize("la,lb,lc", [("row", "row", "row"), ("row", "col", "row"), ("col", "row", "col"),
                                      ("col", "col", "row")])
@pytest.mark.parametrize("cfg", ["f32mfma_128x128x32", "f32mfma_64x64x32"])
def test_f32_vector_kernel_exact_all_layouts(g, oracle, la, lb, lc, cfg):
    """The fp32 kernel that moves float4 groups: several tiles in both directions, ragged edges, a K
    tail (K % 32 != 0), padded leading dimensions, a batch, every combination of operand layouts;
    operands displaced by one element run the general kernel on the same grid instead."""
    w = wl.Workload("t", 300, 260, 72, dtype="f32", layout_a=la, layout_b=lb, epilogue="bias_relu",
                    seed_a=8, seed_b=9, seed_bias=10)
    exact_case(g, oracle, w, cfg, layout_c=lc, pad_a=4, pad_b=8, pad_c=3)
    exact_case(g, oracle, w, cfg, layout_c=lc, offset_a=1)
    exact_case(g, oracle, w, cfg, layout_c=lc, offset_b=3)
    w = wl.Workload("t", 68, 36, 20, dtype="f32", layout_a=la, layout_b=lb, batch=3, seed_a=5, seed_b=6)
    exact_case(g, oracle, w, cfg, layout_c=lc)
    w = wl.Workload("t", 128, 256, 160, dtype="f32", layout_a=la, layout_b=lb, seed_a=1, seed_b=2)
    exact_case(g, oracle, w, cfg, layout_c=lc, lo=-40, hi=40)
    # extents that cannot be cut into float4 groups: the configuration does not apply
    w = wl.Workload("t", 70, 130, 45, dtype="f32", layout_a=la, layout_b=lb)
    with pytest.raises(g.GemmError):
        g.gemm_create_config(gpu_desc(g, w), cfg_index(g, cfg))


@pytest.mark.parametrize("la,lb,lc", [("row", "row", "row"), ("row", "col", "row"), ("col", "row", "col"),
                                      ("col", "col", "row"), ("row", "row", "col")])
def test_f32_small_kernel_exact_all_layouts(g, oracle, la, lb, lc):
    """The fp32 kernel for small problems (16x16 tiles, K split over the four waves): ragged edges,
    K below, at and above one round of 256 columns and not a multiple of 4 (element loads), float4
    loads with padded leading dimensions, displaced operands, a batch with bias and activation."""
    cfg = "f32small_16x16x256"
    for (M, N, K) in [(70, 130, 45), (33, 47, 256), (16, 16, 4), (50, 20, 1500), (100, 36, 772)]:
        w = wl.Workload("t", M, N, K, dtype="f32", layout_a=la, layout_b=lb, seed_a=M, seed_b=N)
        exact_case(g, oracle, w, cfg, layout_c=lc)
    w = wl.Workload("t", 72, 40, 520, dtype="f32", layout_a=la, layout_b=lb, batch=3, epilogue="bias_relu",
                    seed_a=8, seed_b=9, seed_bias=10)
    exact_case(g, oracle, w, cfg, layout_c=lc, pad_a=4, pad_b=8, pad_c=3)
    exact_case(g, oracle, w, cfg, layout_c=lc, pad_a=1, pad_b=2)
    exact_case(g, oracle, w, cfg, layout_c=lc, offset_a=1, offset_b=2)


def test_fp32_config_full_size(g, oracle):
    """The 256^3 fp32 case at full size: true fp32 arithmetic (tolerance 1e-6 forbids
    any narrowing of the operands)."""
    w = wl.WORKLOADS["f32_256"]
    A, B, _ = wl.make_inputs(w)
    ref = run_oracle(oracle, w, A, B, None)
    for cfg in (None, "simt_64x64x16", "simt_32x32x16", "general_mfma32_128x128x16", "general_mfma32_64x64x16",
                "f32mfma_128x128x32", "f32mfma_64x64x32", "f32small_16x16x256"):
        say(f"f32_256 cfg={cfg}")
        C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg) if cfg else -1)
        r = assert_parity(w, C, ref, A, B, None)
        assert r["e1"] < 1e-7
    # transpose invariance on the GPU: C^T = B^T A^T through swapped operands and layouts
    wt = wl.scaled(w, layout_a="col", layout_b="col")
    Ct = run_gpu(g, wt, B, A, None)     # B (K x N row-major) read as B^T column-major; same for A
    ref_t = {k: v.transpose(0, 2, 1) for k, v in ref.items()}
    assert_parity(wt, Ct, ref_t, A, B, None)


def test_fp16_random(g, oracle):
    w = wl.Workload("t", 300, 260, 520, dtype="f16", dist_a=("uniform", 1.0),
                    dist_b=("uniform", 1.0 / np.sqrt(520)), seed_a=21, seed_b=22)
    A, B, _ = wl.make_inputs(w)
    ref = run_oracle(oracle, w, A, B, None)
    for cfg in [None] + mfma_configs(g) + ["simt_64x64x16"]:
        say(f"fp16 cfg={cfg}")
        C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg) if cfg else -1)
        assert_parity(w, C, ref, A, B, None)


def test_batches_and_bias_strides(g, oracle):
    """Each batch reads its own slab; shared bias (stride 0) against one per batch."""
    for cfg in ("mfma_128x128x64_w2x2_s2", "simt_64x64x16", "skinny_m4_w4_g1", "skinnydirect_d2_b512_w4", "skinnydirect_d2_b256_w8",
                "skinnystage_d3_b256"):
        M = 4 if cfg.startswith("skinny") else 96
        w = wl.Workload("t", M, 136, 72, batch=4, epilogue="bias_gelu_erf", seed_a=31, seed_b=32)
        A, B, _ = wl.make_inputs(w)
        bias = wl._draw(("uniform", 1.0), (4 * 136,), 33)
        for sb in (0, 136):
            say(f"batched {cfg} stride_bias={sb}")
            C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg), stride_bias=sb)
            ref = run_oracle(oracle, w, A, B, bias, stride_bias=sb)
            assert_parity(w, C, ref, A, B, bias)
    # a bias stride that is not a multiple of 4 floats: the bias vectors of batches 1..3 start at addresses
    # that are only 4-byte aligned (the matrix-core epilogues read the bias in 16-byte pieces where they can)
    for cfg in ("mfma16_256x256x64_w2x4", "mfma16_128x128x64_w2x2", "mfma16_256x256x64_w2x4_p", "mfma16_128x128x64_w2x2_p",
                "mfma_128x128x64_w2x2_s2", "mfma_256x256x64_w2x4_s2"):
        w = wl.Workload("t", 300, 264, 128, batch=4, epilogue="bias_relu", seed_a=41, seed_b=42)
        A, B, _ = wl.make_inputs(w)
        bias = wl._draw(("uniform", 1.0), (3 * 265 + 264,), 43)
        say(f"batched {cfg} stride_bias=265")
        for od in (None, "f32"):
            C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg), stride_bias=265, out_dtype=od)
            ref = run_oracle(oracle, w, A, B, bias, stride_bias=265)
            assert_parity(w, C, ref, A, B, bias, out_dtype=od)
    # constant per batch: C_b = K (b+1)^2
    w = wl.Workload("t", 64, 64, 64, batch=3)
    A = torch.stack([torch.full((64, 64), float(b + 1)) for b in range(3)]).to(torch.bfloat16)
    C = run_gpu(g, w, A, A.clone(), None, out_dtype="f32")
    for b in range(3):
        assert torch.all(C[b] == 64.0 * (b + 1) ** 2)


def test_misaligned_pointer_is_refused(g):
    w = wl.Workload("t", 64, 64, 64)
    dev = torch.device("cuda:0")
    buf = torch.zeros(64 * 64 + 8, dtype=torch.bfloat16, device=dev)
    C = torch.zeros(64 * 64, dtype=torch.bfloat16, device=dev)
    plan = g.gemm_create(gpu_desc(g, w))
    with pytest.raises(g.GemmError) as e:
        g.gemm_run(plan, buf[1:], buf, C)          # 2-byte aligned A on the 16-byte path
    assert e.value.status == -5
    g.gemm_run(plan, buf, buf, C)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)


def test_tuner_times_every_applicable_configuration(g, oracle):
    """Parameter tuning (Sec. 3.4 of the paper): every instantiation that can run the problem
    is timed, the reported best one is among them, and a plan made from it is correct."""
    w = wl.scaled(wl.WORKLOADS["gelu_8192x16384x4096"], M=300, N=520, K=264)
    A, B, bias = wl.make_inputs(w)
    dev = torch.device("cuda:0")
    Ad, Bd, bd = A.to(dev), B.to(dev), bias.to(dev)
    Cd = torch.empty((1, w.M, w.N), dtype=torch.bfloat16, device=dev)
    desc = gpu_desc(g, w)
    say("tune", w)
    best, times = g.gemm_tune(desc, Ad, Bd, Cd, bd, min_seconds=0.005)
    names = g.config_names()
    assert names[best] in times and times[names[best]] == min(times.values())
    assert all(t > 0 for t in times.values())
    # M = 300: no skinny, no fp8; K = 264 is not a whole number of slabs: no persistent workgroups
    assert {n for n in names if n.startswith(("mfma_", "mfma16_", "simt", "general_")) and not n.endswith("_p")} == set(times)
    plan = g.gemm_create_config(desc, best)
    g.gemm_run(plan, Ad, Bd, Cd, bd)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    ref = run_oracle(oracle, w, A, B, bias)
    assert_parity(w, Cd.cpu(), ref, A, B, bias)


# ---- full benchmark sizes, sampled ------------------------------------------------------------

@pytest.mark.parametrize("name", sorted(wl.WORKLOADS))
def test_full_size_workloads_on_sampled_outputs(g, oracle, name):
    """Every benchmark workload at its full size, with the plan bench.py times (built-in
    choice): sampled outputs (tile-lattice corners + random positions) against the oracle's
    point evaluation, to the E1 tolerance and the E2 bound."""
    from helpers import oracle_problem, e2_bound, E1_TOL
    w = wl.WORKLOADS[name]
    A, B, bias = wl.make_inputs(w)
    say(f"full size {name}")
    C, info = run_gpu(g, w, A, B, bias, return_plan_info=True)
    say("   ", info)
    pb, pi, pj = wl.sample_points(w, 3000, 1234)
    ref = oracle.ref_gemm_points(oracle_problem(oracle, w), wl.storage_numpy(A), wl.storage_numpy(B),
                                 None if bias is None else bias.numpy(), pb, pi, pj, want=("y", "t", "s"))
    got = wl.to_float64(C)[pb, pi, pj]
    err = np.abs(got - ref["y"])
    scale = w.K * float(A.float().abs().max()) * float(B.float().abs().max()) + \
        (float(bias.abs().max()) if bias is not None else 0.0)
    assert np.isfinite(got).all()
    assert err.max() / scale <= E1_TOL[w.dtype]
    assert np.all(err <= e2_bound(w, ref)), float((err / e2_bound(w, ref)).max())
    # properties that hold at any size: nothing left unwritten (the sentinel would show), and the
    # paper's relative criterion on the sampled entries
    eps = 1e-3 * float(np.sqrt(np.mean(ref["y"] ** 2))) + 1e-30
    assert np.mean(err / (np.abs(ref["y"]) + eps) < 0.01) >= 0.99
    # whole 256 x 256 tiles, every element: the first and the last tile, tiles whose ids fall into
    # different classes of the XCD renumbering, and the tiles on both sides of a two-launch seam
    if w.M >= 256 and w.N >= 256:
        import re
        tm, tn = (w.M + 255) // 256, (w.N + 255) // 256
        tiles = {(0, 0), (tm - 1, tn - 1), (tm // 2, tn // 3), (min(9, tm - 1), min(5, tn - 1)), (tm - 1, 0)}
        seam = re.search(r"columns=(\d+)\.\.$", info.strip()) or re.search(r"columns=(\d+)\.\.\s", info)
        if seam:
            c = int(seam.group(1)) // 256
            tiles |= {(tm // 2, c - 1), (tm // 2, c), (0, c)}
        for (ti, tj) in sorted(tiles):
            i0, j0 = ti * 256, tj * 256
            ii, jj = np.meshgrid(np.arange(i0, min(i0 + 256, w.M)), np.arange(j0, min(j0 + 256, w.N)), indexing="ij")
            pi2, pj2 = ii.reshape(-1).astype(np.int64), jj.reshape(-1).astype(np.int64)
            pb2 = np.full(pi2.size, (ti + tj) % w.batch, dtype=np.int64)
            ref2 = oracle.ref_gemm_points(oracle_problem(oracle, w), wl.storage_numpy(A), wl.storage_numpy(B),
                                          None if bias is None else bias.numpy(), pb2, pi2, pj2, want=("y", "t", "s"))
            err2 = np.abs(wl.to_float64(C)[pb2, pi2, pj2] - ref2["y"])
            assert np.all(err2 <= e2_bound(w, ref2)), (ti, tj, float((err2 / e2_bound(w, ref2)).max()))
        say(f"    whole tiles {sorted(tiles)}: ok")


def test_split_plan_two_launches(g, oracle):
    """Shapes whose 256x256 tiles do not fill whole rounds of the CUs are planned as two
    launches (big tiles for the full rounds, another shape for the remaining columns): the
    seam must be invisible.  Integer data: bit exact; bias + ReLU across the seam."""
    w = wl.Workload("t", 4096, 4608, 1024, epilogue="bias_relu", seed_a=3, seed_b=4, seed_bias=5)
    sa, sb = wl.operand_shapes(w)
    A = wl.small_integers(sa, 3, -1, 1)
    B = wl.small_integers(sb, 4, -1, 1)
    bias = wl.small_integers((w.N,), 5, -3, 3, "f32")
    C, info = run_gpu(g, w, A, B, bias, return_plan_info=True, pad_c=8, out_dtype="f32")
    say(info)
    assert " + kernel=" in info
    ref = run_oracle(oracle, w, A, B, bias, want=("y",))
    assert np.array_equal(wl.to_float64(C), ref["y"])


def test_fp32_output_of_every_mfma_tile(g, oracle):
    """fp32 C leaves the matrix-core kernels through an LDS transpose in passes (whole-line
    stores) when its rows are 16-byte aligned, otherwise straight from the accumulator layout:
    both routes, ragged edges, padded rows, batches, bias + activation, every tile shape."""
    for cfg in mfma_configs(g):
        for (M, N, K, batch, pad_c) in [(300, 520, 136, 1, 0), (300, 520, 136, 1, 4), (257, 522, 72, 1, 0),
                                        (130, 260, 64, 3, 0), (64, 100, 64, 1, 1)]:
            w = wl.Workload("t", M, N, K, batch=batch, epilogue="bias_relu", seed_a=11, seed_b=12, seed_bias=13)
            exact_case(g, oracle, w, cfg, out_dtype="f32", pad_c=pad_c)
    for cfg in F8_CONFIGS:
        w = wl.Workload("t", 300, 520, 256, dtype="f8", epilogue="bias_relu", seed_a=11, seed_b=12, seed_bias=13)
        exact_case(g, oracle, w, cfg, out_dtype="f32")
        exact_case(g, oracle, w, cfg, out_dtype="f32", pad_c=1)


def test_tuning_mode_times_once_per_problem_and_keeps_results_exact(g, oracle):
    """Tuning mode (the paper's parameter optimisation as a switch): the first run of a problem
    times the alternatives on the caller's buffers and remembers the winner; results stay bit
    exact on integer data before, during and after; plans with an explicit configuration and a
    second plan of the same problem do no timing of their own."""
    dev = torch.device("cuda:0")
    from helpers import gpu_desc
    w = wl.Workload("t", 300, 520, 264, epilogue="bias_relu", seed_a=3, seed_b=4, seed_bias=5)
    sa, sb = wl.operand_shapes(w)
    A = wl.small_integers(sa, 3, -1, 1).to(dev)
    B = wl.small_integers(sb, 4, -1, 1).to(dev)
    bias = wl.small_integers((w.N,), 5, -3, 3, "f32").to(dev)
    ref = run_oracle(oracle, w, A.cpu(), B.cpu(), bias.cpu(), want=("y",))["y"]
    def run(plan):
        C = torch.full((1, w.M, w.N), -768.0, dtype=wl.TORCH_DTYPE[w.dtype], device=dev)
        g.gemm_run(plan, A, B, C, bias)
        torch.cuda.synchronize()
        return wl.to_float64(C.cpu())
    g.gemm_autotune_clear()
    before = g.gemm_set_autotune(True)
    try:
        assert g.gemm_autotune_entries() == 0
        fixed = g.gemm_create_config(gpu_desc(g, w), cfg_index(g, "mfma_128x128x64_w2x2_s2"))
        assert np.array_equal(run(fixed), ref) and g.gemm_autotune_entries() == 0      # explicit configuration: untouched
        p1 = g.gemm_create(gpu_desc(g, w))
        say("before: " + p1.info())
        assert np.array_equal(run(p1), ref)                                            # timed here
        assert g.gemm_autotune_entries() == 1
        say("after:  " + p1.info())
        assert np.array_equal(run(p1), ref)
        p2 = g.gemm_create(gpu_desc(g, w))                                             # same problem: table hit
        assert np.array_equal(run(p2), ref) and g.gemm_autotune_entries() == 1
        assert p2.info() == p1.info()
        w2 = wl.Workload("t", 4, 520, 264, seed_a=3, seed_b=4)                         # another problem (skinny kernels)
        A2 = wl.small_integers(wl.operand_shapes(w2)[0], 3, -1, 1).to(dev)
        ref2 = run_oracle(oracle, w2, A2.cpu(), B.cpu(), None, want=("y",))["y"]
        p3 = g.gemm_create(gpu_desc(g, w2))
        C2 = torch.empty((1, w2.M, w2.N), dtype=wl.TORCH_DTYPE[w2.dtype], device=dev)
        g.gemm_run(p3, A2, B, C2, None)
        torch.cuda.synchronize()
        assert np.array_equal(wl.to_float64(C2.cpu()), ref2) and g.gemm_autotune_entries() == 2
        for p in (fixed, p1, p2, p3):
            g.gemm_destroy(p)
    finally:
        g.gemm_set_autotune(before)
        g.gemm_autotune_clear()
    # off again: a new plan of the same problem runs as built
    p4 = g.gemm_create(gpu_desc(g, w))
    assert np.array_equal(run(p4), ref) and g.gemm_autotune_entries() == 0 and "(tuned)" not in p4.info()
    g.gemm_destroy(p4)


# ---- split-K ------------------------------------------------------------------------------------

def run_splitk(g, w, A, B, bias, splits, out_dtype=None, layout_c="row", pad_c=0, ws_slack=0):
    dev = torch.device("cuda:0")
    from helpers import gpu_desc
    c_major, c_minor = (w.M, w.N) if layout_c == "row" else (w.N, w.M)
    ldc = c_minor + pad_c
    odt = wl.TORCH_DTYPE[out_dtype or w.out_dtype or w.dtype]
    Cd = torch.full((1, c_major, ldc), -777.0, dtype=odt, device=dev)
    plan = g.gemm_create_splitk(gpu_desc(g, w, out_dtype, layout_c, ldc=ldc), splits)
    info = plan.info()
    n = g.gemm_workspace_bytes(plan)
    ws = torch.full((n // 4 + ws_slack,), float("nan"), dtype=torch.float32, device=dev)
    g.gemm_run_workspace(plan, A.to(dev), B.to(dev), Cd, None if bias is None else bias.to(dev), ws, n)
    torch.cuda.synchronize()
    g.gemm_destroy(plan)
    if ws_slack:
        assert torch.isnan(ws[n // 4:]).all(), "wrote past the stated workspace size"
    Ch = Cd.cpu()
    if pad_c:
        assert torch.all(Ch[:, :, c_minor:] == -777.0)
    Ch = Ch[:, :, :c_minor]
    return (Ch.transpose(1, 2) if layout_c == "col" else Ch).contiguous(), info


def test_splitk_exact_and_against_oracle(g, oracle):
    """Integer data: a split product is bit exact whatever the number of slices (also 1, and
    slices that end inside a slab); random data with every epilogue family against the oracle."""
    w = wl.Workload("t", 200, 136, 1536, epilogue="bias_relu", seed_a=3, seed_b=4, seed_bias=5)
    sa, sb = wl.operand_shapes(w)
    A = wl.small_integers(sa, 3, -1, 1)
    B = wl.small_integers(sb, 4, -1, 1)
    bias = wl.small_integers((w.N,), 5, -3, 3, "f32")
    want = torch.relu(A[0].double() @ B[0].double().T + bias.double())
    for splits in (1, 2, 3, 8, 24, 0):        # 1536 / 24 = 64: one slab per slice; 1536 / 3 = 512
        say(f"split-K exact splits={splits}")
        C, info = run_splitk(g, w, A, B, bias, splits, out_dtype="f32", pad_c=4, ws_slack=64)
        say("   ", info)
        assert torch.equal(C[0].double(), want), splits
    # slices of 40 columns (less than a slab, K tail path in every slice)
    w2 = wl.Workload("t", 70, 50, 320, seed_a=6, seed_b=7)
    sa, sb = wl.operand_shapes(w2)
    A2, B2 = wl.small_integers(sa, 6, -2, 2), wl.small_integers(sb, 7, -2, 2)
    C, info = run_splitk(g, w2, A2, B2, None, 8, out_dtype="f32")
    assert torch.equal(C[0].double(), A2[0].double() @ B2[0].double().T)
    for epilogue, od, lc in [("none", None, "row"), ("bias_gelu_erf", None, "row"), ("bias_swish_scale", "f32", "col"),
                             ("relu", None, "col")]:
        w3 = wl.Workload("t", 300, 264, 4096, dist_b=("normal", 1.5 / 64), epilogue=epilogue, scale=1.5,
                         dist_bias=("uniform", 1.0), seed_a=21, seed_b=22, seed_bias=23)
        A3, B3, bias3 = wl.make_inputs(w3)
        ref = run_oracle(oracle, w3, A3, B3, bias3)
        for splits in (4, 16):
            say(f"split-K {epilogue} out={od} C {lc}-major splits={splits}")
            C, info = run_splitk(g, w3, A3, B3, bias3, splits, out_dtype=od, layout_c=lc, pad_c=8)
            assert_parity(w3, C, ref, A3, B3, bias3, out_dtype=od)
    # fp16
    w4 = wl.Workload("t", 128, 128, 2048, dtype="f16", dist_b=("normal", 1.0 / 45), seed_a=31, seed_b=32)
    A4, B4, _ = wl.make_inputs(w4)
    C, info = run_splitk(g, w4, A4, B4, None, 8)
    assert_parity(w4, C, run_oracle(oracle, w4, A4, B4, None), A4, B4, None)


def test_splitk_full_size_against_plain_plan_and_oracle_samples(g, oracle):
    """The split-K benchmark shape at full size: sampled outputs against the oracle, and the
    whole result against the single-launch plan (both within the E2 bound of the same oracle
    values, so they may differ by rounding only)."""
    from helpers import oracle_problem, e2_bound
    w = wl.WORKLOADS["smallmn_512x512x32768"]
    A, B, bias = wl.make_inputs(w)
    C, info = run_splitk(g, w, A, B, None, 0)
    say("   ", info)
    assert "splitk_16" in info
    pb, pi, pj = wl.sample_points(w, 2000, 77)
    ref = oracle.ref_gemm_points(oracle_problem(oracle, w), wl.storage_numpy(A), wl.storage_numpy(B), None,
                                 pb, pi, pj, want=("y", "t", "s"))
    err = np.abs(wl.to_float64(C)[pb, pi, pj] - ref["y"])
    assert np.all(err <= e2_bound(w, ref)), float((err / e2_bound(w, ref)).max())
    C1 = run_gpu(g, w, A, B, None)
    d = (C.double() - C1.double()).abs().max().item()
    assert d <= 2.0 ** -7 * C1.double().abs().max().item()


# ---- fp8 (E4M3) operands ----------------------------------------------------------------------

F8_CONFIGS = ["mfma8_256x256x128_w2x4_s2", "mfma8_128x128x128_w2x2_s2", "mfma8_256x192x128_w4x2_s2"]


def test_f8_exact_integers_ragged_shapes_and_k_tails(g, oracle):
    """Integers in [-4, 4] are exact in E4M3 and so is everything computed from them: bit-exact
    results for ragged M and N, K below one slab, K with a tail of 1..7 sixteen-byte pieces, padded
    rows, fp32 and bf16 output, bias + ReLU."""
    for cfg in F8_CONFIGS:
        for (M, N, K) in [(300, 260, 16), (70, 90, 112), (257, 129, 128), (130, 70, 144), (256, 256, 400),
                          (33, 500, 1040)]:
            w = wl.Workload("t", M, N, K, dtype="f8", out_dtype="f32", epilogue="bias_relu")
            sa, sb = wl.operand_shapes(w)
            A = wl.small_integers(sa, 3, -4, 4, "f8")
            B = wl.small_integers(sb, 4, -4, 4, "f8")
            bias = wl.small_integers((N,), 5, -3, 3, "f32")
            want = torch.relu(A[0].double() @ B[0].double().T + bias.double())
            say(f"f8 exact {cfg} {M}x{N}x{K}")
            C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg), pad_a=16, pad_b=32, pad_c=4)
            assert torch.equal(C[0].double(), want), (cfg, M, N, K)
    # all ones: every k counted once (8192 is exact in bf16)
    for cfg in F8_CONFIGS:
        for K in (128, 256, 8192):
            w = wl.Workload("t", 130, 70, K, dtype="f8", out_dtype="bf16")
            ones_a = torch.ones((1, 130, K)).to(torch.float8_e4m3fn)
            ones_b = torch.ones((1, 70, K)).to(torch.float8_e4m3fn)
            C = run_gpu(g, w, ones_a, ones_b, None, config=cfg_index(g, cfg))
            assert torch.all(C.float() == float(K)), (cfg, K)


def test_f8_one_hot_k_sweep(g):
    """A[i, k0] = 1 only: C[i, :] = B[:, k0] exactly, k0 over the chunk, MFMA-step and slab seams."""
    K = 400
    ks = [0, 1, 15, 16, 31, 32, 33, 47, 48, 63, 64, 65, 95, 96, 127, 128, 129, 191, 192, 255, 256, 319, 383, 384, 399]
    for cfg in F8_CONFIGS:
        M, N = 300, 140
        w = wl.Workload("t", M, N, K, dtype="f8", out_dtype="f32", seed_b=77)
        A = wl.one_hot_columns(M, K, ks, "f8").unsqueeze(0)
        B = wl.small_integers((1, N, K), 9, -4, 4, "f8")
        say(f"f8 one-hot {cfg}")
        C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg))
        for i in range(M):
            assert torch.equal(C[0, i].double(), B[0, :, ks[i % len(ks)]].double()), (cfg, i)


@pytest.mark.parametrize("epilogue", ["none", "bias_gelu_erf", "bias_swish_scale"])
def test_f8_random_against_oracle(g, oracle, epilogue):
    for cfg, (M, N, K) in [(F8_CONFIGS[0], (300, 520, 1168)), (F8_CONFIGS[1], (130, 140, 272)), (None, (64, 200, 4096))]:
        w = wl.Workload("t", M, N, K, dtype="f8", out_dtype="bf16", dist_a=("normal", 1.0),
                        dist_b=("normal", 1.5 / np.sqrt(K)), epilogue=epilogue, scale=2.0,
                        dist_bias=("uniform", 1.0), seed_a=41, seed_b=42, seed_bias=43)
        A, B, bias = wl.make_inputs(w)
        ref = run_oracle(oracle, w, A, B, bias)
        for od in ("bf16", "f32"):
            say(f"f8 random {epilogue} cfg={cfg} {M}x{N}x{K} out={od}")
            C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg) if cfg else -1, out_dtype=od)
            r = assert_parity(w, C, ref, A.float(), B.float(), bias, out_dtype=od)
            say("   ", r)


def test_f8_batches_and_splitk(g, oracle):
    w = wl.Workload("t", 96, 136, 256, dtype="f8", out_dtype="bf16", batch=3, seed_a=51, seed_b=52)
    A, B, _ = wl.make_inputs(w)
    C = run_gpu(g, w, A, B, None)
    assert_parity(w, C, run_oracle(oracle, w, A, B, None), A.float(), B.float(), None)
    w2 = wl.Workload("t", 200, 136, 4096, dtype="f8", out_dtype="bf16", dist_b=("normal", 1.0 / 64), seed_a=53, seed_b=54)
    A2, B2, _ = wl.make_inputs(w2)
    ref = run_oracle(oracle, w2, A2, B2, None)
    for splits in (4, 0):
        C2, info = run_splitk(g, w2, A2, B2, None, splits)
        say("   ", info)
        assert "mfma8" in info
        assert_parity(w2, C2, ref, A2.float(), B2.float(), None)


def test_k_tail_every_length_on_every_mfma_tile(g):
    """K tails of every length (1 .. all k-steps of a slab), alone and after one full slab, on
    every matrix-core tile shape, integer data, fp32 output: bit exact.  (A tail that fills all
    k-steps ends with MFMAs right before the epilogue reads the accumulators.)"""
    for cfg in mfma_configs(g) + F8_CONFIGS:
        f8 = cfg.startswith("mfma8")
        dt, piece, slab = ("f8", 16, 128) if f8 else ("bf16", 8, 64)
        for K in [p for p in range(piece, slab, piece)] + [slab + p for p in range(piece, slab, piece)]:
            w = wl.Workload("t", 130, 132, K, dtype=dt, out_dtype="f32")
            sa, sb = wl.operand_shapes(w)
            A = wl.small_integers(sa, 3, -3, 3, dt)
            B = wl.small_integers(sb, 4, -3, 3, dt)
            C = run_gpu(g, w, A, B, None, config=cfg_index(g, cfg))
            assert torch.equal(C[0].double(), A[0].double() @ B[0].double().T), (cfg, K)
        say(f"k tails {cfg}: ok")


# ---- persistent workgroups -------------------------------------------------------------------

def test_persistent_workgroups_exact(g, oracle):
    """A persistent workgroup walks over several tiles as one stream of slabs: one, two and three
    tiles per workgroup with a remainder, even and odd slab counts (the LDS stage a tile starts in
    alternates), ragged edges, both output types, bias + activation, padded C rows, batches.
    Integer data: bit exact against the oracle."""
    for cfg in persistent_configs(g):
        tile = 128 if "128x128" in cfg else 256
        per_round = 512 if tile == 128 else 256            # workgroups the chip holds at once
        for (tiles_m, tiles_n, K, batch) in [(2, 3, 128, 1), (17, 17, 192, 1), (24, 23, 128, 1), (3, 2, 320, 3),
                                             (33, 20, 128, 1),
                                             # a workgroup's tiles belong to different problems of the batch
                                             (4, 4, 128, 40 if tile == 128 else 20), (2, 2, 192, 150 if tile == 128 else 70),
                                             (3, 1, 128, 200 if tile == 128 else 100)]:
            if tile == 256 and tiles_m * tiles_n > 300:
                continue                                    # (keeps the oracle's share of the test short)
            M, N = tiles_m * tile - 5, tiles_n * tile - 12
            w = wl.Workload("t", M, N, K, batch=batch, epilogue="bias_relu", seed_a=31, seed_b=32, seed_bias=33)
            say(f"persistent {cfg} {M}x{N}x{K} b{batch}: {tiles_m * tiles_n} tiles on {per_round} workgroups")
            exact_case(g, oracle, w, cfg, lo=-2, hi=2)
            exact_case(g, oracle, wl.scaled(w, epilogue="none"), cfg, out_dtype="f32", pad_c=4)
            if batch > 1 and tiles_m == 4:
                # C rows that are not 16-byte aligned: the launcher runs one tile per workgroup instead,
                # with the plan's batch renumbering switched off
                exact_case(g, oracle, w, cfg, lo=-2, hi=2, pad_c=3)


def test_persistent_workgroups_random_and_misaligned_c(g, oracle):
    """Random data against the oracle on the persistent configurations (several tiles per workgroup,
    GELU epilogue), and a C whose rows are not 16-byte aligned: the plan must still be right (it
    falls back to one tile per workgroup)."""
    for cfg in persistent_configs(g):
        tile = 128 if "128x128" in cfg else 256
        n = 23 if tile == 128 else 17
        w = wl.scaled(wl.WORKLOADS["gelu_8192x16384x4096"], M=n * tile - 3, N=n * tile, K=192)
        A, B, bias = wl.make_inputs(w)
        ref = run_oracle(oracle, w, A, B, bias)
        say(f"persistent random {cfg} {w.M}x{w.N}x{w.K}")
        C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg))
        say("   ", assert_parity(w, C, ref, A, B, bias))
        C = run_gpu(g, w, A, B, bias, config=cfg_index(g, cfg), pad_c=3)     # ldc not a multiple of 8
        assert_parity(w, C, ref, A, B, bias)
