"""Pins for the CPU oracle: everything here is fixed by mathematics or by a
library routine, never by the oracle itself (and never by the GPU path).

Each test names the mistake it is meant to catch.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads as wl

ALL_LAYOUTS = [(la, lb) for la in ("row", "col") for lb in ("row", "col")]


def _code(o, layout):
    return o.ROW_MAJOR if layout == "row" else o.COL_MAJOR


def _dt(o, name):
    return {"f32": o.DTYPE_F32, "bf16": o.DTYPE_BF16, "f16": o.DTYPE_F16}[name]


def _store(logical: np.ndarray, layout: str, ld_pad: int = 0, poison=np.nan):
    """Logical 2-D fp32 matrix -> (flat fp32 storage, ld) in the given layout,
    optionally with ld_pad poisoned padding elements per major index."""
    m = logical if layout == "row" else logical.T
    major, minor = m.shape
    ld = minor + ld_pad
    buf = np.full((major, ld), poison, dtype=np.float32)
    buf[:, :minor] = m
    return buf.reshape(-1), ld


def _as_dtype(flat_f32: np.ndarray, dtype: str):
    t = torch.from_numpy(flat_f32.copy()).to(wl.TORCH_DTYPE[dtype])
    return wl.storage_numpy(t)


# ---- index / loop structure ---------------------------------------------------

def test_hand_worked_2x3x2(oracle):
    """A product small enough to do by hand; catches transposed operands,
    swapped M/N and a reduction over the wrong index."""
    A = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)          # 2 x 3
    B = np.array([[7, 8], [9, 10], [11, 12]], dtype=np.float32)     # 3 x 2
    want = np.array([[58, 64], [139, 154]], dtype=np.float64)
    for la, lb in ALL_LAYOUTS:
        a, lda = _store(A, la)
        b, ldb = _store(B, lb)
        p = oracle.Problem(2, 2, 3, oracle.DTYPE_F32, oracle.DTYPE_F32,
                           _code(oracle, la), _code(oracle, lb), lda, ldb)
        y = oracle.ref_gemm(p, a, b)["y"][0]
        assert np.array_equal(y, want), (la, lb)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("la,lb", ALL_LAYOUTS)
def test_brute_force_rational_4x4x4(oracle, dtype, la, lb):
    """Python-loop product in exact rational arithmetic on small integers:
    bit-exact agreement required in every dtype and layout."""
    A = wl.small_integers((4, 4), 11, dtype="f32").numpy()
    B = wl.small_integers((4, 4), 12, dtype="f32").numpy()
    a, lda = _store(A, la)
    b, ldb = _store(B, lb)
    p = oracle.Problem(4, 4, 4, _dt(oracle, dtype), _dt(oracle, dtype),
                       _code(oracle, la), _code(oracle, lb), lda, ldb)
    y = oracle.ref_gemm(p, _as_dtype(a, dtype), _as_dtype(b, dtype))["y"][0]
    for i in range(4):
        for j in range(4):
            exact = sum(Fraction(float(A[i, k])) * Fraction(float(B[k, j])) for k in range(4))
            assert Fraction(float(y[i, j])) == exact


@pytest.mark.parametrize("la,lb", ALL_LAYOUTS)
def test_rectangular_against_integer_matmul(oracle, la, lb):
    """M != N != K with padded leading dimensions whose padding holds NaN:
    catches swapped extents, a wrong leading dimension and reads of padding."""
    M, N, K = 5, 7, 9
    A = wl.small_integers((M, K), 21, dtype="f32").numpy()
    B = wl.small_integers((K, N), 22, dtype="f32").numpy()
    a, lda = _store(A, la, ld_pad=3)
    b, ldb = _store(B, lb, ld_pad=2)
    p = oracle.Problem(M, N, K, oracle.DTYPE_F32, oracle.DTYPE_F32,
                       _code(oracle, la), _code(oracle, lb), lda, ldb)
    out = oracle.ref_gemm(p, a, b, want=("y", "s"))
    want = A.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(out["y"][0], want.astype(np.float64))
    want_s = np.abs(A).astype(np.int64) @ np.abs(B).astype(np.int64)
    assert np.array_equal(out["s"][0], want_s.astype(np.float64))


def test_fp64_accumulation_against_rationals(oracle):
    """bf16 operands with full mantissas: the oracle must be within K ulps(fp64)
    of the exactly rounded rational result; an fp32 accumulator would miss by
    ~2^-24 relative and fail."""
    w = wl.Workload("t", 8, 8, 8, dist_a=("normal", 1.0), dist_b=("normal", 1.0),
                    seed_a=31, seed_b=32)
    A, B, _ = wl.make_inputs(w)
    p = oracle.Problem(8, 8, 8)
    out = oracle.ref_gemm(p, wl.storage_numpy(A), wl.storage_numpy(B), want=("y", "s"))
    Af, Bf = wl.to_float64(A)[0], wl.to_float64(B)[0]      # A: M x K ; B stored N x K
    for i in range(8):
        for j in range(8):
            exact = sum(Fraction(Af[i, k]) * Fraction(Bf[j, k]) for k in range(8))
            err = abs(Fraction(float(out["y"][0, i, j])) - exact)
            assert err <= Fraction(8 * 2.0 ** -53) * Fraction(float(out["s"][0, i, j]))
            exact_s = sum(abs(Fraction(Af[i, k]) * Fraction(Bf[j, k])) for k in range(8))
            assert abs(Fraction(float(out["s"][0, i, j])) - exact_s) <= Fraction(8 * 2.0 ** -53) * exact_s


# ---- closed forms ---------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_identity_and_permutation(oracle, dtype):
    """A = I gives C = B; a permutation matrix permutes rows; exact in every dtype."""
    n = 16
    w = wl.Workload("t", n, n, n, dtype=dtype, seed_a=41, seed_b=42)
    _, B, _ = wl.make_inputs(w)                                # stored N x K (col-major B)
    Blog = wl.to_float64(B)[0].T                               # logical K x N
    eye = torch.eye(n).to(wl.TORCH_DTYPE[dtype])
    p = oracle.Problem(n, n, n, _dt(oracle, dtype), _dt(oracle, dtype))
    y = oracle.ref_gemm(p, wl.storage_numpy(eye), wl.storage_numpy(B))["y"][0]
    assert np.array_equal(y, Blog)
    perm = np.random.Generator(np.random.Philox(key=43)).permutation(n)
    P = torch.zeros(n, n)
    P[torch.arange(n), torch.from_numpy(perm)] = 1.0           # row i picks row perm[i] of B
    y = oracle.ref_gemm(p, wl.storage_numpy(P.to(wl.TORCH_DTYPE[dtype])),
                        wl.storage_numpy(B))["y"][0]
    assert np.array_equal(y, Blog[perm, :])
    # B = I gives C = A
    A, _, _ = wl.make_inputs(w)
    y = oracle.ref_gemm(p, wl.storage_numpy(A), wl.storage_numpy(eye))["y"][0]
    assert np.array_equal(y, wl.to_float64(A)[0])


@pytest.mark.parametrize("K", [1, 128, 256, 4096, 8192, 14336])
def test_all_ones_gives_K(oracle, K):
    """Every k contributes exactly once."""
    M, N = 3, 5
    ones_a = np.full(M * K, 0x3F80, dtype=np.uint16)           # bf16 1.0
    ones_b = np.full(N * K, 0x3F80, dtype=np.uint16)
    y = oracle.ref_gemm(oracle.Problem(M, N, K), ones_a, ones_b)["y"][0]
    assert np.array_equal(y, np.full((M, N), float(K)))


def test_one_hot_selects_row_of_b(oracle):
    """A with a single 1 per row at k0 copies row k0 of B: catches a dropped,
    duplicated or shifted k."""
    M, N, K = 6, 10, 37
    ks = [0, 1, 17, 35, 36, 20]
    A = wl.one_hot_columns(M, K, ks)
    w = wl.Workload("t", M, N, K, seed_b=52)
    _, B, _ = wl.make_inputs(w)
    y = oracle.ref_gemm(oracle.Problem(M, N, K), wl.storage_numpy(A), wl.storage_numpy(B))["y"][0]
    Bl = wl.to_float64(B)[0]                                    # N x K
    for i in range(M):
        assert np.array_equal(y[i], Bl[:, ks[i]])


def test_rank_one(oracle):
    """K = 1: C[i,j] = a_i * b_j exactly."""
    M, N = 9, 11
    w = wl.Workload("t", M, N, 1, seed_a=61, seed_b=62)
    A, B, _ = wl.make_inputs(w)
    y = oracle.ref_gemm(oracle.Problem(M, N, 1), wl.storage_numpy(A), wl.storage_numpy(B))["y"][0]
    a = wl.to_float64(A)[0, :, 0]
    b = wl.to_float64(B)[0, :, 0]
    assert np.array_equal(y, np.outer(a, b))


def test_transpose_invariance_bit_exact(oracle):
    """C^T = B^T A^T with the same k order: identical to the last bit."""
    M, N, K = 13, 17, 29
    w = wl.Workload("t", M, N, K, seed_a=71, seed_b=72)
    A, B, _ = wl.make_inputs(w)                                 # A: M x K row-major ; B: N x K (col-major K x N)
    a, b = wl.storage_numpy(A), wl.storage_numpy(B)
    y = oracle.ref_gemm(oracle.Problem(M, N, K), a, b)["y"][0]
    # B^T is N x K row-major = the same buffer; A^T is K x M column-major = the same buffer.
    yt = oracle.ref_gemm(oracle.Problem(N, M, K), b, a)["y"][0]
    assert np.array_equal(yt, y.T)


def test_random_against_numpy_fp64(oracle):
    """Random bf16 data against numpy's fp64 matmul (a library routine with a
    different summation order): agreement to a few ulps of S."""
    M, N, K = 33, 65, 300
    w = wl.Workload("t", M, N, K, seed_a=81, seed_b=82)
    A, B, _ = wl.make_inputs(w)
    out = oracle.ref_gemm(oracle.Problem(M, N, K), wl.storage_numpy(A), wl.storage_numpy(B),
                          want=("y", "s"))
    want = wl.to_float64(A)[0] @ wl.to_float64(B)[0].T
    assert np.all(np.abs(out["y"][0] - want) <= 2 * K * 2.0 ** -53 * out["s"][0])


# ---- epilogue ---------------------------------------------------------------------

def test_gelu_point_values(oracle):
    """GELU_erf(x) = x * Phi(x) with Phi from the normal table; the tanh form
    differs visibly at x = 1."""
    table = {1.0: 0.8413447460685429, -1.0: -0.15865525393145707,
             2.0: 1.9544997361036416, 0.5: 0.34573123063700656, 0.0: 0.0}
    for x, want in table.items():
        assert abs(oracle.activation(oracle.EPI_GELU_ERF, x) - want) < 1e-15
        assert abs(oracle.activation(oracle.EPI_BIAS_GELU_ERF, x) - want) < 1e-15
    assert abs(oracle.activation(oracle.EPI_BIAS_GELU_TANH, 1.0) - 0.84119199) < 1e-7
    from scipy.stats import norm
    for x in np.linspace(-6, 6, 97):
        assert abs(oracle.activation(oracle.EPI_GELU_ERF, x) - x * norm.cdf(x)) < 1e-14
        for e in (oracle.EPI_GELU_ERF, oracle.EPI_BIAS_GELU_TANH):
            # odd-part identity holds for both forms
            assert abs(oracle.activation(e, x) - oracle.activation(e, -x) - x) < 1e-14
        u = math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)
        assert abs(oracle.activation(oracle.EPI_BIAS_GELU_TANH, x) - 0.5 * x * (1 + math.tanh(u))) < 1e-14


def test_relu_and_identity(oracle):
    for e in (oracle.EPI_RELU, oracle.EPI_BIAS_RELU):
        assert oracle.activation(e, -3.5) == 0.0
        assert oracle.activation(e, 2.25) == 2.25
    for e in (oracle.EPI_NONE, oracle.EPI_BIAS):
        assert oracle.activation(e, -3.5) == -3.5


def test_sigmoid_point_values_and_identities(oracle):
    """sigma(ln 3) = 3/4, sigma(-ln 3) = 1/4, sigma(0) = 1/2; sigma(t) + sigma(-t) = 1;
    sigma(t) = (1 + tanh(t/2)) / 2 (library tanh); tails do not overflow."""
    assert abs(oracle.sigmoid(math.log(3.0)) - 0.75) < 1e-16
    assert abs(oracle.sigmoid(-math.log(3.0)) - 0.25) < 1e-16
    assert oracle.sigmoid(0.0) == 0.5
    for t in np.linspace(-30, 30, 121):
        assert abs(oracle.sigmoid(t) + oracle.sigmoid(-t) - 1.0) < 1e-15
        assert abs(oracle.sigmoid(t) - 0.5 * (1.0 + math.tanh(0.5 * t))) < 1e-15
    assert oracle.sigmoid(800.0) == 1.0 and oracle.sigmoid(-800.0) == 0.0
    assert abs(oracle.sigmoid(-50.0) / math.exp(-50.0) - 1.0) < 1e-15


def test_swish_scale_and_sigmoid_scale_residual(oracle):
    """swish_scale(t) = c t sigma(t); sigmoid_scale_residual(t) = c sigma(t) + t.
    Worked values at t = +-ln 3 and 0, the odd / even part identities
    (swish(t) - swish(-t) = c t; ssr(t) + ssr(-t) = c), linearity in c, and the
    large-|t| limits.  A scale applied before the sigmoid, a missing residual or a
    residual that is scaled too would fail one of these."""
    ln3 = math.log(3.0)
    for sw, sr in ((oracle.EPI_SWISH_SCALE, oracle.EPI_SIGMOID_SCALE_RESIDUAL),
                   (oracle.EPI_BIAS_SWISH_SCALE, oracle.EPI_BIAS_SIGMOID_SCALE_RESIDUAL)):
        assert abs(oracle.epilogue(sw, ln3, 2.0) - 1.5 * ln3) < 1e-15
        assert abs(oracle.epilogue(sw, -ln3, 2.0) + 0.5 * ln3) < 1e-15
        assert oracle.epilogue(sw, 0.0, 7.0) == 0.0
        assert abs(oracle.epilogue(sr, ln3, 2.0) - (1.5 + ln3)) < 1e-15
        assert abs(oracle.epilogue(sr, -ln3, 2.0) - (0.5 - ln3)) < 1e-15
        assert oracle.epilogue(sr, 0.0, 7.0) == 3.5
        for t in np.linspace(-12, 12, 49):
            for c in (0.5, 1.0, -3.0):
                assert abs(oracle.epilogue(sw, t, c) - oracle.epilogue(sw, -t, c) - c * t) < 1e-13
                assert abs(oracle.epilogue(sr, t, c) + oracle.epilogue(sr, -t, c) - c) < 1e-13
                assert abs(oracle.epilogue(sw, t, c) - c * oracle.epilogue(sw, t, 1.0)) < 1e-13
                assert abs(oracle.epilogue(sr, t, c) - t - c * (oracle.epilogue(sr, t, 1.0) - t)) < 1e-13
            # scale 0 kills swish and leaves the residual alone
            assert oracle.epilogue(sw, t, 0.0) == 0.0 and oracle.epilogue(sr, t, 0.0) == t
        assert abs(oracle.epilogue(sw, 40.0, 1.5) - 60.0) < 1e-12
        assert abs(oracle.epilogue(sw, -40.0, 1.5)) < 1e-15
        assert abs(oracle.epilogue(sr, 40.0, 1.5) - 41.5) < 1e-12
        assert abs(oracle.epilogue(sr, -40.0, 1.5) + 40.0) < 1e-12
    # the older epilogues ignore the scale
    assert oracle.epilogue(oracle.EPI_RELU, 2.25, 9.0) == 2.25
    assert oracle.epilogue(oracle.EPI_BIAS, -1.5, 9.0) == -1.5


def test_scaled_epilogues_inside_the_product(oracle):
    """Through ref_gemm: all-ones operands give t = K + bias[j]; the output is the scalar
    formula of t, with the problem's scale, for every element."""
    M, N, K = 3, 5, 4
    bias = np.array([-6, -4.5, -4, -3, 0], dtype=np.float32)       # t = -2, -0.5, 0, 1, 4
    ones_a = np.full(M * K, 0x3F80, dtype=np.uint16)
    ones_b = np.full(N * K, 0x3F80, dtype=np.uint16)
    t = K + bias.astype(np.float64)
    sig = 0.5 * (1.0 + np.tanh(0.5 * t))
    p = oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS_SWISH_SCALE, scale=2.5)
    out = oracle.ref_gemm(p, ones_a, ones_b, bias, want=("y", "t"))
    assert np.array_equal(out["t"][0], np.tile(t, (M, 1)))
    assert np.allclose(out["y"][0], np.tile(2.5 * t * sig, (M, 1)), rtol=0, atol=1e-15)
    p = oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS_SIGMOID_SCALE_RESIDUAL, scale=-0.75)
    y = oracle.ref_gemm(p, ones_a, ones_b, bias)["y"][0]
    assert np.allclose(y, np.tile(-0.75 * sig + t, (M, 1)), rtol=0, atol=1e-15)
    p = oracle.Problem(M, N, K, epilogue=oracle.EPI_SWISH_SCALE, scale=2.0)
    y = oracle.ref_gemm(p, ones_a, ones_b)["y"][0]
    assert np.allclose(y, 2.0 * K * 0.5 * (1.0 + math.tanh(0.5 * K)), rtol=0, atol=1e-15)
    pts = oracle.ref_gemm_points(oracle.Problem(M, N, K, epilogue=oracle.EPI_SIGMOID_SCALE_RESIDUAL, scale=3.0),
                                 ones_a, ones_b, None, [0, 0], [0, 2], [1, 4])["y"]
    assert np.allclose(pts, 3.0 * 0.5 * (1.0 + math.tanh(0.5 * K)) + K, rtol=0, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.ref_gemm(oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS_SWISH_SCALE), ones_a, ones_b, None)
    with pytest.raises(ValueError):
        oracle.ref_gemm(oracle.Problem(M, N, K, epilogue=oracle.EPI_SWISH_SCALE), ones_a, ones_b, bias)


def test_bias_is_per_column_added_once_before_activation(oracle):
    """A = 0 -> C[i,j] = act(bias[j]); all-ones -> K + bias[j].  Catches a
    per-row bias, a bias added after the activation or twice."""
    M, N, K = 4, 6, 8
    bias = np.array([-3, -1, 0.5, 1, 2, 4], dtype=np.float32)
    zeros = np.zeros(M * K, dtype=np.uint16)
    ones = np.full(N * K, 0x3F80, dtype=np.uint16)
    p = oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS_RELU)
    y = oracle.ref_gemm(p, zeros, ones, bias)["y"][0]
    assert np.array_equal(y, np.tile(np.maximum(bias, 0).astype(np.float64), (M, 1)))
    p = oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS)
    y = oracle.ref_gemm(p, np.full(M * K, 0x3F80, dtype=np.uint16), ones, bias)["y"][0]
    assert np.array_equal(y, np.tile(K + bias.astype(np.float64), (M, 1)))
    p = oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS_GELU_ERF)
    out = oracle.ref_gemm(p, np.full(M * K, 0xBF80, dtype=np.uint16), ones, bias, want=("y", "t"))
    assert np.array_equal(out["t"][0], np.tile(-K + bias.astype(np.float64), (M, 1)))
    from scipy.stats import norm
    assert np.allclose(out["y"][0], out["t"][0] * norm.cdf(out["t"][0]), rtol=0, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.ref_gemm(oracle.Problem(M, N, K, epilogue=oracle.EPI_BIAS), zeros, ones, None)
    with pytest.raises(ValueError):
        oracle.ref_gemm(oracle.Problem(M, N, K), zeros, ones, bias)


# ---- batches ------------------------------------------------------------------------

def test_batches_use_their_own_slab(oracle):
    """Batch b filled with the constant b+1: C_b = K (b+1)^2; a shared bias
    (stride 0) against one bias per batch."""
    Bt, M, N, K = 3, 2, 4, 5
    A = np.concatenate([np.full(M * K, float(b + 1), dtype=np.float32) for b in range(Bt)])
    B = np.concatenate([np.full(N * K, float(b + 1), dtype=np.float32) for b in range(Bt)])
    p = oracle.Problem(M, N, K, oracle.DTYPE_F32, oracle.DTYPE_F32, batch=Bt)
    y = oracle.ref_gemm(p, A, B)["y"]
    for b in range(Bt):
        assert np.array_equal(y[b], np.full((M, N), K * (b + 1.0) ** 2))
    bias = np.arange(Bt * N, dtype=np.float32)
    p = oracle.Problem(M, N, K, oracle.DTYPE_F32, oracle.DTYPE_F32, batch=Bt,
                       epilogue=oracle.EPI_BIAS, stride_bias=N)
    y = oracle.ref_gemm(p, A, B, bias)["y"]
    for b in range(Bt):
        assert np.array_equal(y[b], K * (b + 1.0) ** 2 + np.tile(bias[b * N:(b + 1) * N], (M, 1)))
    p = oracle.Problem(M, N, K, oracle.DTYPE_F32, oracle.DTYPE_F32, batch=Bt,
                       epilogue=oracle.EPI_BIAS, stride_bias=0)
    y = oracle.ref_gemm(p, A, B, bias[:N])["y"]
    for b in range(Bt):
        assert np.array_equal(y[b], K * (b + 1.0) ** 2 + np.tile(bias[:N], (M, 1)))
    # non-packed batch strides, gap poisoned
    gap = 7
    A2 = np.full(Bt * (M * K + gap), np.nan, dtype=np.float32)
    for b in range(Bt):
        A2[b * (M * K + gap): b * (M * K + gap) + M * K] = b + 1.0
    p = oracle.Problem(M, N, K, oracle.DTYPE_F32, oracle.DTYPE_F32, batch=Bt, stride_a=M * K + gap)
    y = oracle.ref_gemm(p, A2, B)["y"]
    for b in range(Bt):
        assert np.array_equal(y[b], np.full((M, N), K * (b + 1.0) ** 2))


def test_points_agree_with_full(oracle):
    w = wl.Workload("t", 19, 23, 31, epilogue="bias_gelu_erf", batch=2, seed_a=91, seed_b=92, seed_bias=93)
    A, B, bias = wl.make_inputs(w)
    p = oracle.Problem(w.M, w.N, w.K, epilogue=oracle.EPI_BIAS_GELU_ERF, batch=2)
    full = oracle.ref_gemm(p, wl.storage_numpy(A), wl.storage_numpy(B), bias.numpy(), want=("y", "t", "s"))
    pb, pi, pj = wl.sample_points(w, 50, 94, tile=8)
    pts = oracle.ref_gemm_points(p, wl.storage_numpy(A), wl.storage_numpy(B), bias.numpy(),
                                 pb, pi, pj, want=("y", "t", "s"))
    for k in ("y", "t", "s"):
        assert np.array_equal(pts[k], full[k][pb, pi, pj])
    with pytest.raises(ValueError):
        oracle.ref_gemm_points(p, wl.storage_numpy(A), wl.storage_numpy(B), bias.numpy(),
                               [0], [w.M], [0])


# ---- storage formats ------------------------------------------------------------------

def test_bf16_decode_exhaustive(oracle):
    """All 65 536 bf16 patterns against the definition (upper half of binary32)."""
    bits = np.arange(65536, dtype=np.uint32)
    want = (bits << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    for b in range(65536):
        got = oracle.bf16_bits_to_double(int(b))
        assert (math.isnan(got) and math.isnan(want[b])) or got == want[b]


def test_f16_decode_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    for b in range(65536):
        got = oracle.f16_bits_to_double(b)
        assert (math.isnan(got) and math.isnan(want[b])) or got == want[b]


def test_f8e4m3_decode_exhaustive_and_products(oracle):
    """All 256 codes of OCP E4M3: the format's defining values by hand (1 = 0x38, largest 448 = 0x7E,
    smallest subnormal 2^-9 = 0x01, smallest normal 2^-6 = 0x08, NaN only at S.1111.111, no
    infinity), monotone in the code for each sign, and equal to the library's decoding; then a
    small product with fp8 operands against exact integer arithmetic."""
    val = [oracle.f8e4m3_bits_to_double(c) for c in range(256)]
    assert val[0x00] == 0.0 and val[0x80] == 0.0 and math.copysign(1.0, val[0x80]) == -1.0
    assert val[0x38] == 1.0 and val[0xB8] == -1.0 and val[0x40] == 2.0 and val[0x3C] == 1.5
    assert val[0x7E] == 448.0 and val[0x78] == 256.0 and val[0x77] == 240.0
    assert val[0x01] == 2.0 ** -9 and val[0x07] == 7 * 2.0 ** -9 and val[0x08] == 2.0 ** -6
    assert math.isnan(val[0x7F]) and math.isnan(val[0xFF])
    assert all(math.isfinite(v) for c, v in enumerate(val) if c & 0x7F != 0x7F)
    pos = val[0:0x7F]
    assert all(a < b for a, b in zip(pos, pos[1:]))
    assert all(val[c | 0x80] == -val[c] for c in range(0x7F))
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.nan_to_num(lib, nan=1e9), np.nan_to_num(np.array(val), nan=1e9))
    # 3 x 4 x 5 product of small integers stored as fp8, column-major B (K contiguous)
    rng = np.random.default_rng(3)
    A = rng.integers(-4, 5, (3, 5)); B = rng.integers(-4, 5, (4, 5))
    a8 = torch.from_numpy(A.astype(np.float32)).to(torch.float8_e4m3fn)
    b8 = torch.from_numpy(B.astype(np.float32)).to(torch.float8_e4m3fn)
    p = oracle.Problem(3, 4, 5, oracle.DTYPE_F8E4M3, oracle.DTYPE_F8E4M3)
    y = oracle.ref_gemm(p, wl.storage_numpy(a8), wl.storage_numpy(b8))["y"][0]
    assert np.array_equal(y, (A @ B.T).astype(np.float64))


def test_bf16_round_to_nearest_even(oracle):
    """Ties: 1 + 2^-8 -> 1.0 ; 1 + 3*2^-8 -> 1 + 2^-6 ; round trip of every
    finite pattern; agreement with the library cast used by the generators."""
    assert oracle.f32_to_bf16_rne(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.bf16_bits_to_double(oracle.f32_to_bf16_rne(1.0 + 3 * 2.0 ** -8)) == 1.0 + 2.0 ** -6
    assert oracle.f32_to_bf16_rne(1.0 + 2.0 ** -8 + 2.0 ** -20) == 0x3F81
    assert oracle.f32_to_bf16_rne(3.4e38) == 0x7F80          # overflow -> +inf
    for b in range(0, 65536, 3):
        v = oracle.bf16_bits_to_double(b)
        if not math.isnan(v):
            assert oracle.f32_to_bf16_rne(v) == b
    x = wl._draw(("normal", 1.0), (4096,), 101)
    lib = wl.storage_numpy(x.to(torch.bfloat16))
    mine = np.array([oracle.f32_to_bf16_rne(float(v)) for v in x.numpy()], dtype=np.uint16)
    assert np.array_equal(lib, mine)


def test_f16_round_to_nearest_even(oracle):
    assert oracle.f32_to_f16_rne(1.0 + 2.0 ** -11) == 0x3C00   # tie -> even
    assert oracle.f32_to_f16_rne(1.0 + 3 * 2.0 ** -11) == 0x3C02
    assert oracle.f32_to_f16_rne(65519.0) == 0x7BFF
    assert oracle.f32_to_f16_rne(65520.0) == 0x7C00
    assert oracle.f32_to_f16_rne(2.0 ** -25) == 0x0000         # tie at half the smallest subnormal
    assert oracle.f32_to_f16_rne(3 * 2.0 ** -25) == 0x0002
    x = np.concatenate([wl._draw(("normal", s), (2048,), 102 + i).numpy()
                        for i, s in enumerate((1.0, 1e-4, 1e-7, 3e4))])
    lib = x.astype(np.float16).view(np.uint16)
    mine = np.array([oracle.f32_to_f16_rne(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(lib, mine)
