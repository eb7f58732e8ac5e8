"""Pins for the CPU oracle: each test checks it against something other than itself --
exact rational brute force, numpy's fp64 matmul, the decomposition identity of the paper's
Section 3.2 / Algorithm 1, the adjoint identity, closed-form GELU values and structured
inputs with known answers.  Shapes are non-square so that a transposed operand, a swapped
index or a wrong reduce axis fails."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import axo_synth as syn
import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _frac(bits):
    f = syn.bf16_bits_to_f64(np.asarray(bits, dtype=np.uint16).reshape(1, -1))[0]
    return [Fraction(float(v)) for v in f]


def _rand(shape, seed, stream, sigma=1.0):
    return syn.normal_bf16(seed, stream, shape, sigma)


# ---- P1: exact brute force in rational arithmetic ---------------------------------------
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 5, 7), (17, 8, 24), (2, 9, 4)])
def test_brute_force_exact_rational(M, K, N):
    X, W, dY = _rand((M, K), 11, 0), _rand((K, N), 11, 1, 0.02), _rand((M, N), 11, 2)
    Xq = [_frac(X[i]) for i in range(M)]
    Wq = [_frac(W[i]) for i in range(K)]
    Gq = [_frac(dY[i]) for i in range(M)]
    Y, dX, dW = oracle.fc_fwd(X, W), oracle.fc_dgrad(dY, W), oracle.fc_wgrad(X, dY)
    assert Y.shape == (M, N) and dX.shape == (M, K) and dW.shape == (K, N)
    for t in range(M):
        for n in range(N):
            ex = sum(Xq[t][k] * Wq[k][n] for k in range(K))
            assert abs(Fraction(Y[t, n]) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 200)
    for t in range(M):
        for k in range(K):
            ex = sum(Gq[t][n] * Wq[k][n] for n in range(N))
            assert abs(Fraction(dX[t, k]) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 200)
    for k in range(K):
        for n in range(N):
            ex = sum(Xq[t][k] * Gq[t][n] for t in range(M))
            assert abs(Fraction(dW[k, n]) - ex) <= abs(ex) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 200)


# ---- P2: numpy fp64 matmul on config 1 ---------------------------------------------------
def test_numpy_matmul_cfg1():
    L = syn.configs()["cfg1"][0]
    d = syn.layer_inputs(L)
    Xf, Wf, Gf = (syn.bf16_bits_to_f64(d[k]) for k in ("X", "W", "dY"))
    for got, ref in ((oracle.fc_fwd(d["X"], d["W"]), Xf @ Wf),
                     (oracle.fc_dgrad(d["dY"], d["W"]), Gf @ Wf.T),
                     (oracle.fc_wgrad(d["X"], d["dY"]), Xf.T @ Gf)):
        assert np.linalg.norm(got - ref) <= 1e-12 * np.linalg.norm(ref)


def test_row_subset_equals_full_rows():
    X, W, dY = _rand((37, 24), 3, 0), _rand((24, 40), 3, 1, 0.02), _rand((37, 40), 3, 2)
    rows = [36, 0, 5, 5, 19]
    assert np.array_equal(oracle.fc_fwd(X, W, rows=rows), oracle.fc_fwd(X, W)[rows])
    assert np.array_equal(oracle.fc_dgrad(dY, W, rows=rows), oracle.fc_dgrad(dY, W)[rows])
    krows = [23, 1, 7]
    assert np.array_equal(oracle.fc_wgrad(X, dY, rows=krows), oracle.fc_wgrad(X, dY)[krows])
    assert oracle.fc_fwd(X, W, rows=[]).shape == (0, 40)


def test_leading_dimension_views():
    big = _rand((50, 64), 5, 0)
    Wb = _rand((64, 48), 5, 1, 0.02)
    Xv, Wv = big[7:30, 8:40], Wb[8:40, 16:40]  # strided views, ld > row length
    ref = syn.bf16_bits_to_f64(np.ascontiguousarray(Xv)) @ syn.bf16_bits_to_f64(np.ascontiguousarray(Wv))
    assert np.allclose(oracle.fc_fwd(Xv, Wv), ref, rtol=1e-13, atol=0)


# ---- P3: decomposition identity (Section 3.2, Algorithm 1) -----------------------------
def test_decomposition_identity_cfg1_grid222():
    L = syn.configs()["cfg1_grid222"][0]
    g = syn.global_inputs(L)
    Y, dX, dW = oracle.assemble_from_shards(g["X"], g["W"], g["dY"], L.grid)
    for got, ref in ((Y, oracle.fc_fwd(g["X"], g["W"])), (dX, oracle.fc_dgrad(g["dY"], g["W"])),
                     (dW, oracle.fc_wgrad(g["X"], g["dY"]))):
        assert np.linalg.norm(got - ref) <= 1e-12 * np.linalg.norm(ref)


@pytest.mark.parametrize("grid", [(2, 1, 4), (1, 3, 2), (4, 2, 1), (3, 2, 2)])
@pytest.mark.parametrize("transposed", [False, True])
def test_decomposition_identity_asymmetric_grids(grid, transposed):
    T, K, N = 24, 36, 48  # divisible by 1..4 and pairwise different
    Xg, Wg, dYg = _rand((T, K), 7, 0), _rand((K, N), 7, 1, 0.02), _rand((T, N), 7, 2)
    Xf, Wf, Gf = (syn.bf16_bits_to_f64(a) for a in (Xg, Wg, dYg))
    Y, dX, dW = oracle.assemble_from_shards(Xg, Wg, dYg, grid, transposed)
    assert np.allclose(Y, Xf @ Wf, rtol=1e-12, atol=1e-15)
    assert np.allclose(dX, Gf @ Wf.T, rtol=1e-12, atol=1e-15)
    assert np.allclose(dW, Xf.T @ Gf, rtol=1e-12, atol=1e-15)


def test_shard_shapes_follow_axes():
    # K over Gx, N over Gy, T over Gz; transposed swaps the roles of X and Y
    rt, rk, rn = oracle.shard_slices(24, 36, 48, (2, 3, 4), (1, 2, 3))
    assert (rt, rk, rn) == (slice(18, 24), slice(18, 36), slice(32, 48))
    rt, rk, rn = oracle.shard_slices(24, 36, 48, (2, 3, 4), (1, 2, 3), transposed=True)
    assert (rt, rk, rn) == (slice(18, 24), slice(24, 36), slice(24, 48))
    # Algorithm 1 as printed: I_{k,j} has m/Gz rows and k/Gy columns, W_{j,i} has n/Gx columns
    assert (rk.stop - rk.start, rn.stop - rn.start) == (36 // 3, 48 // 2)


# ---- P4: adjoint identity -------------------------------------------------------------
def test_adjoint_identity():
    X, W, dY = _rand((33, 20), 9, 0), _rand((20, 28), 9, 1, 0.02), _rand((33, 28), 9, 2)
    Xf, Wf, Gf = (syn.bf16_bits_to_f64(a) for a in (X, W, dY))
    a = np.sum(Gf * oracle.fc_fwd(X, W))
    b = np.sum(oracle.fc_dgrad(dY, W) * Xf)
    c = np.sum(oracle.fc_wgrad(X, dY) * Wf)
    assert abs(a - b) <= 1e-12 * abs(a) and abs(a - c) <= 1e-12 * abs(a)


# ---- P5: error budget of the comparison (rounding mode) ----------------------------------
def test_compare_metric_and_rounding_budget():
    rng = np.random.default_rng(0)
    ref = rng.standard_normal((256, 1024)) * 0.9
    rne = syn.f32_to_bf16_bits(ref.astype(np.float32))
    trunc = (ref.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    r = oracle.compare_bf16(rne, ref)
    t = oracle.compare_bf16(trunc, ref)
    # round-to-nearest-even costs about 1.7e-3 relative Frobenius, truncation about twice that
    assert 1.4e-3 < r["rel_fro"] < 1.9e-3 and r["n_bad"] == 0 and r["n_nonfinite"] == 0
    assert 2.8e-3 < t["rel_fro"] < 3.8e-3
    # independent numpy evaluation of the same two metrics
    c = syn.bf16_bits_to_f64(rne)
    assert math.isclose(r["rel_fro"], np.linalg.norm(c - ref) / np.linalg.norm(ref), rel_tol=1e-12)
    worst = np.max(np.abs(c - ref) / np.max(np.abs(ref), axis=1, keepdims=True))
    assert math.isclose(r["max_rel_row"], worst, rel_tol=1e-12)
    # a planted gross error is counted
    bad = rne.copy()
    bad[3, 5] = 0x42C8  # 100.0
    assert oracle.compare_bf16(bad, ref)["n_bad"] >= 1
    nan = rne.copy()
    nan[0, 0] = 0x7FC0
    assert oracle.compare_bf16(nan, ref)["n_nonfinite"] == 1


# ---- P6: GELU ---------------------------------------------------------------------------
def test_gelu_golden_values():
    for line in open(os.path.join(GOLD, "gelu_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        form, x, v = line.split()
        f = oracle.gelu_erf if form == "erf" else oracle.gelu_tanh
        assert math.isclose(f(float(x)), float(v), rel_tol=1e-13, abs_tol=1e-16), line


def test_gelu_invariants():
    from scipy.stats import norm
    xs = np.linspace(-10, 10, 2001)
    worst = 0.0
    for x in xs:
        e, t = oracle.gelu_erf(x), oracle.gelu_tanh(x)
        assert math.isclose(e - oracle.gelu_erf(-x), x, rel_tol=1e-12, abs_tol=1e-14)
        assert math.isclose(t - oracle.gelu_tanh(-x), x, rel_tol=1e-12, abs_tol=1e-14)
        assert math.isclose(e, x * norm.cdf(x), rel_tol=1e-10, abs_tol=1e-15)
        worst = max(worst, abs(e - t))
    assert 3e-4 < worst < 1e-3  # the two forms differ by about 4.7e-4 at most
    assert oracle.gelu_tanh(0.0) == 0.0 and oracle.gelu_erf(0.0) == 0.0
    assert math.isclose(oracle.gelu_tanh(9.0), 9.0, rel_tol=1e-12)
    assert -1e-10 < oracle.gelu_tanh(-9.0) <= 0.0


def test_epilogue_applies_after_the_sum():
    X, W = _rand((9, 16), 2, 0), _rand((16, 24), 2, 1, 0.3)
    b = _rand((1, 24), 2, 3, 0.5)[0]
    bf = syn.bf16_bits_to_f64(b.reshape(1, -1))[0]
    Y0 = oracle.fc_fwd(X, W)
    Yb = oracle.fc_fwd(X, W, b, oracle.EPI_BIAS)
    assert np.allclose(Yb, Y0 + bf[None, :], rtol=1e-14, atol=0)
    Yt = oracle.fc_fwd(X, W, b, oracle.EPI_BIAS_GELU_TANH)
    Ye = oracle.fc_fwd(X, W, b, oracle.EPI_BIAS_GELU_ERF)
    Yneg_t = oracle.fc_fwd(X ^ np.uint16(0x8000), W, b ^ np.uint16(0x8000), oracle.EPI_BIAS_GELU_TANH)
    Yneg_e = oracle.fc_fwd(X ^ np.uint16(0x8000), W, b ^ np.uint16(0x8000), oracle.EPI_BIAS_GELU_ERF)
    # GELU(v) - GELU(-v) = v with v the biased pre-activation: pins that the activation acts on Y0+b
    assert np.allclose(Yt - Yneg_t, Yb, rtol=1e-12, atol=1e-14)
    assert np.allclose(Ye - Yneg_e, Yb, rtol=1e-12, atol=1e-14)
    with pytest.raises(ValueError):
        oracle.fc_fwd(X, W, None, oracle.EPI_BIAS)


# ---- P7: structured inputs with exact answers ----------------------------------------
def test_structured_inputs():
    one = np.uint16(0x3F80)
    X = _rand((12, 16), 4, 0)
    eye = np.zeros((16, 16), dtype=np.uint16)
    eye[np.arange(16), np.arange(16)] = one
    assert np.array_equal(oracle.fc_fwd(X, eye), syn.bf16_bits_to_f64(X))
    assert np.array_equal(oracle.fc_dgrad(X, eye), syn.bf16_bits_to_f64(X))
    W = _rand((16, 40), 4, 1, 0.02)
    ones = np.full((5, 16), one, dtype=np.uint16)
    colsum = syn.bf16_bits_to_f64(W).sum(axis=0)
    assert np.allclose(oracle.fc_fwd(ones, W), np.tile(colsum, (5, 1)), rtol=1e-13, atol=0)
    hot = np.zeros((5, 16), dtype=np.uint16)
    hot[2, 11] = np.uint16(0x4000)  # 2.0 at (2, 11)
    Y = oracle.fc_fwd(hot, W)
    assert np.array_equal(Y[2], 2.0 * syn.bf16_bits_to_f64(W)[11]) and not Y[[0, 1, 3, 4]].any()
    # wgrad of a one-hot X picks one row of dY into one row of dW
    dY = _rand((5, 40), 4, 2)
    dW = oracle.fc_wgrad(hot, dY)
    assert np.array_equal(dW[11], 2.0 * syn.bf16_bits_to_f64(dY)[2]) and not np.delete(dW, 11, axis=0).any()


# ---- input generator ------------------------------------------------------------------
def test_generator_is_seeded_and_region_consistent():
    a = syn.normal_bf16(0, 0, (64, 48), 1.0)
    assert np.array_equal(a, syn.normal_bf16(0, 0, (64, 48), 1.0))
    assert not np.array_equal(a, syn.normal_bf16(1, 0, (64, 48), 1.0))
    assert not np.array_equal(a, syn.normal_bf16(0, 1, (64, 48), 1.0))
    assert np.array_equal(a[10:20, 8:40], syn.normal_bf16_region(0, 0, 48, 10, 10, 8, 32, 1.0))
    big = syn.bf16_bits_to_f64(syn.normal_bf16(0, 2, (512, 512), 0.02))
    assert abs(big.mean()) < 2e-4 and abs(big.std() - 0.02) < 2e-4
    L = syn.configs()["cfg1_grid222"][0]
    g = syn.global_inputs(L)
    s = syn.layer_inputs(L, (1, 0, 1))
    assert np.array_equal(s["X"], g["X"][256:512, 512:1024]) and np.array_equal(s["W"], g["W"][512:1024, 0:512])
    assert np.array_equal(s["dY"], g["dY"][256:512, 0:512])


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8, -(1.0 + 2 ** -8)], dtype=np.float32)
    got = syn.f32_to_bf16_bits(f)
    assert list(got) == [0x3F80, 0x3F80, 0x3F81, 0x3F82, 0xBF80]


def test_single_rounding_to_bf16_against_exact_rationals():
    """oracle.rne_bf16_bits against a brute-force search in exact rational arithmetic: of the two bf16
    neighbours of x the nearer one, the even one on a tie.  Values chosen to sit on and next to ties,
    where a double rounding through fp32 goes wrong."""
    from fractions import Fraction

    def bf16_value(bits):
        return Fraction(float(np.array([bits], dtype=np.uint16).astype(np.uint32).__lshift__(16).view(np.float32)[0]))

    def brute(x):
        fx = Fraction(x)
        neg = fx < 0
        mag = -fx if neg else fx
        lo, hi = 0, 0x7F7F                      # largest bf16 magnitude not above mag, by bisection on the bits
        while lo < hi:
            mid = (lo + hi + 1) // 2
            if bf16_value(mid) <= mag:
                lo = mid
            else:
                hi = mid - 1
        below, above = bf16_value(lo), bf16_value(lo + 1)
        if mag - below < above - mag:
            pick = lo
        elif mag - below > above - mag:
            pick = lo + 1
        else:
            pick = lo if lo % 2 == 0 else lo + 1
        return pick | (0x8000 if neg and pick != 0 else 0) if pick != 0 else (0x8000 if neg else 0)

    rng = np.random.default_rng(11)
    xs = list(rng.standard_normal(200) * 10.0 ** rng.integers(-6, 6, 200))
    for base in (1.0, 1.5, 3.0, 0.0078125, 1000.0):
        ulp = 2.0 ** (np.floor(np.log2(base)) - 7)
        for k in (0, 1, 2, 3):
            tie = base + (k + 0.5) * ulp          # exactly between two bf16 values
            xs += [tie, -tie, np.nextafter(tie, 0.0), np.nextafter(tie, 1e9),
                   tie + ulp * 2.0 ** -30, tie - ulp * 2.0 ** -30]   # lost when rounding to fp32 first
    xs = np.array(xs, dtype=np.float64)
    got = oracle.rne_bf16_bits(xs)
    want = np.array([brute(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want), np.argwhere(got != want)[:5]


def test_ulp_distance_counts_bf16_steps():
    ref = np.array([1.0, 1.0, 1.0, -2.0, 0.0, 0.0, 3.14159, 1e-3], dtype=np.float64)
    one, nxt, prv = 0x3F80, 0x3F81, 0x3F7F
    cand = np.array([one, nxt, prv, 0xC001, 0x8000, 0x0001, 0x4049, 0x3A83], dtype=np.uint16)
    # 1.0 exact / one up / one down (across the binade); -2.0 one step away; -0 equals +0; the
    # smallest denormal is one step from zero; pi rounds to 0x4049; 1e-3 rounds to 0x3A83
    assert list(oracle.ulp_distance_bf16(cand, ref)) == [0, 1, 1, 1, 0, 1, 0, 0]
