"""Pins for the CPU oracle: everything here checks oracle/ against something that is NOT
the oracle - exact rational arithmetic, numpy's own conversions and matmul, closed forms,
textbook values, structural invariants.  No GPU needed.

The paper (Sec. III-C / III-D) states the operation only as a skinny matrix product with
bias / residual additions; it prints no worked numbers, so the pins are mathematical.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def frac_of_half(h: np.float16) -> Fraction:
    return Fraction(float(h))  # every fp16 is exactly a double, Fraction(float) is exact


def frac_to_half(fr: Fraction) -> np.float16:
    """Round a rational to fp16, nearest-even, with rational arithmetic only."""
    if fr == 0:
        return np.float16(0.0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = max(math.floor(math.log2(a)), -14)
    # guard against log2 rounding at powers of two
    while Fraction(2) ** e > a and e > -14:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    unit = Fraction(2) ** (e - 10)
    q = a / unit
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    val = fl * unit
    if val >= 65520:
        return np.float16(sign * np.inf)
    return np.float16(sign * float(val))


def brute_gemm(X, W, bias=None, R=None):
    """Exact rational X.W (+bias) (+R)."""
    B, K = X.shape
    N = W.shape[1]
    out = [[Fraction(0)] * N for _ in range(B)]
    for b in range(B):
        for n in range(N):
            s = Fraction(0)
            for k in range(K):
                s += frac_of_half(X[b, k]) * frac_of_half(W[k, n])
            if bias is not None:
                s += frac_of_half(bias[n])
            if R is not None:
                s += frac_of_half(R[b, n])
            out[b][n] = s
    return out


def small_exact(rng, shape):
    """fp16 values that are small integers times powers of two: all sums exact in fp64."""
    m = rng.integers(-8, 9, size=shape).astype(np.float64)
    p = rng.integers(-3, 3, size=shape).astype(np.float64)
    return (m * np.exp2(p)).astype(np.float16)


# ----------------------------------------------------------------------------- fp16 <-> fp64
def test_half_to_double_exhaustive_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    mine = orc.half_to_double(bits)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.array_equal(np.signbit(mine[~nan]), np.signbit(ref[~nan]))


def test_double_to_half_roundtrip_and_ties():
    bits = np.arange(0x7C00, dtype=np.uint16)           # all non-negative finite fp16
    vals = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(orc.double_to_half(vals).view(np.uint16), bits)
    assert np.array_equal(orc.double_to_half(-vals).view(np.uint16), bits | 0x8000)
    # exact midpoints between neighbours go to the even neighbour
    mid = 0.5 * (vals[:-1] + vals[1:])
    got = orc.double_to_half(mid).view(np.uint16)
    want = np.where(bits[:-1] % 2 == 0, bits[:-1], bits[1:])
    assert np.array_equal(got, want)
    # one fp64 ulp off the midpoint goes to the nearer neighbour
    assert np.array_equal(orc.double_to_half(np.nextafter(mid, np.inf)).view(np.uint16), bits[1:])
    assert np.array_equal(orc.double_to_half(np.nextafter(mid, -np.inf)).view(np.uint16), bits[:-1])
    # overflow threshold: 65520 is the midpoint between 65504 and 2^16 -> inf (ties-to-even)
    edge = orc.double_to_half(np.array([65504.0, 65519.99, 65520.0, 1e6, -65520.0, 2.0 ** -25,
                                        np.nextafter(2.0 ** -25, 1.0), 2.0 ** -26, 0.0, -0.0]))
    assert list(edge.view(np.uint16)) == [0x7BFF, 0x7BFF, 0x7C00, 0x7C00, 0xFC00, 0x0000,
                                          0x0001, 0x0000, 0x0000, 0x8000]


def test_double_to_half_is_single_rounding():
    # 1 + 2^-11 + 2^-30 lies just above the midpoint of 1 and 1+2^-10: a float32 detour
    # would first round to the midpoint and then to even (1.0); one rounding gives 1+2^-10.
    v = 1.0 + 2.0 ** -11 + 2.0 ** -30
    assert orc.double_to_half(np.array([v]))[0] == np.float16(1.0 + 2.0 ** -10)
    assert np.float64(v).astype(np.float32).astype(np.float16) == np.float16(1.0)


def test_double_to_half_random_vs_numpy_and_rationals():
    rng = np.random.default_rng(7)
    v = np.concatenate([rng.standard_normal(500_000) * 4.0,
                        rng.standard_normal(250_000) * 1e-4,     # around the subnormal border
                        rng.standard_normal(250_000) * 3e4])     # around overflow
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16)                               # numpy: one RNE step
    got = orc.double_to_half(v)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))
    for x in v[:300].tolist() + v[500_000:500_300].tolist() + v[750_000:750_100].tolist():
        assert orc.double_to_half(np.array([x]))[0].view(np.uint16) == \
            frac_to_half(Fraction(x)).view(np.uint16)


# ----------------------------------------------------------------------------- GeLU
def test_gelu_golden_closed_forms():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gelu_closed_form.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 7
    for xs, vs, hs in rows:
        x, v, hbits = float(xs), float(vs), int(hs, 16)
        assert orc.gelu(x) == pytest.approx(v, rel=1e-15, abs=1e-17)
        # fp16 column: rational rounding of the stored value (independent of the oracle) ...
        assert frac_to_half(Fraction(v)).view(np.uint16) == hbits
        # ... and the oracle's epilogue reaches it through a 1x1 GeMM  1*x -> gelu
        Y = orc.gemm(np.array([[x]], np.float16), np.array([[1.0]], np.float16), epi=orc.EPI_GELU)
        assert Y.view(np.uint16)[0, 0] == hbits


def test_gelu_identities():
    # x Phi(x) - (-x) Phi(-x) = x (Phi(x) + Phi(-x)) = x
    for x in np.linspace(-8, 8, 161):
        assert orc.gelu(x) - orc.gelu(-x) == pytest.approx(x, abs=1e-14)
    # standard normal CDF table values
    assert orc.gelu(1.0) / 1.0 == pytest.approx(0.8413447460685429, rel=1e-15)
    assert orc.gelu(2.0) / 2.0 == pytest.approx(0.9772498680518208, rel=1e-15)
    assert orc.gelu(3.0) / 3.0 == pytest.approx(0.9986501019683699, rel=1e-15)
    # global minimum of x Phi(x): where Phi(x) + x phi(x) = 0, x ~ -0.7517915
    xs = np.linspace(-1.5, 0.0, 150001)
    vals = np.array([orc.gelu(x) for x in xs[::50]])
    i = int(vals.argmin())
    assert xs[::50][i] == pytest.approx(-0.7517915, abs=1e-3)
    assert vals[i] == pytest.approx(-0.16997120748, abs=1e-7)
    assert np.all(np.diff(np.array([orc.gelu(x) for x in np.linspace(-0.75, 6, 500)])) > 0)
    # far tails round to +-x / -0 in fp16
    Y = orc.gemm(np.array([[6.0], [-6.0]], np.float16), np.array([[1.0]], np.float16), epi=orc.EPI_GELU)
    assert list(Y.view(np.uint16).ravel()) == [0x4600, 0x8000]
    # tanh approximation differs visibly from the erf form: the oracle must be the erf form
    x = 2.7
    tanh_form = 0.5 * x * (1 + math.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))
    assert abs(orc.gelu(x) - tanh_form) > 1e-4


# ----------------------------------------------------------------------------- GeMM
def test_tiny_golden_case():
    d = {}
    for l in open(os.path.join(GOLDEN, "tiny_gemm_case.txt")):
        if l.strip() and not l.startswith("#"):
            k, *v = l.split()
            d[k] = np.array([float(t) for t in v])
    X = d["X"].reshape(1, 4).astype(np.float16)
    W = d["W"].reshape(4, 2).astype(np.float16)
    bias = d["bias"].astype(np.float16)
    R = d["residual"].reshape(1, 2).astype(np.float16)
    assert np.array_equal(orc.gemm(X, W, bias, epi=orc.EPI_BIAS).astype(np.float64)[0], d["acc_plus_bias"])
    assert np.array_equal(orc.gemm(X, W, bias, R, epi=orc.EPI_BIAS | orc.EPI_RES).astype(np.float64)[0],
                          d["with_residual"])
    # GeLU of the same pre-activations, against math.erf evaluated here
    Y, pre = orc.gemm(X, W, bias, epi=orc.EPI_BIAS | orc.EPI_GELU, return_pre=True)
    for j, v in enumerate(d["acc_plus_bias"]):
        want = 0.5 * v * (1 + math.erf(v / math.sqrt(2)))
        assert pre[0, j] == pytest.approx(want, rel=1e-14)
        assert Y[0, j] == frac_to_half(Fraction(want))
    # without the bias flag the bias must not be added
    assert np.array_equal(orc.gemm(X, W, epi=0).astype(np.float64)[0], d["acc_plus_bias"] - d["bias"])


@pytest.mark.parametrize("B,K,N", [(1, 1, 1), (1, 5, 3), (3, 7, 2), (2, 8, 8), (4, 3, 6), (5, 6, 4)])
def test_brute_force_exact_rationals(B, K, N):
    rng = np.random.default_rng(B * 100 + K * 10 + N)
    X, W = small_exact(rng, (B, K)), small_exact(rng, (K, N))
    bias, R = small_exact(rng, (N,)), small_exact(rng, (B, N))
    for epi, bb, rr in [(0, None, None), (orc.EPI_BIAS, bias, None),
                        (orc.EPI_BIAS | orc.EPI_RES, bias, R), (orc.EPI_RES, None, R)]:
        Y, pre = orc.gemm(X, W, bb, rr, epi=epi, return_pre=True)
        ref = brute_gemm(X, W, bb, rr)
        for b in range(B):
            for n in range(N):
                assert Fraction(float(pre[b, n])) == ref[b][n]          # sums are exact here
                assert Y[b, n].view(np.uint16) == frac_to_half(ref[b][n]).view(np.uint16) or \
                    (Y[b, n] == 0 and ref[b][n] == 0)


def test_brute_force_gaussian_inputs_non_square():
    # realistic values (inexact sums), non-square so a transposed operand cannot pass
    rng = np.random.default_rng(11)
    B, K, N = 3, 37, 5
    X = rng.standard_normal((B, K)).astype(np.float16)
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
    bias = (rng.standard_normal(N) * 0.02).astype(np.float16)
    R = rng.standard_normal((B, N)).astype(np.float16)
    Y, pre = orc.gemm(X, W, bias, R, epi=orc.EPI_BIAS | orc.EPI_RES, return_pre=True)
    ref = brute_gemm(X, W, bias, R)
    for b in range(B):
        for n in range(N):
            assert float(pre[b, n]) == pytest.approx(float(ref[b][n]), rel=1e-13, abs=1e-15)
            assert Y[b, n].view(np.uint16) == frac_to_half(ref[b][n]).view(np.uint16)
    # GeLU variant: gelu applied to (acc + bias), never to the residual
    Yg, preg = orc.gemm(X, W, bias, epi=orc.EPI_BIAS | orc.EPI_GELU, return_pre=True)
    refb = brute_gemm(X, W, bias, None)
    for b in range(B):
        for n in range(N):
            v = float(refb[b][n])
            assert preg[b, n] == pytest.approx(0.5 * v * (1 + math.erf(v / math.sqrt(2))), rel=1e-12, abs=1e-15)


def test_identity_onehot_twohot_weights():
    rng = np.random.default_rng(3)
    B, K = 4, 96
    X = rng.standard_normal((B, K)).astype(np.float16)
    eye = np.eye(K, dtype=np.float16)
    assert np.array_equal(orc.gemm(X, eye).view(np.uint16), X.view(np.uint16))
    perm = rng.permutation(K)
    P = np.zeros((K, K), np.float16)
    P[perm, np.arange(K)] = 1.0                                  # column n picks row perm[n]
    assert np.array_equal(orc.gemm(X, P).view(np.uint16), X[:, perm].view(np.uint16))
    # two ones per column: Y = RNE16(x_i + x_j), one rounding of the exact sum
    N = 40
    i, j = rng.integers(0, K, N), rng.integers(0, K, N)
    j = np.where(i == j, (j + 1) % K, j)
    T = np.zeros((K, N), np.float16)
    T[i, np.arange(N)] = 1.0
    T[j, np.arange(N)] = 1.0
    want = (X[:, i].astype(np.float64) + X[:, j].astype(np.float64)).astype(np.float16)
    assert np.array_equal(orc.gemm(X, T).view(np.uint16), want.view(np.uint16))


def test_linearity_additivity_independence():
    rng = np.random.default_rng(5)
    B, K, N = 8, 300, 70
    X = rng.standard_normal((B, K)).astype(np.float16)
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
    Y, pre = orc.gemm(X, W, return_pre=True)
    # zero-bias linearity, exact for powers of two (before and after rounding)
    # (scaling up only: scaling down could push inputs into the fp16 subnormal range)
    normal = np.abs(Y.astype(np.float64)) >= 2.0 ** -14
    for a in (2.0, 8.0, 32.0):
        Ya, prea = orc.gemm((X.astype(np.float64) * a).astype(np.float16), W, return_pre=True)
        assert np.array_equal(prea, a * pre)
        assert np.array_equal(Ya.astype(np.float64)[normal], (Y.astype(np.float64) * a)[normal])
    # general scalar: to fp64 accuracy, using an X whose scaling by 3 is exact in fp16
    Xs = (rng.integers(-100, 100, (B, K))).astype(np.float16)
    _, p1 = orc.gemm(Xs, W, return_pre=True)
    _, p3 = orc.gemm((Xs.astype(np.float64) * 3).astype(np.float16), W, return_pre=True)
    assert np.allclose(p3, 3 * p1, rtol=1e-12, atol=1e-13)
    # additivity over a split of K
    _, pa = orc.gemm(X[:, :128], W[:128], return_pre=True)
    _, pb = orc.gemm(X[:, 128:], W[128:], return_pre=True)
    assert np.allclose(pa + pb, pre, rtol=1e-12, atol=1e-14)
    # column independence (bit-exact) and row independence (bit-exact)
    assert np.array_equal(orc.gemm(X, np.ascontiguousarray(W[:, 13:50])).view(np.uint16),
                          Y[:, 13:50].view(np.uint16))
    for b in (0, 5):
        assert np.array_equal(orc.gemm(X[b:b + 1], W).view(np.uint16), Y[b:b + 1].view(np.uint16))
    # thread count changes nothing
    assert np.array_equal(orc.gemm(X, W, threads=1).view(np.uint16), Y.view(np.uint16))


def test_against_numpy_float64_matmul_and_statistics():
    from paper_2207_00032_amd import workloads as wl
    K, N, B = 1024, 768, 8
    W, bias, X, R = wl.make_gemm_inputs(K, N, B, seed=0, config_id=99, gemm_id=0)
    Y, pre = orc.gemm(X, W, bias, R, epi=orc.EPI_BIAS | orc.EPI_RES, return_pre=True)
    ref = X.astype(np.float64) @ W.astype(np.float64) + bias.astype(np.float64) + R.astype(np.float64)
    assert np.allclose(pre, ref, rtol=1e-12, atol=1e-13)
    assert np.array_equal(Y.view(np.uint16), ref.astype(np.float16).view(np.uint16))
    # sample std of X.W with sigma_w = 0.02, sigma_x = 1 is 0.02 sqrt(K)
    _, p0 = orc.gemm(X, W, return_pre=True)
    assert p0.std() == pytest.approx(0.02 * math.sqrt(K), rel=0.05)
    # scipy's erf agrees with libm's through the GeLU epilogue
    from scipy.special import erf as sp_erf
    _, pg = orc.gemm(X, W, bias, epi=orc.EPI_BIAS | orc.EPI_GELU, return_pre=True)
    v = X.astype(np.float64) @ W.astype(np.float64) + bias.astype(np.float64)
    assert np.allclose(pg, 0.5 * v * (1 + sp_erf(v / math.sqrt(2))), rtol=1e-11, atol=1e-14)


def test_bad_arguments_rejected():
    X = np.zeros((2, 4), np.float16)
    W = np.zeros((4, 3), np.float16)
    with pytest.raises(ValueError):
        orc.gemm(X, np.zeros((5, 3), np.float16))
    with pytest.raises((ValueError, TypeError)):
        orc.gemm(X, W, None, epi=orc.EPI_BIAS)
    with pytest.raises(TypeError):
        orc.gemm(X.astype(np.float32), W)


# ----------------------------------------------------------------------------- layout
@pytest.mark.parametrize("K,N", [(32, 64), (8, 1), (40, 24), (103, 71), (264, 200), (512, 1024)])
def test_layout_is_a_pure_permutation_with_zero_padding(K, N):
    rng = np.random.default_rng(K * 1000 + N)
    W = rng.integers(1, 65536, size=(K, N), dtype=np.uint16)      # no zeros: padding is identifiable
    flat = orc.layout_weights(W)
    KS, P = orc.layout_dims(K, N)
    assert flat.size == P * KS * 4 * 64 * 8
    assert np.array_equal(orc.unlayout_weights(flat, K, N), W)
    assert np.array_equal(np.sort(flat[flat != 0]), np.sort(W.ravel()))
    assert (flat == 0).sum() == flat.size - K * N


def test_layout_index_formula_brute_force():
    K, N = 70, 90
    W = (np.arange(K * N, dtype=np.uint32) % 65535 + 1).astype(np.uint16).reshape(K, N)
    flat = orc.layout_weights(W)
    KS, _ = orc.layout_dims(K, N)
    for k in range(K):
        for n in range(N):
            p, t, i = n // 64, (n % 64) // 16, n % 16
            ks, g, e = k // 32, (k % 32) // 8, k % 8
            assert KS == 8 * -(-(-(-K // 32)) // 8)
            lane = g * 16 + i
            assert flat[((((p * KS + ks) * 4 + t) * 64 + lane) * 8) + e] == W[k, n]


# ----------------------------------------------------------------------------- acceptance rule
def test_ulp16_and_check_close():
    assert orc.ulp16(1.0) == 2.0 ** -10 and orc.ulp16(1.999) == 2.0 ** -10
    assert orc.ulp16(4.0) == 2.0 ** -8 and orc.ulp16(7.9) == 2.0 ** -8
    assert orc.ulp16(1e-6) == 2.0 ** -24 and orc.ulp16(0.0) == 2.0 ** -24
    assert orc.ulp16(-300.0) == 2.0 ** -2
    w = np.array([8.0, 8.0, 0.1, 0.1, np.inf], np.float16)
    ok, _ = orc.check_close(np.array([8.0 + 2 * 2 ** -7, 8.0, 0.1 + 9e-4, 0.1, np.inf], np.float16), w)
    assert ok
    ok, rep = orc.check_close(np.array([8.0 + 3 * 2 ** -7, 8.0, 0.1, 0.1, np.inf], np.float16), w)
    assert not ok and rep["n_bad"] == 1
    ok, _ = orc.check_close(np.array([8.0, 8.0, 0.1 + 2e-3, 0.1, np.inf], np.float16), w)
    assert not ok
    ok, _ = orc.check_close(np.array([8.0, 8.0, 0.1, 0.1, 65504.0], np.float16), w)
    assert not ok


# ----------------------------------------------------------------------------- layer norm
def test_layernorm_golden_and_closed_forms():
    d = {}
    for l in open(os.path.join(GOLDEN, "layernorm_case.txt")):
        if l.strip() and not l.startswith("#"):
            k, *v = l.split()
            d[k] = np.array([float(t) for t in v])
    y, pre = orc.layernorm(d["x"].reshape(1, 4).astype(np.float16), d["gamma"].astype(np.float16),
                           d["beta"].astype(np.float16), d["eps"][0], return_pre=True)
    assert np.allclose(pre[0], d["y"], rtol=0, atol=1e-15)
    assert np.array_equal(y[0].astype(np.float64), d["y"])
    K = 64
    g = np.linspace(0.5, 2.0, K).astype(np.float16)
    b = np.linspace(-1.0, 1.0, K).astype(np.float16)
    # a constant row has zero variance: every output is beta
    y = orc.layernorm(np.full((1, K), 3.25, np.float16), g, b, 1e-5)
    assert np.array_equal(y[0].view(np.uint16), b.view(np.uint16))
    # alternating +-1: mean 0, variance 1 -> x / sqrt(1 + eps) * gamma + beta
    x = np.tile(np.array([1.0, -1.0], np.float16), K // 2).reshape(1, K)
    eps = float(np.float32(1e-5))
    _, pre = orc.layernorm(x, g, b, 1e-5, return_pre=True)
    want = x[0].astype(np.float64) / math.sqrt(1.0 + eps) * g.astype(np.float64) + b.astype(np.float64)
    assert np.allclose(pre[0], want, rtol=1e-15, atol=0)


def test_layernorm_invariants_and_numpy():
    rng = np.random.default_rng(21)
    B, K = 5, 777
    X = (rng.standard_normal((B, K)) * 3 + 1.5).astype(np.float16)
    g = (1 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    b = (0.1 * rng.standard_normal(K)).astype(np.float16)
    y, pre = orc.layernorm(X, g, b, 1e-5, return_pre=True)
    Xd = X.astype(np.float64)
    mu = Xd.mean(axis=1, keepdims=True)
    var = ((Xd - mu) ** 2).mean(axis=1, keepdims=True)            # biased variance
    ref = (Xd - mu) / np.sqrt(var + float(np.float32(1e-5))) * g.astype(np.float64) + b.astype(np.float64)
    assert np.allclose(pre, ref, rtol=1e-12, atol=1e-13)
    assert np.array_equal(y.view(np.uint16), ref.astype(np.float16).view(np.uint16))
    # unbiased variance (K-1) would be visibly different: the oracle uses the biased one
    ref_unbiased = (Xd - mu) / np.sqrt(var * K / (K - 1) + 1e-5) * g.astype(np.float64) + b.astype(np.float64)
    assert np.abs(pre - ref_unbiased).max() > 1e-4
    # with gamma = 1, beta = 0, eps = 0 the output has mean 0 and variance 1 ...
    one, zero = np.ones(K, np.float16), np.zeros(K, np.float16)
    _, p0 = orc.layernorm(X, one, zero, 0.0, return_pre=True)
    assert np.allclose(p0.mean(axis=1), 0, atol=1e-13) and np.allclose((p0 ** 2).mean(axis=1), 1, rtol=1e-12)
    # ... and is invariant to a power-of-two scaling of the row (exact in fp16)
    _, p2 = orc.layernorm((Xd * 4).astype(np.float16), one, zero, 0.0, return_pre=True)
    assert np.allclose(p2, p0, rtol=1e-12, atol=1e-13)
    # rows are independent
    assert np.array_equal(orc.layernorm(X[2:3], g, b, 1e-5).view(np.uint16), y[2:3].view(np.uint16))
    with pytest.raises(ValueError):
        orc.layernorm(X, g[:-1], b, 1e-5)
