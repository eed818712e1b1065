"""Pins of the oracle's INT8 functions (symmetric quantisation, exact-integer GeMM) against things
other than themselves: a hand-worked case, exact rational brute force, properties that any correct
symmetric quantiser has, and the special case in which the INT8 path must reproduce the fp16 GeMM
oracle bit for bit (integer-valued operands with amax = 127: every scale is exactly 1)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _golden():
    d = {}
    for l in open(os.path.join(GOLDEN, "int8_quantize_case.txt")):
        if l.strip() and not l.startswith("#"):
            k, *v = l.split()
            d[k] = [float(t) for t in v]
    return d


def test_quantize_hand_worked_case_rows_and_columns():
    d = _golden()
    X = np.array([d["a_values"], d["b_values"]], np.float16)
    q, s = orc.quantize_rows(X)
    assert q.tolist() == [[int(v) for v in d["a_codes"]], [int(v) for v in d["b_codes"]]]
    assert s[0] == np.float32(d["a_scale_num"][0]) / np.float32(d["a_scale_den"][0]) == 1.0
    assert s[1] == np.float32(np.float32(2.0) / np.float32(127.0))
    # columns: the same lines as columns of a [4,2] matrix give the same codes and scales
    qc, sc = orc.quantize_columns(np.ascontiguousarray(X.T))
    assert np.array_equal(qc, q.T) and np.array_equal(sc, s)


def test_quantize_properties():
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((7, 301)) * np.exp(rng.uniform(-3, 3, (7, 1)))).astype(np.float16)
    X[3] = 0                                            # an all-zero line: codes 0, scale 0
    q, s = orc.quantize_rows(X)
    Xd = X.astype(np.float64)
    amax = np.abs(Xd).max(axis=1)
    assert np.all(np.abs(q).max(axis=1)[amax > 0] == 127) and np.all(np.abs(q) <= 127)
    assert not q[3].any() and s[3] == 0.0
    # the element of largest magnitude gets +-127 with its sign
    for b in np.flatnonzero(amax > 0):
        j = np.argmax(np.abs(Xd[b]))
        assert q[b, j] == int(np.sign(Xd[b, j])) * 127
    # scale is amax/127 rounded to binary32; the reconstruction error is at most half a step
    # (plus the binary32 rounding of the reciprocal, below 1e-6 of a step per code unit)
    assert np.array_equal(s, (amax.astype(np.float32) / np.float32(127)).astype(np.float32))
    err = np.abs(Xd - q * s.astype(np.float64)[:, None])
    assert np.all(err <= s.astype(np.float64)[:, None] * (0.5 + 2e-4))
    # odd symmetry, and invariance of the codes under an exact (power of two) rescaling
    q2, s2 = orc.quantize_rows((-X))
    assert np.array_equal(q2, -q) and np.array_equal(s2, s)
    keep = np.abs(Xd).max(axis=1) < 1000
    q4, s4 = orc.quantize_rows((X[keep].astype(np.float32) * 4).astype(np.float16))
    assert np.array_equal(q4, q[keep]) and np.array_equal(s4, s[keep] * np.float32(4))
    # monotone: a larger value never gets a smaller code
    for b in (0, 5):
        order = np.argsort(Xd[b], kind="stable")
        assert np.all(np.diff(q[b][order].astype(int)) >= 0)


def test_quantize_ties_round_to_even_in_binary32():
    # amax = 127 -> reciprocal scale exactly 1: x.5 values are exact ties
    vals = np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 62.5, 63.5], np.float16)
    q, s = orc.quantize_rows(vals.reshape(1, -1))
    assert s[0] == 1.0 and q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 62, 64]


def _exact_i8(Xq, sx, Wq, sw, bias, R, epi):
    """Exact rational evaluation of the definition on tiny inputs; GeLU needs erf, so only
    the bias / residual epilogues are evaluated here."""
    B, K = Xq.shape
    N = Wq.shape[1]
    out = np.empty((B, N), np.float16)
    for b in range(B):
        for n in range(N):
            acc = sum(int(Xq[b, k]) * int(Wq[k, n]) for k in range(K))
            v = Fraction(acc) * Fraction(float(sx[b])) * Fraction(float(sw[n]))
            if epi & orc.EPI_BIAS:
                v += Fraction(float(bias[n]))
            if epi & orc.EPI_RES:
                v += Fraction(float(R[b, n]))
            # nearest fp16, ties to even, from the exact rational: candidates around float(v)
            f = np.float16(float(v))
            cands = sorted({np.nextafter(f, np.float16(-np.inf)), f, np.nextafter(f, np.float16(np.inf))},
                           key=lambda c: (abs(Fraction(float(c)) - v), int(np.float16(c).view(np.uint16)) & 1))
            out[b, n] = cands[0]
    return out


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_gemm_i8_exact_rational_brute_force(seed):
    rng = np.random.default_rng(seed)
    B, K, N = 3, 37, 5
    Xq = rng.integers(-127, 128, (B, K), dtype=np.int8)
    Wq = rng.integers(-127, 128, (K, N), dtype=np.int8)
    sx = rng.uniform(1e-3, 0.05, B).astype(np.float32)
    sw = rng.uniform(1e-4, 1e-3, N).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16)
    R = rng.standard_normal((B, N)).astype(np.float16)
    for epi in (0, orc.EPI_BIAS, orc.EPI_RES, orc.EPI_BIAS | orc.EPI_RES):
        got = orc.gemm_i8(Xq, sx, Wq, sw, bias, R, epi)
        want = _exact_i8(Xq, sx, Wq, sw, bias, R, epi)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), epi


def test_int8_path_reduces_to_the_fp16_gemm_when_scales_are_one():
    """Integer-valued X and W with amax = 127 in every row / column quantise to themselves with
    scale 1, so the whole INT8 path must give the fp16 GeMM oracle's bits (all epilogues)."""
    rng = np.random.default_rng(9)
    B, K, N = 4, 96, 70
    X = rng.integers(-20, 21, (B, K)).astype(np.float16)
    W = rng.integers(-3, 4, (K, N)).astype(np.float16)
    X[:, 0] = 127
    W[0, :] = -127
    bias = (rng.standard_normal(N)).astype(np.float16)
    R = rng.standard_normal((B, N)).astype(np.float16)
    Wq, sw = orc.quantize_columns(W)
    Xq, sx = orc.quantize_rows(X)
    assert np.all(sw == 1) and np.all(sx == 1)
    assert np.array_equal(Wq, W.astype(np.int8)) and np.array_equal(Xq, X.astype(np.int8))
    for epi in (0, orc.EPI_BIAS, orc.EPI_BIAS | orc.EPI_GELU, orc.EPI_BIAS | orc.EPI_RES, orc.EPI_GELU):
        a = orc.gemm_i8_from_fp16(X, Wq, sw, bias, R, epi)
        b = orc.gemm(X, W, bias, R, epi=epi)
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), epi


def test_gemm_i8_structure():
    rng = np.random.default_rng(3)
    B, K, N = 5, 64, 64
    X = rng.standard_normal((B, K)).astype(np.float16)
    Xq, sx = orc.quantize_rows(X)
    # 127 * identity with scale 1/127: the GeMM returns the de-quantised activations
    Wq = (127 * np.eye(K, dtype=np.int64)).astype(np.int8)
    sw = np.full(N, 1.0 / 127.0, np.float32)
    y, pre = orc.gemm_i8(Xq, sx, Wq, sw, return_pre=True)
    want = Xq.astype(np.float64) * 127 * sx.astype(np.float64)[:, None] * np.float64(np.float32(1.0 / 127.0))
    assert np.allclose(pre, want, rtol=1e-15, atol=0)
    # scales act linearly, rows and columns are independent, a zero code row gives the epilogue of 0
    Wr = rng.integers(-127, 128, (K, N), dtype=np.int8)
    s1 = rng.uniform(1e-3, 1e-2, N).astype(np.float32)
    _, p1 = orc.gemm_i8(Xq, sx, Wr, s1, return_pre=True)
    _, p2 = orc.gemm_i8(Xq, sx * np.float32(2), Wr, s1, return_pre=True)
    assert np.array_equal(p2, 2 * p1)
    _, p3 = orc.gemm_i8(Xq[1:2], sx[1:2], Wr[:, 7:9], s1[7:9], return_pre=True)
    assert np.array_equal(p3, p1[1:2, 7:9])
    numpy_acc = Xq.astype(np.int64) @ Wr.astype(np.int64)
    assert np.allclose(p1, numpy_acc * sx.astype(np.float64)[:, None] * s1.astype(np.float64)[None, :], rtol=1e-15)
    bias = rng.standard_normal(N).astype(np.float16)
    z = orc.gemm_i8(np.zeros((1, K), np.int8), np.zeros(1, np.float32), Wr, s1, bias, None, orc.EPI_BIAS | orc.EPI_GELU)
    bd = bias.astype(np.float64)
    want = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in bd]).astype(np.float16)
    assert np.array_equal(z[0].view(np.uint16), want.view(np.uint16))
    with pytest.raises(ValueError):
        orc.gemm_i8(Xq, sx[:-1], Wr, s1)


def test_quantisation_error_of_the_whole_path_is_what_the_step_sizes_allow():
    """End to end against the fp16 GeMM oracle: |int8 path - fp16 path| is bounded by the
    quantisation steps (a sanity bound, and the reason INT8 outputs are NOT compared with the
    fp16 oracle in the parity tests)."""
    rng = np.random.default_rng(11)
    B, K, N = 4, 512, 48
    X = rng.standard_normal((B, K)).astype(np.float16)
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
    Wq, sw = orc.quantize_columns(W)
    _, p8 = orc.gemm_i8(*orc.quantize_rows(X), Wq, sw, return_pre=True)
    _, p16 = orc.gemm(X, W, return_pre=True)
    Xq, sx = orc.quantize_rows(X)
    bound = (np.abs(X.astype(np.float64)).sum(axis=1)[:, None] * sw.astype(np.float64)[None, :] / 2 +
             np.abs(W.astype(np.float64)).sum(axis=0)[None, :] * sx.astype(np.float64)[:, None] / 2 +
             K * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :] / 4) * 1.001
    assert np.all(np.abs(p8 - p16) <= bound)
    assert np.abs(p8 - p16).max() > 1e-4               # and it is not the same computation


def test_layernorm_in_front_of_int8_closed_forms():
    """Layer-norm, then INT8.  Rows of alternating +-a have mean 0 and variance a^2, so they
    normalise to +-1/sqrt(1 + eps/a^2), which rounds to +-1 in fp16 for eps = 1e-5: with gamma = g
    (a power of two) and beta = 0 every code is +-127 and the row scale g/127, hence
    Y[b,n] = g * sum_k (+-1) * Wq[k,n] * sw[n], exactly (small integers).  A second case keeps beta:
    the normalised values +-g + c must be quantised AFTER the rounding to fp16."""
    K, N, B = 64, 5, 3
    rng = np.random.default_rng(5)
    sign = np.where(np.arange(K) % 2 == 0, 1.0, -1.0)
    X = np.stack([sign * a for a in (0.5, 3.0, 40.0)]).astype(np.float16)
    Wq = rng.integers(-127, 128, (K, N)).astype(np.int8)
    sw = np.array([1.0, 0.5, 2.0, 0.25, 1.0], np.float32)
    for g in (1.0, 0.25, 4.0):
        gamma = np.full(K, g, np.float16)
        beta = np.zeros(K, np.float16)
        Y = orc.gemm_i8_ln_from_fp16(X, gamma, beta, 1e-5, Wq, sw)
        want = g * (sign[:, None] * Wq.astype(np.float64)).sum(axis=0) * sw
        assert np.array_equal(Y, np.tile(want, (B, 1)).astype(np.float16))
    # with beta = 0.5 and gamma = 1: values 1.5 and -0.5, amax 1.5, codes 127 and rint(-0.5 * 127/1.5) = -42
    gamma = np.ones(K, np.float16)
    beta = np.full(K, 0.5, np.float16)
    Xq, sx = orc.quantize_rows(orc.layernorm(X, gamma, beta, 1e-5))
    assert np.array_equal(Xq, np.tile(np.where(sign > 0, 127, -42).astype(np.int8), (B, 1)))
    assert np.array_equal(sx, np.full(B, np.float32(1.5) / np.float32(127), np.float32))
    Y = orc.gemm_i8_ln_from_fp16(X, gamma, beta, 1e-5, Wq, sw)
    want = (np.where(sign > 0, 127, -42)[:, None] * Wq.astype(np.float64)).sum(axis=0) * np.float64(sx[0]) * sw
    assert np.array_equal(Y, np.tile(want, (B, 1)).astype(np.float16))
    # and it is the composition, step by step
    Xn = orc.layernorm(X, gamma, beta, 1e-5)
    assert np.array_equal(Y, orc.gemm_i8_from_fp16(Xn, Wq, sw))


def test_layout_i8_index_formula():
    rng = np.random.default_rng(2)
    K, N = 200, 150
    Wq = rng.integers(-127, 128, (K, N), dtype=np.int8)
    flat = orc.layout_weights_i8(Wq)
    KS, P = orc.layout_dims_i8(K, N)
    assert (KS, P) == (8, 3) and flat.size == P * KS * 4 * 64 * 16
    for k, n in [(0, 0), (15, 15), (16, 0), (63, 63), (64, 64), (199, 149), (100, 70), (17, 129)]:
        p, t, i = n // 64, (n % 64) // 16, n % 16
        ks, g, e = k // 64, (k % 64) // 16, k % 16
        assert flat[((((p * KS + ks) * 4 + t) * 64 + (g * 16 + i)) * 16) + e] == Wq[k, n]
    assert np.count_nonzero(flat) == np.count_nonzero(Wq)          # everything else is zero padding
