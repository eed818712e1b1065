"""Pins of the oracle's single-token attention with a KV cache against things other than itself:
a hand-worked case, weight patterns with closed forms, invariances of softmax attention, the
cache update, and a case whose softmax weights are exact rationals."""
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_hand_worked_case():
    d = {}
    for l in open(os.path.join(GOLDEN, "attention_case.txt")):
        if l.strip() and not l.startswith("#"):
            k, *v = l.split()
            d[k] = np.array([float(t) for t in v], np.float16)
    Kc = np.zeros((1, 1, 4, 2), np.float16)
    Vc = np.zeros((1, 1, 4, 2), np.float16)
    Kc[0, 0, 0], Kc[0, 0, 1], Vc[0, 0, 0], Vc[0, 0, 1] = d["k0"], d["k1"], d["v0"], d["v1"]
    Vc[0, 0, 2:] = 99                                     # beyond the cached tokens: must not matter
    qkv = np.stack([d["q"], d["kn"], d["vn"]]).reshape(1, 3, 1, 2)
    out, K2, V2, pre = orc.attn_decode(qkv, Kc, Vc, pos=2, scale=1.0, return_pre=True)
    assert np.allclose(pre[0], d["out"].astype(np.float64), rtol=0, atol=1e-15)
    assert np.array_equal(out[0], d["out"])
    assert np.array_equal(K2[0, 0, 2], d["kn"]) and np.array_equal(V2[0, 0, 2], d["vn"])
    assert np.array_equal(V2[0, 0, 3], Vc[0, 0, 3]) and np.array_equal(K2[0, 0, :2], Kc[0, 0, :2])


def _rand(B, H, S, d, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, 3, H, d)).astype(np.float16), rng.standard_normal((B, H, S, d)).astype(np.float16),
            rng.standard_normal((B, H, S, d)).astype(np.float16))


def test_first_token_returns_its_own_value_and_fills_the_cache():
    qkv, Kc, Vc = _rand(2, 3, 5, 8, 0)
    out, K2, V2 = orc.attn_decode(qkv, Kc, Vc, pos=0)
    assert np.array_equal(out.reshape(2, 3, 8).view(np.uint16), qkv[:, 2].view(np.uint16))     # softmax of one score is 1
    assert np.array_equal(K2[:, :, 0].view(np.uint16), qkv[:, 1].view(np.uint16))
    assert np.array_equal(V2[:, :, 0].view(np.uint16), qkv[:, 2].view(np.uint16))
    assert np.array_equal(K2[:, :, 1:], Kc[:, :, 1:]) and np.array_equal(V2[:, :, 1:], Vc[:, :, 1:])


def test_closed_form_weights():
    # equal keys -> uniform weights -> mean of the values (including the new one)
    qkv, Kc, Vc = _rand(1, 2, 9, 4, 1)
    Kc[:] = Kc[:, :, :1]
    qkv[:, 1] = Kc[:, :, 0]
    _, _, _, pre = orc.attn_decode(qkv, Kc, Vc, pos=6, return_pre=True)
    want = (Vc[:, :, :6].astype(np.float64).sum(axis=2) + qkv[:, 2].astype(np.float64)) / 7
    assert np.allclose(pre.reshape(1, 2, 4), want, rtol=1e-14, atol=1e-15)
    # scores 0 and ln(w) via the scale: weights 1/(1+w), w/(1+w)
    for w in (2.0, 3.0, 0.25):
        Kc = np.zeros((1, 1, 2, 2), np.float16); Vc = np.zeros((1, 1, 2, 2), np.float16)
        Vc[0, 0, 0] = [8, -4]
        qkv = np.zeros((1, 3, 1, 2), np.float16)
        qkv[0, 0, 0] = [1, 0]; qkv[0, 1, 0] = [1, 0]; qkv[0, 2, 0] = [-2, 6]          # new key: score = scale
        _, _, _, pre = orc.attn_decode(qkv, Kc, Vc, pos=1, scale=math.log(w), return_pre=True)
        want = (np.array([8.0, -4.0]) + w * np.array([-2.0, 6.0])) / (1 + w)
        assert np.allclose(pre[0], want, rtol=1e-14)
    # a dominating key: the output is its value to within exp(-gap)
    qkv, Kc, Vc = _rand(1, 1, 6, 8, 2)
    Kc[0, 0, 3] = (qkv[0, 0, 0].astype(np.float32) * 40).astype(np.float16)
    _, _, _, pre = orc.attn_decode(qkv, Kc, Vc, pos=5, scale=1.0, return_pre=True)
    assert np.allclose(pre[0], Vc[0, 0, 3].astype(np.float64), atol=1e-30 + 10 * math.exp(-100))


def test_invariances():
    qkv, Kc, Vc = _rand(2, 2, 12, 8, 3)
    pos = 9
    out, _, _, pre = orc.attn_decode(qkv, Kc, Vc, pos, return_pre=True)
    # cached positions can be permuted (keys and values together)
    perm = np.random.default_rng(0).permutation(pos)
    K2, V2 = Kc.copy(), Vc.copy()
    K2[:, :, :pos], V2[:, :, :pos] = Kc[:, :, perm], Vc[:, :, perm]
    _, _, _, pre2 = orc.attn_decode(qkv, K2, V2, pos, return_pre=True)
    assert np.allclose(pre2, pre, rtol=1e-13, atol=1e-15)
    # a shift of every score by a constant (query component along a direction all keys share) changes nothing
    K3 = Kc.copy(); q3 = qkv.copy()
    K3[..., 0] = 1; q3[:, 1, :, 0] = 1
    _, _, _, a = orc.attn_decode(q3, K3, Vc, pos, return_pre=True)
    q4 = q3.copy(); q4[:, 0, :, 0] = (q3[:, 0, :, 0].astype(np.float32) + 8).astype(np.float16)
    _, _, _, b = orc.attn_decode(q4, K3, Vc, pos, return_pre=True)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)
    # outputs are convex combinations of the values; heads and sequences are independent
    vals = np.concatenate([Vc[:, :, :pos], qkv[:, 2][:, :, None]], axis=2).astype(np.float64)
    p = pre.reshape(2, 2, 8)
    assert np.all(p <= vals.max(axis=2) + 1e-12) and np.all(p >= vals.min(axis=2) - 1e-12)
    o1, _, _ = orc.attn_decode(qkv[1:2, :, 1:2], Kc[1:2, 1:2], Vc[1:2, 1:2], pos)
    assert np.array_equal(o1[0].view(np.uint16), out[1, 8:16].view(np.uint16))
    # scale defaults to 1/sqrt(d)
    o2, _, _ = orc.attn_decode(qkv, Kc, Vc, pos, scale=1 / math.sqrt(8))
    assert np.array_equal(o2.view(np.uint16), out.view(np.uint16))
    with pytest.raises(RuntimeError):
        orc.attn_decode(qkv, Kc, Vc, 12)


def test_against_library_softmax():
    """The same definition assembled from library routines (scipy's softmax, numpy's einsum) in fp64."""
    from scipy.special import softmax
    qkv, Kc, Vc = _rand(3, 4, 40, 16, 4)
    pos = 33
    _, _, _, pre = orc.attn_decode(qkv, Kc, Vc, pos, return_pre=True)
    q = qkv[:, 0].astype(np.float64)
    keys = np.concatenate([Kc[:, :, :pos], qkv[:, 1][:, :, None]], axis=2).astype(np.float64)
    vals = np.concatenate([Vc[:, :, :pos], qkv[:, 2][:, :, None]], axis=2).astype(np.float64)
    w = softmax(np.einsum("bhd,bhsd->bhs", q, keys) / 4.0, axis=-1)
    want = np.einsum("bhs,bhsd->bhd", w, vals).reshape(3, -1)
    assert np.allclose(pre, want, rtol=1e-12, atol=1e-14)
