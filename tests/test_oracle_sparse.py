"""Pins of the sparsified-cache oracle: it reduces to the dense oracle when nothing is dropped,
agrees with a scalar-loop evaluation of the definition, ignores dropped tokens and their order."""
import math

import numpy as np

from oracle import attention as orc
from oracle.sparse import sparse_decode_attention, compact

RNG = np.random.default_rng(11)


def _case(B=2, T=24, Hq=4, Hkv=2, d=8):
    q = RNG.standard_normal((B, Hq, d)).astype(np.float32)
    K = RNG.standard_normal((B, T, Hkv, d)).astype(np.float32)
    V = RNG.standard_normal((B, T, Hkv, d)).astype(np.float32)
    return q, K, V


def test_keeping_everything_is_dense_attention():
    q, K, V = _case()
    B, T, Hkv = K.shape[0], K.shape[1], K.shape[2]
    lens = np.array([T, T - 5], np.int32)
    keep = [[np.arange(lens[b]) for _ in range(Hkv)] for b in range(B)]
    got = sparse_decode_attention(q, K, V, keep)
    want = orc.decode_attention(0, np.array([0], np.int32), [K], [V], q, lens)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_scalar_loops_on_a_tiny_case():
    q, K, V = _case(B=1, T=7, Hq=2, Hkv=1, d=4)
    keep = [[np.array([5, 0, 3])]]
    got = sparse_decode_attention(q, K, V, keep)
    for hq in range(2):
        w = [math.exp(sum(float(q[0, hq, c]) * float(K[0, t, 0, c]) for c in range(4)) / 2.0) for t in (5, 0, 3)]
        for c in range(4):
            ref = sum(wi * float(V[0, t, 0, c]) for wi, t in zip(w, (5, 0, 3))) / sum(w)
            assert abs(got[0, hq, c] - ref) < 1e-12


def test_dropped_tokens_and_order_do_not_matter():
    q, K, V = _case()
    keep = [[np.sort(RNG.choice(24, size=n, replace=False)) for n in (9, 17)] for _ in range(2)]
    base = sparse_decode_attention(q, K, V, keep)
    K2, V2 = K.copy(), V.copy()
    for b in range(2):
        for h in range(2):
            gone = np.setdiff1d(np.arange(24), keep[b][h])
            K2[b, gone, h] = 1e4                      # junk in dropped tokens
            V2[b, gone, h] = -1e4
    np.testing.assert_allclose(sparse_decode_attention(q, K2, V2, keep), base, rtol=1e-12)
    shuffled = [[RNG.permutation(s) for s in row] for row in keep]
    np.testing.assert_allclose(sparse_decode_attention(q, K, V, shuffled), base, rtol=1e-12, atol=1e-14)
    # the same through the compacted cache and per-head lengths
    Kc, Vc, counts = compact(K, V, keep)
    front = [[np.arange(counts[b, h]) for h in range(2)] for b in range(2)]
    np.testing.assert_allclose(sparse_decode_attention(q, Kc, Vc, front), base, rtol=1e-12, atol=1e-14)
    assert counts.tolist() == [[9, 17], [9, 17]]


def test_one_kept_token_returns_its_value_and_none_returns_zero():
    q, K, V = _case(B=1, T=5, Hq=2, Hkv=2, d=4)
    out = sparse_decode_attention(q, K, V, [[np.array([3]), np.array([], np.int64)]])
    np.testing.assert_allclose(out[0, 0], V[0, 3, 0], rtol=1e-12)
    assert np.all(out[0, 1] == 0)


def test_a_token_with_a_vanishing_weight_can_be_dropped():
    q, K, V = _case(B=1, T=6, Hq=1, Hkv=1, d=4)
    K[0, 2, 0] = -50.0 * q[0, 0] / np.dot(q[0, 0], q[0, 0])      # score -25: weight ~ e^-25 of the others
    full = sparse_decode_attention(q, K, V, [[np.arange(6)]])
    dropped = sparse_decode_attention(q, K, V, [[np.array([0, 1, 3, 4, 5])]])
    assert np.abs(full - dropped).max() < 1e-8 and np.abs(full - dropped).max() > 0
