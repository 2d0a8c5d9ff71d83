"""Pins of the attention oracle against facts it does not itself supply.

Closed forms and brute force fix the definition (scale 1/sqrt(d), softmax over keys,
weighted sum of values, grouped-query head mapping); torch's fp64 scaled-dot-product
attention is the library routine the unshared case reduces to; the sharing substitution
(paper Sec. 3.2) is pinned by identity-map and donor-substitution invariants.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention as orc

RNG = np.random.default_rng(20241018)


def _f32(*shape):
    return RNG.standard_normal(shape).astype(np.float32)


def _decode1(q, K, V, n, L=1, layer=0, share=None, **kw):
    """Single-layer helper: q [B,Hq,d], K/V [B,T,Hkv,d]."""
    share = np.arange(L, dtype=np.int32) if share is None else share
    Ks = [None] * L
    Vs = [None] * L
    Ks[share[layer]] = K
    Vs[share[layer]] = V
    return orc.decode_attention(layer, share, Ks, Vs, q, np.asarray(n), **kw)


def test_closed_form_prescribed_probabilities():
    # q = (sqrt(2), 0), k_j = (ln a_j, junk)  =>  z_j = ln a_j  =>  p_j = a_j / sum(a)
    a = np.array([1.0, 2.0, 3.0])
    q = np.array([[[math.sqrt(2.0), 0.0]]], dtype=np.float32)            # B=1,Hq=1,d=2
    K = np.zeros((1, 3, 1, 2), np.float32)
    K[0, :, 0, 0] = np.log(a)
    K[0, :, 0, 1] = [7.0, -3.0, 11.0]                                    # q[1]=0 kills it
    V = np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 50.0]], np.float32).reshape(1, 3, 1, 2)
    out, probs = _decode1(q, K, V, [3], return_probs=True)
    np.testing.assert_allclose(probs[0, 0, :3], a / a.sum(), rtol=2e-7)
    want = (a / 6.0) @ np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 50.0]])
    np.testing.assert_allclose(out[0, 0], want, rtol=2e-7)


def test_scale_is_inverse_sqrt_d():
    # d = 4, q = (2,0,0,0), k = (ln 3, ..) vs (0, ..): z = (ln 3, 0) => p = (3/4, 1/4)
    q = np.zeros((1, 1, 4), np.float32); q[0, 0, 0] = 2.0
    K = np.zeros((1, 2, 1, 4), np.float32); K[0, 0, 0, 0] = math.log(3.0)
    V = np.zeros((1, 2, 1, 4), np.float32); V[0, 0, 0, :] = 1.0
    out = _decode1(q, K, V, [2])
    np.testing.assert_allclose(out[0, 0], 0.75, rtol=2e-7)


def test_special_cases():
    d, n = 2, 3
    q = _f32(1, 1, d)
    V = _f32(1, n, 1, d)
    # all keys equal => uniform weights => mean of the values
    K = np.repeat(_f32(1, 1, 1, d), n, axis=1)
    np.testing.assert_allclose(_decode1(q, K, V, [n])[0, 0], V[0, :, 0].astype(np.float64).mean(0), rtol=1e-12)
    # one key => its value row
    np.testing.assert_array_equal(_decode1(q, K, V, [1])[0, 0], V[0, 0, 0].astype(np.float64))
    # constant values => that constant
    Vc = np.full((1, n, 1, d), 2.5, np.float32)
    np.testing.assert_allclose(_decode1(q, _f32(1, n, 1, d), Vc, [n])[0, 0], 2.5, rtol=1e-14)
    # a dominating key => its value row
    K2 = np.zeros((1, n, 1, d), np.float32); K2[0, 1, 0] = 200.0 * q[0, 0] / (q[0, 0] ** 2).sum()
    np.testing.assert_allclose(_decode1(q, K2, V, [n])[0, 0], V[0, 1, 0], rtol=1e-12)
    # empty cache => zeros
    np.testing.assert_array_equal(_decode1(q, K, V, [0])[0, 0], np.zeros(d))


def test_brute_force_python_loops():
    B, Hq, Hkv, d, T = 2, 4, 2, 3, 5
    q, K, V = _f32(B, Hq, d), _f32(B, T, Hkv, d), _f32(B, T, Hkv, d)
    n = [5, 2]
    got = _decode1(q, K, V, n)
    for b in range(B):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            z = [sum(float(q[b, h, c]) * float(K[b, j, g, c]) for c in range(d)) / math.sqrt(d)
                 for j in range(n[b])]
            e = [math.exp(x - max(z)) for x in z]
            for c in range(d):
                want = sum(e[j] / sum(e) * float(V[b, j, g, c]) for j in range(n[b]))
                assert got[b, h, c] == pytest.approx(want, rel=1e-12, abs=1e-15)


@pytest.mark.parametrize("Hq,Hkv,d,T", [(4, 4, 8, 17), (8, 2, 16, 33), (6, 1, 4, 9)])
def test_against_torch_sdpa_fp64(Hq, Hkv, d, T):
    B = 3
    q, K, V = _f32(B, Hq, d), _f32(B, T, Hkv, d), _f32(B, T, Hkv, d)
    n = RNG.integers(1, T + 1, size=B)
    got = _decode1(q, K, V, n)
    for b in range(B):
        kk = torch.from_numpy(K[b, :n[b]]).double().permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        vv = torch.from_numpy(V[b, :n[b]]).double().permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        qq = torch.from_numpy(q[b]).double()[:, None, :]
        want = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv)[:, 0].numpy()
        np.testing.assert_allclose(got[b], want, rtol=1e-10, atol=1e-12)


def test_causal_prefill_against_torch_and_decode():
    B, T_new, Hq, Hkv, d, T = 2, 5, 4, 2, 8, 16
    q, K, V = _f32(B, T_new, Hq, d), _f32(B, T, Hkv, d), _f32(B, T, Hkv, d)
    start = np.array([0, 9], np.int32)
    share = np.zeros(1, np.int32)
    got = orc.shared_attention(0, share, [K], [V], q, start)
    for b in range(B):
        n_tot = start[b] + T_new
        kk = torch.from_numpy(K[b, :n_tot]).double().permute(1, 0, 2).repeat_interleave(2, 0)
        vv = torch.from_numpy(V[b, :n_tot]).double().permute(1, 0, 2).repeat_interleave(2, 0)
        qq = torch.from_numpy(q[b]).double().permute(1, 0, 2)
        mask = torch.arange(n_tot)[None, :] <= (start[b] + torch.arange(T_new))[:, None]
        want = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, attn_mask=mask)
        np.testing.assert_allclose(got[b], want.permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)
        # row i of the prefill is the decode step that sees start+i+1 tokens
        for i in range(T_new):
            dec = orc.decode_attention(0, share, [K[b:b + 1]], [V[b:b + 1]], q[b:b + 1, i],
                                       [start[b] + i + 1])
            np.testing.assert_array_equal(dec[0], got[b, i])


def test_softmax_rows_sum_to_one():
    B, Hq, Hkv, d, T = 2, 4, 2, 16, 40
    q, K, V = _f32(B, Hq, d), _f32(B, T, Hkv, d), _f32(B, T, Hkv, d)
    _, probs = _decode1(q, K, V, [40, 7], return_probs=True)
    np.testing.assert_allclose(probs.sum(-1), 1.0, atol=1e-12)
    assert probs[1, :, 7:].max() == 0.0 and probs.min() >= 0.0


def test_identity_map_is_unshared_and_recipient_reads_donor():
    L, B, Hq, Hkv, d, T = 4, 2, 4, 2, 8, 12
    Ks = [_f32(B, T, Hkv, d) for _ in range(L)]
    Vs = [_f32(B, T, Hkv, d) for _ in range(L)]
    qs = [_f32(B, Hq, d) for _ in range(L)]
    n = np.array([12, 5])
    ident = np.arange(L, dtype=np.int32)
    unshared = [_decode1(qs[l], Ks[l], Vs[l], n) for l in range(L)]
    for l in range(L):
        np.testing.assert_array_equal(orc.decode_attention(l, ident, Ks, Vs, qs[l], n), unshared[l])
    share = np.array([0, 1, 2, 1], np.int32)              # layer 3 reads layer 1
    Ks_s, Vs_s = list(Ks), list(Vs)
    Ks_s[3] = Vs_s[3] = None                              # the recipient stores nothing
    got = orc.decode_attention(3, share, Ks_s, Vs_s, qs[3], n)
    np.testing.assert_array_equal(got, _decode1(qs[3], Ks[1], Vs[1], n))
    assert np.abs(got - unshared[3]).max() > 1e-3         # and it is not layer 3's own cache
    for l in range(3):                                    # the other layers are untouched
        np.testing.assert_array_equal(orc.decode_attention(l, share, Ks_s, Vs_s, qs[l], n), unshared[l])


def test_gqa_head_mapping():
    B, Hkv, d, T, group = 1, 2, 8, 10, 3
    K, V = _f32(B, T, Hkv, d), _f32(B, T, Hkv, d)
    q1 = _f32(B, Hkv, d)
    # duplicated query heads in a group give duplicated outputs; heads map contiguously
    q = np.repeat(q1, group, axis=1)
    out = _decode1(q, K, V, [T])
    mha = _decode1(q1, K, V, [T])                          # group 1 on the same kv heads
    for h in range(Hkv * group):
        np.testing.assert_array_equal(out[0, h], mha[0, h // group])
    # GQA equals MHA over explicitly replicated kv heads
    qr = _f32(B, Hkv * group, d)
    np.testing.assert_array_equal(
        _decode1(qr, K, V, [T]),
        _decode1(qr, np.repeat(K, group, axis=2), np.repeat(V, group, axis=2), [T]))


def test_key_shift_invariance():
    B, Hq, Hkv, d, T = 1, 2, 1, 8, 20
    q, K, V = _f32(B, Hq, d), _f32(B, T, Hkv, d), _f32(B, T, Hkv, d)
    u = _f32(d)
    a = _decode1(q, K, V, [T])
    b = _decode1(q, (K.astype(np.float64) + u).astype(np.float32), V, [T])
    np.testing.assert_allclose(a, b, rtol=1e-5, atol=1e-6)  # fp32 rounding of K+u only


def test_paged_equals_contiguous_bitwise():
    B, Hq, Hkv, d, bs, nblk = 2, 4, 2, 8, 4, 5
    T = bs * nblk
    K, V, q = _f32(B, T, Hkv, d), _f32(B, T, Hkv, d), _f32(B, Hq, d)
    table = RNG.permutation(B * nblk + 3)[:B * nblk].reshape(B, nblk).astype(np.int32)
    Kp = np.full((B * nblk + 3, bs, Hkv, d), np.nan, np.float32)
    Vp = np.full_like(Kp, np.nan)
    for b in range(B):
        for j in range(T):
            Kp[table[b, j // bs], j % bs] = K[b, j]
            Vp[table[b, j // bs], j % bs] = V[b, j]
    n = [T, 7]
    np.testing.assert_array_equal(_decode1(q, K, V, n), _decode1(q, Kp, Vp, n, block_table=table))


def test_bf16_bits_read_exactly():
    B, Hq, Hkv, d, T = 1, 2, 2, 8, 6
    tq, tk, tv = (torch.randn(s, generator=torch.Generator().manual_seed(i)).bfloat16()
                  for i, s in enumerate([(B, Hq, d), (B, T, Hkv, d), (B, T, Hkv, d)]))
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    a = _decode1(bits(tq), bits(tk), bits(tv), [T])
    b = _decode1(tq.float().numpy(), tk.float().numpy(), tv.float().numpy(), [T])
    np.testing.assert_array_equal(a, b)
    assert bits(torch.tensor([1.0, -2.0, 0.5]).bfloat16()).tolist() == [0x3F80, 0xC000, 0x3F00]


def test_append_writes_only_own_cache_layers():
    L, B, Hkv, d, T = 3, 2, 2, 4, 8
    share = np.array([0, 1, 0], np.int32)
    Ks = [np.zeros((B, T, Hkv, d), np.float32), np.zeros((B, T, Hkv, d), np.float32), None]
    Vs = [np.zeros((B, T, Hkv, d), np.float32), np.zeros((B, T, Hkv, d), np.float32), None]
    k, v = _f32(B, 2, Hkv, d), _f32(B, 2, Hkv, d)
    start = np.array([0, 5])
    assert orc.append_kv(0, share, Ks, Vs, k, v, start) is True
    assert orc.append_kv(2, share, Ks, Vs, k, v, start) is False
    np.testing.assert_array_equal(Ks[0][1, 5:7], k[1]); np.testing.assert_array_equal(Vs[0][0, 0:2], v[0])
    assert Ks[0][1, :5].max() == 0 and Ks[1].max() == 0


def test_paged_append_lands_where_the_paged_reader_looks():
    """The append's page addressing (block = table[b][j / block size], row j % block size) is pinned
    against an independent statement of it: rows appended through a permuted table, in several
    calls of ragged sizes that straddle page ends, then attended to through the same table, give
    bitwise the result of the same appends to a plain contiguous cache; blocks no sequence owns
    keep their NaN fill, so a row written to a wrong block would either be missed or poison a result."""
    B, Hq, Hkv, d, bs, nblk = 2, 4, 2, 8, 4, 5
    T = bs * nblk
    share = np.array([0, 0], np.int32)
    table = RNG.permutation(B * nblk + 3)[:B * nblk].reshape(B, nblk).astype(np.int32)
    Kc, Vc = [np.zeros((B, T, Hkv, d), np.float32), None], [np.zeros((B, T, Hkv, d), np.float32), None]
    Kp = [np.full((B * nblk + 3, bs, Hkv, d), np.nan, np.float32), None]
    Vp = [np.full((B * nblk + 3, bs, Hkv, d), np.nan, np.float32), None]
    pos = np.array([0, 0])
    for rows in (3, 6, 1, 7):                                 # 17 of the 20 positions, page ends crossed mid-call
        k, v = _f32(B, rows, Hkv, d), _f32(B, rows, Hkv, d)
        assert orc.append_kv(0, share, Kc, Vc, k, v, pos) is True
        assert orc.append_kv(0, share, Kp, Vp, k, v, pos, block_table=table) is True
        assert orc.append_kv(1, share, Kp, Vp, k, v, pos, block_table=table) is False    # the recipient stores nothing
        pos = pos + rows
    owned = np.zeros(B * nblk + 3, bool)
    owned[table.ravel()] = True
    assert np.isnan(Kp[0][~owned]).all() and np.isnan(Vp[0][~owned]).all()
    q = _f32(B, Hq, d)
    for n in ([17, 17], [16, 5], [1, 13]):
        for layer in (0, 1):
            want = orc.decode_attention(layer, share, Kc, Vc, q, np.asarray(n))
            got = orc.decode_attention(layer, share, Kp, Vp, q, np.asarray(n), block_table=table)
            assert np.isfinite(got).all()
            np.testing.assert_array_equal(got, want)
    # and position by position against the definition of the page table
    for b in range(B):
        for j in range(17):
            np.testing.assert_array_equal(Kp[0][table[b, j // bs], j % bs], Kc[0][b, j])
            np.testing.assert_array_equal(Vp[0][table[b, j // bs], j % bs], Vc[0][b, j])
