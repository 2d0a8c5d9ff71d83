"""Oracle of attention over an intra-layer sparsified cache (test infrastructure only).

The paper combines layer sharing with token-dropping methods (H2O, PyramidInfer; "Compatibility
with Intra-layer Compression" and the appendix on their reproduction): every layer that keeps a
cache sparsifies it with the other method's own rule, and a layer that shares reads the already
sparsified cache of its donor.  Which tokens are kept is that other method's business; what the
attention then computes has a plain definition, written out here in float64: for a kv head with
kept token set S,
    out = sum_{t in S} softmax_S(q . k_t / sqrt(d))_t  v_t ,
the softmax being normalised over S only.  The result does not depend on the order of S.
"""
import numpy as np


def _f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def sparse_decode_attention(q, K, V, keep):
    """q [B, Hq, d]; K, V [B, T, Hkv, d] (float or bf16 bit patterns); keep[b][h]: indices of the
    tokens kv head h of sequence b still holds.  Returns float64 [B, Hq, d]; an empty set gives 0."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    B, Hq, d = q.shape
    Hkv = K.shape[2]
    group = Hq // Hkv
    out = np.zeros((B, Hq, d))
    for b in range(B):
        for hq in range(Hq):
            h = hq // group
            S = np.asarray(keep[b][h], dtype=np.int64)
            if S.size == 0:
                continue
            s = K[b, S, h, :] @ q[b, hq] / np.sqrt(d)
            p = np.exp(s - s.max())
            p /= p.sum()
            out[b, hq] = p @ V[b, S, h, :]
    return out


def compact(K, V, keep, capacity=None):
    """The compacted cache: kept tokens of every (sequence, kv head) moved to the front in the order
    of `keep`, the rest zero.  Returns (K', V', counts[B, Hkv])."""
    K, V = np.asarray(K), np.asarray(V)
    B, T, Hkv, d = K.shape
    T2 = T if capacity is None else capacity
    K2, V2 = np.zeros((B, T2, Hkv, d), K.dtype), np.zeros((B, T2, Hkv, d), V.dtype)
    counts = np.zeros((B, Hkv), np.int32)
    for b in range(B):
        for h in range(Hkv):
            S = np.asarray(keep[b][h], dtype=np.int64)
            K2[b, :S.size, h] = K[b, S, h]
            V2[b, :S.size, h] = V[b, S, h]
            counts[b, h] = S.size
    return K2, V2, counts
