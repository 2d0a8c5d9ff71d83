"""Oracle of the fused key/value projection + rotary embedding + append (test infrastructure only).

What a layer that keeps its own cache computes before it stores K/V (the paper's "KV cache
computation", Sec. 3.2 / abstract; the host model's ordinary projection):
    k = x . Wk^T,  v = x . Wv^T
    rotary pairs (c, c + d/2) of every key head:  k[c]' = k[c] cos - k[c+d/2] sin,
                                                  k[c+d/2]' = k[c+d/2] cos + k[c] sin
with cos, sin taken from caller-supplied tables at the token's position.  Everything in float64;
the result is returned unrounded (the store rounds it to bf16).
"""
import numpy as np


def _f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def project_kv(x, w_k, w_v, Hkv, d, start_pos, rope_cos=None, rope_sin=None):
    """x [B, T, hidden]; w_k, w_v [Hkv*d, hidden]; returns (k, v) float64 [B, T, Hkv, d]."""
    x, w_k, w_v = _f64(x), _f64(w_k), _f64(w_v)
    B, T, hidden = x.shape
    k = (x.reshape(B * T, hidden) @ w_k.T).reshape(B, T, Hkv, d)
    v = (x.reshape(B * T, hidden) @ w_v.T).reshape(B, T, Hkv, d)
    if rope_cos is not None:
        h = d // 2
        cos, sin = np.asarray(rope_cos, np.float64), np.asarray(rope_sin, np.float64)
        out = np.empty_like(k)
        for b in range(B):
            for i in range(T):
                p = int(start_pos[b]) + i
                lo, hi = k[b, i, :, :h], k[b, i, :, h:]
                out[b, i, :, :h] = lo * cos[p] - hi * sin[p]
                out[b, i, :, h:] = hi * cos[p] + lo * sin[p]
        k = out
    return k, v
