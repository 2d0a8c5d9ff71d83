"""Pins of the projection oracle: torch fp64 linear layers, the rotation's closed forms."""
import numpy as np
import torch

from oracle.projection import project_kv

RNG = np.random.default_rng(3)


def test_projection_is_a_linear_layer():
    B, T, hidden, Hkv, d = 2, 3, 16, 2, 8
    x = RNG.standard_normal((B, T, hidden)).astype(np.float32)
    wk = RNG.standard_normal((Hkv * d, hidden)).astype(np.float32)
    wv = RNG.standard_normal((Hkv * d, hidden)).astype(np.float32)
    k, v = project_kv(x, wk, wv, Hkv, d, [0, 0])
    tk = torch.nn.functional.linear(torch.from_numpy(x).double(), torch.from_numpy(wk).double())
    tv = torch.nn.functional.linear(torch.from_numpy(x).double(), torch.from_numpy(wv).double())
    np.testing.assert_allclose(k.reshape(B, T, -1), tk.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v.reshape(B, T, -1), tv.numpy(), rtol=1e-12, atol=1e-12)


def test_rotation_closed_forms():
    B, T, Hkv, d, hidden = 1, 4, 1, 4, 4
    wk = np.eye(4, dtype=np.float32)                      # k = x
    x = np.zeros((B, T, hidden), np.float32)
    x[0, :, 0] = 1.0                                      # k = (1, 0 | 0, 0): pair (channel 0, channel 2)
    P = 8
    ang = np.outer(np.arange(P), [np.pi / 2, 0.1])        # pair 0 turns a quarter circle per position
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    k, v = project_kv(x, wk, wk, Hkv, d, [1], cos, sin)
    # position 1: (1,0) rotated by 90 degrees -> (0,1): channel 0 -> 0, channel 2 -> 1
    np.testing.assert_allclose(k[0, 0, 0], [0, 0, 1, 0], atol=1e-7)
    np.testing.assert_allclose(k[0, 1, 0], [-1, 0, 0, 0], atol=1e-7)     # position 2: 180 degrees
    np.testing.assert_allclose(v[0, :, 0, 0], 1.0)                       # values are not rotated
    # rotations preserve the norm of every pair and compose additively in the position
    xr = RNG.standard_normal((1, 1, 4)).astype(np.float32)
    k1, _ = project_kv(xr, wk, wk, 1, 4, [3], cos, sin)
    k0, _ = project_kv(xr, wk, wk, 1, 4, [0], cos, sin)
    assert abs(np.hypot(k1[0, 0, 0, 0], k1[0, 0, 0, 2]) - np.hypot(k0[0, 0, 0, 0], k0[0, 0, 0, 2])) < 1e-6
    # relative-position property: <rot_p(a), rot_q(b)> depends on p - q only
    a, b = RNG.standard_normal((1, 1, 4)).astype(np.float32), RNG.standard_normal((1, 1, 4)).astype(np.float32)
    def rot(vec, p): return project_kv(vec, wk, wk, 1, 4, [p], cos, sin)[0][0, 0, 0]
    assert abs(rot(a, 5) @ rot(b, 2) - rot(a, 4) @ rot(b, 1)) < 1e-5
