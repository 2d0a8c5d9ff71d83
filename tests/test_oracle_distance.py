"""Pins of the layer-distance oracle (paper Sec. 3.1.2, Algorithm 1).

Closed forms, metric axioms and torch.cdist (the library routine the one-sample case reduces
to) fix: mean over samples taken before the distance, keys and values both counted,
Euclidean norm over the whole flattened vector.
"""
import math

import numpy as np
import torch

from oracle import attention as orc
from paper_2410_18517_amd import inputs

RNG = np.random.default_rng(7)


def _kv(S, L, N):
    return RNG.standard_normal((S, L, 2, N)).astype(np.float32)


def test_three_four_five():
    kv = np.zeros((1, 2, 2, 1), np.float32)
    kv[0, 1, 0, 0] = 3.0        # keys differ by 3
    kv[0, 1, 1, 0] = -4.0       # values differ by 4
    dK2, dV2, D = orc.layer_distance(kv)
    assert dK2[0, 1] == 9.0 and dV2[0, 1] == 16.0 and D[0, 1] == 5.0 and D[1, 0] == 5.0
    assert D[0, 0] == 0.0 and D[1, 1] == 0.0


def test_constant_offset_closed_form():
    S, N, c = 3, 50, 0.75
    base = _kv(S, 1, N)
    kv = np.concatenate([base, base + np.float32(c)], axis=1)
    _, _, D = orc.layer_distance(kv)
    assert abs(D[0, 1] - c * math.sqrt(2 * N)) < 1e-5 * D[0, 1]   # fp32 rounding of base + c


def test_mean_over_samples_comes_first():
    # two samples that cancel: the mean cache is zero, so the distance is zero although
    # every per-sample distance is large
    x = _kv(1, 2, 20)
    kv = np.concatenate([x, -x], axis=0)
    _, _, D = orc.layer_distance(kv)
    assert D.max() == 0.0
    # and in general D equals the one-sample distance of the fp64 sample mean
    kv = _kv(5, 4, 30)
    mean = kv.astype(np.float64).mean(0, keepdims=True)
    flat = torch.from_numpy(mean[0].reshape(4, -1))
    np.testing.assert_allclose(orc.layer_distance(kv)[2], torch.cdist(flat, flat).numpy(), rtol=1e-9, atol=1e-12)


def test_one_sample_is_cdist_of_concatenated_kv():
    kv = _kv(1, 6, 40)
    dK2, dV2, D = orc.layer_distance(kv)
    flat = torch.from_numpy(kv[0].reshape(6, -1)).double()
    np.testing.assert_allclose(D, torch.cdist(flat, flat).numpy(), rtol=1e-10, atol=1e-12)
    k = torch.from_numpy(kv[0, :, 0]).double()
    np.testing.assert_allclose(dK2, torch.cdist(k, k).numpy() ** 2, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(D ** 2, dK2 + dV2, rtol=1e-12)


def test_metric_axioms_and_invariances():
    S, L, N = 4, 5, 64
    kv = _kv(S, L, N)
    _, _, D = orc.layer_distance(kv)
    np.testing.assert_array_equal(D, D.T)
    assert np.all(np.diag(D) == 0.0)
    for a in range(L):
        for b in range(L):
            for c in range(L):
                assert D[a, c] <= D[a, b] + D[b, c] + 1e-12
    # homogeneity under an exactly representable scale
    np.testing.assert_allclose(orc.layer_distance(kv * np.float32(-4.0))[2], 4.0 * D, rtol=1e-13)
    # a common permutation of the flattened index changes only the summation order
    p = RNG.permutation(N)
    np.testing.assert_allclose(orc.layer_distance(kv[..., p])[2], D, rtol=1e-12)


def test_structured_noise_free_input_closed_form():
    S, L, Hkv, T, d = 2, 4, 2, 3, 8
    kv = inputs.calibration_kv(S, L, Hkv, T, d, 1, noise=0.0, dtype="f32").numpy()
    # every (kv-head, token) row of a layer repeats the same d-vector r_l = a_l * beta_l
    rows = kv[0].reshape(L, 2, Hkv * T, d)
    assert np.array_equal(rows[:, :, :1].repeat(Hkv * T, 2), rows)
    r = rows[:, :, 0].astype(np.float64)                    # [L, 2, d]
    _, _, D = orc.layer_distance(kv)
    for a in range(L):
        for b in range(L):
            want = math.sqrt(Hkv * T * ((r[a] - r[b]) ** 2).sum())
            assert abs(D[a, b] - want) <= 1e-12 * max(want, 1.0)


def test_bf16_input_read_exactly():
    t = inputs.calibration_kv(3, 3, 1, 4, 8, 2)
    assert t.dtype == torch.bfloat16
    a = orc.layer_distance(inputs.to_oracle_array(t))[2]
    b = orc.layer_distance(t.float().numpy())[2]
    np.testing.assert_array_equal(a, b)
