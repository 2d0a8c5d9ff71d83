"""Pins of the similarity oracle (Sec. 3.1.2): closed forms and torch's fp64 cosine."""
import math

import numpy as np
import torch

from oracle.similarity import avg_cos_sim

RNG = np.random.default_rng(5)


def test_closed_forms():
    a = RNG.standard_normal((4, 50)).astype(np.float32)
    for mode in (0, 1):
        assert abs(avg_cos_sim(a, a, mode) - 1.0) < 1e-12
        assert abs(avg_cos_sim(a, -a, mode) + 1.0) < 1e-12
        assert abs(avg_cos_sim(a, 3.5 * a, mode) - 1.0) < 1e-7          # scale invariance
    x = np.zeros((1, 2), np.float32); y = np.zeros((1, 2), np.float32)
    x[0] = [1, 0]; y[0] = [1, 1]
    assert abs(avg_cos_sim(x, y, 0) - math.cos(math.pi / 4)) < 1e-12      # 45 degrees
    y[0] = [0, 7]
    assert avg_cos_sim(x, y, 0) == 0.0 and avg_cos_sim(x, y, 1) == 0.0     # orthogonal
    assert avg_cos_sim(x, np.zeros_like(x), 0) == 0.0                      # zero vector


def test_the_two_readings_differ_where_they_should():
    # sentences (1,0) and (-1,0) against (1,0) and (1,0): per-sentence cosines are +1 and -1
    # (average 0), while the averaged vectors are (0,0) and (1,0) (cosine defined as 0); a second
    # case: (1,0),(0,1) vs (1,0),(1,0): averaged (.5,.5) vs (1,0) -> cos 45 deg; per sentence 1 and 0
    a = np.array([[1, 0], [0, 1]], np.float32); b = np.array([[1, 0], [1, 0]], np.float32)
    assert abs(avg_cos_sim(a, b, 0) - math.sqrt(0.5)) < 1e-12
    assert abs(avg_cos_sim(a, b, 1) - 0.5) < 1e-12


def test_against_torch_fp64():
    a = RNG.standard_normal((6, 200)).astype(np.float32)
    b = (a + 0.5 * RNG.standard_normal((6, 200))).astype(np.float32)
    ta, tb = torch.from_numpy(a).double(), torch.from_numpy(b).double()
    want0 = torch.nn.functional.cosine_similarity(ta.mean(0), tb.mean(0), dim=0).item()
    want1 = torch.nn.functional.cosine_similarity(ta, tb, dim=1).mean().item()
    assert abs(avg_cos_sim(a, b, 0) - want0) < 1e-12 and abs(avg_cos_sim(a, b, 1) - want1) < 1e-12
    bits = lambda t: torch.from_numpy(t).bfloat16().view(torch.int16).numpy().view(np.uint16)
    vals = lambda t: torch.from_numpy(t).bfloat16().float().numpy()
    assert avg_cos_sim(bits(a), bits(b), 0) == avg_cos_sim(vals(a), vals(b), 0)
