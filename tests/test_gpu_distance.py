"""GPU parity: layer-distance matrix (paper Sec. 3.1.2) vs the fp64 oracle, and the strategy
walk fed from it.  Tolerance: relative Frobenius error of D <= 1e-4 (fp32 accumulation)."""
import numpy as np
import pytest
import torch

from oracle import attention as orc
from oracle import share_map as osm
from paper_2410_18517_amd import inputs
from helpers import REL_DISTANCE

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _compare(kb, kv):
    dK2, dV2, D = (t.cpu().numpy().astype(np.float64) for t in kb.kvs_layer_distance(kv.cuda()))
    oK2, oV2, oD = orc.layer_distance(inputs.to_oracle_array(kv))
    for got, want in ((dK2, oK2), (dV2, oV2), (D, oD)):
        assert np.linalg.norm(got - want) <= REL_DISTANCE * np.linalg.norm(want)
        off = ~np.eye(len(want), dtype=bool)
        assert np.abs(got[off] / want[off] - 1).max() <= 5 * REL_DISTANCE
    assert np.array_equal(D, D.T) and np.all(np.diag(D) == 0)
    return D, oD


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("S,L,Hkv,T,d", [(1, 2, 1, 1, 8), (3, 5, 2, 7, 8), (30, 48, 2, 16, 64), (4, 64, 1, 33, 8),
                                          (2, 7, 1, 300, 8),
                                          # beyond 64 layers (80: the largest model of the paper's appendix): half
                                          # the chunk, up to two pair blocks per thread
                                          (5, 65, 2, 16, 64), (7, 80, 1, 37, 8), (3, 128, 1, 21, 8), (30, 80, 8, 8, 128)])
def test_distance_small(kb, dtype, S, L, Hkv, T, d):
    kv = inputs.calibration_kv(S, L, Hkv, T, d, S * 1000 + L, dtype=dtype)
    _compare(kb, kv)


def test_distance_three_four_five(kb):
    kv = torch.zeros(1, 2, 2, 8)
    kv[0, 1, 0, 0] = 3.0
    kv[0, 1, 1, 5] = -4.0
    dK2, dV2, D = kb.kvs_layer_distance(kv.cuda())
    assert D[0, 1].item() == 5.0 and dK2[0, 1].item() == 9.0 and dV2[1, 0].item() == 16.0


def test_distance_feeds_the_strategy_walk(kb):
    L, C_ = 48, 14
    kv = inputs.calibration_kv(6, L, 2, 32, 64, 77)
    D, oD = _compare(kb, kv)
    got = kb.kvs_build_share_map(D.astype(np.float32), C_)
    want = osm.build_share_map(D.astype(np.float32), L, C_)      # same matrix to both walks
    assert (got[0], got[1].tolist(), got[2].tolist(), got[3], got[4]) == want
    assert got[3] == L - C_
