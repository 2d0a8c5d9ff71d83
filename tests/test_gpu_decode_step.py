"""GPU parity of the one-launch decode step (append of the step's token + attention) against the
oracle's append followed by its attention, and against the two separate calls."""
import numpy as np
import pytest
import torch

from oracle import attention as orc
from paper_2410_18517_amd import inputs
from helpers import Case, rel_l2_rows, stored_fp8, REL_L2_ATTENTION

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


@pytest.mark.parametrize("dtype,Hq,Hkv,d,split", [("bf16", 8, 2, 128, 0), ("bf16", 8, 2, 128, 64), ("bf16", 12, 4, 64, 0),
                                                  ("bf16", 16, 1, 128, 128), ("f32", 4, 2, 64, 0), ("fp8", 8, 2, 128, 0)])
def test_decode_step_is_append_then_attention(kb, dtype, Hq, Hkv, d, split):
    L, B, cap, T0 = 3, 5, 272, 200
    share = np.array([0, 1, 1], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, dtype, cap, share, paged=True, seed=81, fill_tokens=T0)
    row_dt = case.row_dtype
    # lengths after this step: first token of an empty sequence, a page's first and last row, mid-page, full
    lens = np.array([1, 17, 32, 150, T0 + 1], np.int32)
    K = [None if x is None else np.concatenate([x, np.zeros((B, cap - T0, Hkv, d), x.dtype)], 1) for x in case.K]
    V = [None if x is None else np.concatenate([x, np.zeros((B, cap - T0, Hkv, d), x.dtype)], 1) for x in case.V]
    tol = 1e-5 if dtype == "f32" else REL_L2_ATTENTION
    assert kb.lib().kvs_testing_force_split_tokens(split) == kb.KVS_OK
    try:
        for layer in (1, 2, 0):                                # donor, its recipient, an unrelated layer
            k_new = inputs.normal((B, 1, Hkv, d), 81, layer, 700, dtype=row_dt)
            v_new = inputs.normal((B, 1, Hkv, d), 81, layer, 701, dtype=row_dt)
            q = case.q(layer)
            before = case.store.pool.clone()
            got = kb.kvs_decode_step(case.store, layer, q.cuda(), k_new.cuda(), v_new.cuda(), lens).cpu().numpy()
            ko, vo = inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new)
            if dtype == "fp8":
                ko, vo = stored_fp8(ko), stored_fp8(vo)
            wrote = orc.append_kv(layer, share, K, V, ko, vo, lens - 1)
            assert wrote == (share[layer] == layer)
            if not wrote:
                assert torch.equal(before, case.store.pool)    # a recipient stores nothing
            want = orc.decode_attention(layer, share, K, V, inputs.to_oracle_array(q), lens)
            assert rel_l2_rows(got, want).max() <= tol, layer
            # the store now holds the token: the plain attention call sees the same thing, and the row reads back
            again = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens).cpu().numpy()
            assert rel_l2_rows(again, want).max() <= tol, layer
            donor = int(share[layer])
            for b in range(B):
                kk, vv = kb.kvs_gather_kv(case.store, layer, int(lens[b]) - 1, 1, B)
                assert np.array_equal(inputs.to_oracle_array(kk)[b, 0], K[donor][b, lens[b] - 1])
                assert np.array_equal(inputs.to_oracle_array(vv)[b, 0], V[donor][b, lens[b] - 1])
    finally:
        assert kb.lib().kvs_testing_force_split_tokens(0) == kb.KVS_OK


def test_decode_step_edge_lengths(kb):
    """A length of zero stores nothing and gives a zero row; a length beyond the capacity attends to
    the whole capacity and stores nothing."""
    L, Hq, Hkv, d, B, cap = 1, 4, 2, 128, 3, 48
    case = Case(kb, L, Hq, Hkv, d, B, "bf16", cap, np.array([0], np.int32), paged=True, seed=82, fill_tokens=cap)
    lens = np.array([0, cap + 9, cap], np.int32)
    k_new = inputs.normal((B, 1, Hkv, d), 82, 700)
    v_new = inputs.normal((B, 1, Hkv, d), 82, 701)
    q = case.q(0)
    got = kb.kvs_decode_step(case.store, 0, q.cuda(), k_new.cuda(), v_new.cuda(), lens).cpu().numpy()
    assert np.all(got[0] == 0)
    K, V = [case.K[0].copy()], [case.V[0].copy()]
    K[0][2, cap - 1] = inputs.to_oracle_array(k_new)[2, 0]      # the only position inside the capacity
    V[0][2, cap - 1] = inputs.to_oracle_array(v_new)[2, 0]
    want = orc.decode_attention(0, np.array([0], np.int32), K, V, inputs.to_oracle_array(q), np.minimum(lens, cap))
    assert rel_l2_rows(got[1:], want[1:]).max() <= REL_L2_ATTENTION
    k_after, _ = kb.kvs_gather_kv(case.store, 0, 0, cap, B)
    k_before = inputs.to_oracle_array(k_after)
    assert np.array_equal(k_before[0], case.K[0][0]) and np.array_equal(k_before[1], case.K[0][1])   # nothing stored
    assert np.array_equal(k_before[2, cap - 1], inputs.to_oracle_array(k_new)[2, 0])                    # last slot filled
