"""GPU parity of the decode kernel that shares the launch's pages out by tokens: the workgroups
take equal runs of the line of (kv head, sequence) pages, so a share may begin in the middle of one
sequence, hold several whole ones (each finished and written inside the share) and end in the
middle of another (its parts merged by whoever arrives last).  The cases put the cuts everywhere:
many tiny sequences per share, empty sequences between others, one sequence spread over most of
the grid, page counts on both sides of a multiple of eight, and a step that carries its own token
into sequences of every kind.  Every output vector is held to 5e-3 relative L2 of the fp64 oracle."""
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


def _decode_and_check(kb, case, layer, lens):
    q = case.q(layer)
    got = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens)
    again = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens)
    assert torch.equal(got, again)                       # the merge order is fixed: repeated calls agree bitwise
    want = orc.decode_attention(layer, case.share_map, case.K, case.V, inputs.to_oracle_array(q), lens)
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION, (layer, rel_l2_rows(got, want).max())


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 128), (6, 6, 64), (16, 1, 128)])
def test_many_short_sequences_per_share(kb, dtype, Hq, Hkv, d):
    """64 sequences of 0 to 400 tokens: a share of the line holds several whole sequences, and
    sequences without any key sit between the others."""
    B, cap = 64, 400
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, dtype, cap, share, paged=True, seed=101)
    rng = np.random.default_rng(101 + Hq)
    lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
    lens[[0, 7, 8, 33, 63]] = [0, 0, 0, cap, 0]          # empty ones at both ends and next to each other
    lens[[1, 2, 3, 4, 5]] = [1, 16, 17, 127, 128]        # one token, page ends, the end of an octet of pages
    for layer in (0, 1):
        _decode_and_check(kb, case, layer, lens)
    _decode_and_check(kb, case, 1, np.zeros(B, np.int32))  # nothing anywhere: every row is zero
    one = np.zeros(B, np.int32)
    one[41] = 129
    _decode_and_check(kb, case, 0, one)                  # a single short sequence: most workgroups have no share


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("lens", [[6000, 3, 0, 129], [6000, 6000, 6000, 6000], [1, 1, 1, 5999], [0, 0, 4097, 0],
                                  [1024, 1025, 1023, 1152]])
def test_long_sequences_spread_over_the_grid(kb, dtype, lens):
    """Few (sequence, kv head) pairs and a long context: one sequence's pages are shared among most
    of the grid's workgroups, the short ones fall inside single shares."""
    Hq, Hkv, d, cap = 8, 2, 128, 6000
    share = np.array([0, 1, 0], np.int32)
    case = Case(kb, 3, Hq, Hkv, d, len(lens), dtype, cap, share, paged=True, seed=103)
    for layer in (1, 2):
        _decode_and_check(kb, case, layer, np.asarray(lens, np.int32))


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_step_with_its_own_token_across_shares(kb, dtype):
    """kvs_decode_step over sequences of every kind: the new token is the sequence's only one, falls
    on a page's first and last row, behind a long prefix shared among many workgroups, at the last
    position of the capacity and beyond it (not stored); the store afterwards holds the rows."""
    Hq, Hkv, d, cap = 8, 2, 128, 2048
    lens = np.array([1, 0, 17, 32, 129, 1025, 2047, 2048, 2049, 641, 1, 300], np.int32)
    B = len(lens)
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, dtype, cap, share, paged=True, seed=107)    # every position holds a token already:
    K, V = [case.K[0].copy(), None], [case.V[0].copy(), None]                      # the step's token replaces one
    k_new = inputs.normal((B, 1, Hkv, d), 107, 700)
    v_new = inputs.normal((B, 1, Hkv, d), 107, 701)
    ko, vo = inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new)
    if dtype == "fp8":
        ko, vo = stored_fp8(ko), stored_fp8(vo)
    q = case.q(0)
    got = kb.kvs_decode_step(case.store, 0, q.cuda(), k_new.cuda(), v_new.cuda(), lens).cpu().numpy()
    for b in range(B):
        if 1 <= lens[b] <= cap:
            K[0][b, lens[b] - 1], V[0][b, lens[b] - 1] = ko[b, 0], vo[b, 0]
    want = orc.decode_attention(0, share, K, V, inputs.to_oracle_array(q), np.minimum(lens, cap))
    assert np.isfinite(got).all()
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    # what the step stored is what a later plain call (also through the recipient layer) attends to
    later = kb.kvs_decode_attention(case.store, 1, q.cuda(), np.minimum(lens, cap)).cpu().numpy()
    assert rel_l2_rows(later, want).max() <= REL_L2_ATTENTION
    for b in range(B):
        if 1 <= lens[b] <= cap:
            kk, vv = kb.kvs_gather_kv(case.store, 0, int(lens[b]) - 1, 1, B)
            assert np.array_equal(inputs.to_oracle_array(kk)[b, 0], ko[b, 0]) and np.array_equal(inputs.to_oracle_array(vv)[b, 0], vo[b, 0])


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("n_wg", [2, 5, 40, 3000])
def test_other_grid_sizes(kb, dtype, n_wg):
    """A handful of workgroups (every share holds several sequences and parts of others) and more
    workgroups than the line has octets (single-octet shares, idle workgroups, one sequence merged
    from more than a hundred parts)."""
    Hq, Hkv, d, cap = 8, 2, 128, 9000
    lens = np.array([9000, 4500, 31, 0, 8193], np.int32)
    share = np.array([0, 0], np.int32)
    assert kb.lib().kvs_testing_set_decode_workgroups(n_wg) == kb.KVS_OK
    try:
        case = Case(kb, 2, Hq, Hkv, d, len(lens), dtype, cap, share, paged=True, seed=109)
        _decode_and_check(kb, case, 1, lens)
        _decode_and_check(kb, case, 0, lens[::-1].copy())
    finally:
        assert kb.lib().kvs_testing_set_decode_workgroups(0) == kb.KVS_OK


def test_large_launches_stream_on_three_quarters_of_the_grid(kb):
    """From 24 octets per launched workgroup on, a launch over bf16 pages of 128 channels shares its
    line among three quarters of the workgroups and the rest leave at once (the memory system serves
    fewer streams more evenly): with 64 launched the result is, bit for bit, that of 48, for equal and
    for ragged lengths and for a step that carries its own token; a launch whose shares are whole
    segments keeps all its workgroups."""
    Hq, Hkv, d = 8, 2, 128
    share = np.array([0, 0], np.int32)
    ragged = np.array([16384, 10001, 12800, 15000, 11111, 16000, 13000, 14567], np.int32)
    assert sum((int(n) + 127) // 128 for n in ragged) * Hkv >= 24 * 64
    case = Case(kb, 2, Hq, Hkv, d, 8, "bf16", 16384, share, paged=True, seed=113)
    q = case.q(1)
    outs = {}
    try:
        for n_wg in (64, 48):
            assert kb.lib().kvs_testing_set_decode_workgroups(n_wg) == kb.KVS_OK
            for name, lens in (("equal", np.full(8, 12288, np.int32)), ("ragged", ragged)):
                outs[name, n_wg] = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
                if n_wg == 64:
                    want = orc.decode_attention(1, share, case.K, case.V, inputs.to_oracle_array(q), lens)
                    assert rel_l2_rows(outs[name, n_wg], want).max() <= REL_L2_ATTENTION
        for name in ("equal", "ragged"):
            assert np.array_equal(outs[name, 64], outs[name, 48]), name
        # whole segments per share: 64 (sequence, kv head) segments of 24 octets on 64 workgroups
        assert kb.lib().kvs_testing_set_decode_workgroups(64) == kb.KVS_OK
        whole = Case(kb, 2, 8, 8, d, 8, "bf16", 3072, share, paged=True, seed=127)
        _decode_and_check(kb, whole, 1, np.full(8, 3072, np.int32))
        # a step with its own token on the large ragged launch
        k_new = inputs.normal((8, 1, Hkv, d), 113, 700)
        v_new = inputs.normal((8, 1, Hkv, d), 113, 701)
        K, V = [case.K[0].copy(), None], [case.V[0].copy(), None]
        for b in range(8):
            K[0][b, ragged[b] - 1] = inputs.to_oracle_array(k_new)[b, 0]
            V[0][b, ragged[b] - 1] = inputs.to_oracle_array(v_new)[b, 0]
        got = kb.kvs_decode_step(case.store, 0, q.cuda(), k_new.cuda(), v_new.cuda(), ragged).cpu().numpy()
        want = orc.decode_attention(0, share, K, V, inputs.to_oracle_array(q), ragged)
        assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    finally:
        assert kb.lib().kvs_testing_set_decode_workgroups(0) == kb.KVS_OK
