"""GPU parity of the fp8 (E4M3) slots: storing is compared bit-exactly with the storage oracle
(codes are integers), attention over the stored values with the attention oracle at the usual
tolerance.  The oracle never sees a value that came from the GPU: it rounds the same seeded bf16
rows with its own rule."""
import numpy as np
import pytest
import torch

from oracle import attention as orc
from oracle.fp8 import encode_e4m3
from paper_2410_18517_amd import inputs
from helpers import Case, rel_l2_rows, stored_fp8, REL_L2_ATTENTION

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _bf16_tensor(bits):
    return torch.from_numpy(bits.astype(np.uint16).view(np.int16)).view(torch.bfloat16)


@pytest.mark.parametrize("d", [128, 64])
def test_every_bf16_value_is_stored_as_the_oracle_rounds_it(kb, d):
    """All 65536 bf16 bit patterns (zeros, subnormals, ties, values beyond 448, infinities, NaNs)
    through append and gather, as keys and as values."""
    Hkv, B = 2, 2
    n_rows = 65536 // (Hkv * d)                     # per sequence half of the patterns
    T = n_rows // B
    cap = (T + 15) // 16 * 16
    store = kb.KVStore(np.array([0], np.int32), Hkv, Hkv, d, "fp8", B * cap // 16, cap // 16)
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    rng = np.random.default_rng(9)
    kbits, vbits = rng.permutation(bits).reshape(B, T, Hkv, d), rng.permutation(bits).reshape(B, T, Hkv, d)
    assert kb.kvs_append_kv(store, 0, _bf16_tensor(kbits).cuda(), _bf16_tensor(vbits).cuda(), np.zeros(B, np.int32)) == kb.KVS_OK
    k, v = kb.kvs_gather_kv(store, 0, 0, T, B)
    for got, src in ((inputs.to_oracle_array(k), kbits), (inputs.to_oracle_array(v), vbits)):
        want = stored_fp8(src)
        nan = (want & 0x7fff) > 0x7f80
        assert np.array_equal(got[~nan], want[~nan])
        assert np.all((got[nan] & 0x7fff) > 0x7f80)                  # NaN stays NaN (payload free)
    # and the bytes in the pool are the oracle's codes: look one page up by hand (head 0, page 0)
    pool = store.pool.cpu().numpy()
    page_k = pool[:16 * d]
    t, c = 5, 37
    idx = (((c // 64) * 4 + (c % 32) // 8) * 16 + t) * 16 + ((c // 32) % 2) * 8 + c % 8
    val = (np.array([kbits[0, t, 0, c]], np.uint32) << 16).view(np.float32).astype(np.float64)
    if np.isfinite(val[0]):
        assert page_k[idx] == encode_e4m3(val)[0]


@pytest.mark.parametrize("Hq,Hkv,d,split", [(8, 2, 128, 0), (8, 2, 128, 64), (4, 4, 64, 0), (14, 2, 128, 128)])
def test_decode_over_fp8_slots(kb, Hq, Hkv, d, split):
    L, B, cap = 4, 3, 528
    share = np.array([0, 1, 0, 1], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "fp8", cap, share, paged=True, seed=71)
    assert case.store.pool.numel() == 2 * (B * 33 + 3) * Hkv * 2 * 16 * d      # one byte per element
    lens = np.array([cap, 301, 16], np.int32)
    assert kb.lib().kvs_testing_force_split_tokens(split) == kb.KVS_OK
    try:
        for layer in range(L):
            q = case.q(layer)
            got = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens).cpu().numpy()
            want = orc.decode_attention(layer, share, case.K, case.V, inputs.to_oracle_array(q), lens)
            assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION, layer
    finally:
        assert kb.lib().kvs_testing_force_split_tokens(0) == kb.KVS_OK


def test_decode_step_and_prefill_over_fp8_slots(kb):
    L, Hq, Hkv, d, B, cap, T0 = 2, 8, 2, 128, 2, 160, 100
    share = np.array([0, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "fp8", cap, share, paged=True, seed=72, fill_tokens=T0)
    # a decode step: append one row (quantised on the way in), attend
    k_new, v_new = inputs.normal((B, 1, Hkv, d), 72, 500), inputs.normal((B, 1, Hkv, d), 72, 501)
    pos = np.array([T0, 40], np.int32)
    assert kb.kvs_append_kv(case.store, 1, k_new.cuda(), v_new.cuda(), pos) == kb.KVS_NOOP
    assert kb.kvs_append_kv(case.store, 0, k_new.cuda(), v_new.cuda(), pos) == kb.KVS_OK
    K = np.zeros((B, cap, Hkv, d), np.uint16); V = np.zeros_like(K)
    K[:, :T0], V[:, :T0] = case.K[0], case.V[0]
    for b in range(B):
        K[b, pos[b]] = stored_fp8(inputs.to_oracle_array(k_new))[b, 0]
        V[b, pos[b]] = stored_fp8(inputs.to_oracle_array(v_new))[b, 0]
    q = case.q(1)
    got = kb.kvs_decode_attention(case.store, 1, q.cuda(), pos + 1).cpu().numpy()
    want = orc.decode_attention(1, share, [K, None], [V, None], inputs.to_oracle_array(q), pos + 1)
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    # causal prefill of 37 rows over the same slot
    T_new = 37
    start = np.array([3, 40 - T_new + 1], np.int32)
    qp = case.q(1, rows=T_new)
    got = kb.kvs_prefill_attention(case.store, 1, qp.cuda(), start).cpu().numpy()
    want = orc.shared_attention(1, share, [K, None], [V, None], inputs.to_oracle_array(qp), start)
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION


# Shapes that reach the shared-page prefill kernels over fp8 slots (see test_gpu_attention.py for
# the rule): 8 wavefronts x 2 tiles, 4 wavefronts x 1 tile, both head sizes, one column block per
# head (pages streamed past the caches) and several.
@pytest.mark.parametrize("d,Hq,Hkv,B,T_new", [(128, 16, 8, 16, 150), (128, 8, 8, 32, 128), (128, 16, 8, 16, 100),
                                              (64, 8, 8, 64, 64), (64, 8, 8, 16, 300)])
def test_shared_page_prefill_over_fp8_slots(kb, d, Hq, Hkv, B, T_new):
    L, cap = 2, 416
    share = np.array([0, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "fp8", cap, share, paged=True, seed=73)
    rng = np.random.default_rng(73)
    start = rng.integers(0, cap - T_new + 1, size=B).astype(np.int32)
    start[0], start[-1] = 0, cap - T_new
    q = case.q(1, rows=T_new)
    got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start).cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, B // 2, B - 1):
        want = orc.shared_attention(1, share, [case.K[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                    inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
        assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, b
    # the same rows as a short chunk, which takes the page-splitting kernel: each is within the bar of
    # the oracle (the short chunk is checked against it too), hence within twice the bar of the other
    tail = 8
    short = kb.kvs_prefill_attention(case.store, 1, q[:, -tail:].contiguous().cuda(), start + (T_new - tail)).cpu().numpy()
    b = B - 1
    want = orc.shared_attention(1, share, [case.K[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                inputs.to_oracle_array(q[b:b + 1, -tail:].contiguous()), start[b:b + 1] + (T_new - tail))
    assert rel_l2_rows(short[b:b + 1], want).max() <= REL_L2_ATTENTION
    assert rel_l2_rows(short, got[:, -tail:].astype(np.float64)).max() <= 2 * REL_L2_ATTENTION


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("paged", [True, False])
def test_chunk_appends_at_ragged_positions_store_the_oracle_codes(kb, d, paged):
    """Several rows at once into an fp8 store, starting and ending inside pages (the page-wise append
    writes whole 16-byte pieces where all four tokens of a piece are new and single bytes elsewhere):
    what was written reads back as the oracle rounds it, what was there before is untouched, and the
    one-row append of a decode step lands in the same places."""
    L, Hq, Hkv, B, cap, T0, T = 2, 4, 2, 3, 96, 37, 20
    share = np.array([0, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "fp8", cap, share, paged=paged, seed=41, fill_tokens=T0)
    start = np.array([37, 5, 62], np.int32)                  # continues, overwrites the middle, leaves a gap
    k_new = inputs.normal((B, T, Hkv, d), 41, 500)
    v_new = inputs.normal((B, T, Hkv, d), 41, 501)
    assert kb.kvs_append_kv(case.store, 0, k_new.cuda(), v_new.cuda(), start) == kb.KVS_OK
    Ko = np.zeros((B, cap, Hkv, d), np.uint16); Vo = np.zeros((B, cap, Hkv, d), np.uint16)
    Ko[:, :T0], Vo[:, :T0] = case.K[0], case.V[0]
    for b in range(B):
        Ko[b, start[b]:start[b] + T] = stored_fp8(inputs.to_oracle_array(k_new))[b]
        Vo[b, start[b]:start[b] + T] = stored_fp8(inputs.to_oracle_array(v_new))[b]
    one_k = inputs.normal((B, 1, Hkv, d), 41, 502)
    one_v = inputs.normal((B, 1, Hkv, d), 41, 503)
    at = start + T                                            # one more row behind each chunk
    assert kb.kvs_append_kv(case.store, 0, one_k.cuda(), one_v.cuda(), at) == kb.KVS_OK
    for b in range(B):
        Ko[b, at[b]] = stored_fp8(inputs.to_oracle_array(one_k))[b, 0]
        Vo[b, at[b]] = stored_fp8(inputs.to_oracle_array(one_v))[b, 0]
    for layer in (0, 1):                                      # the recipient reads the same slot
        k, v = kb.kvs_gather_kv(case.store, layer, 0, cap, B)
        k, v = inputs.to_oracle_array(k), inputs.to_oracle_array(v)
        for b in range(B):
            for lo, hi in ((0, T0), (start[b], start[b] + T + 1)):
                assert np.array_equal(k[b, lo:hi], Ko[b, lo:hi]) and np.array_equal(v[b, lo:hi], Vo[b, lo:hi]), (layer, b, lo)
