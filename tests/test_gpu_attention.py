"""GPU parity: decode and causal-prefill attention over the shared store vs the fp64 oracle.

Tolerance (both stores): every output vector within 5e-3 relative L2 of the oracle; fp32 stores
are held to 1e-5.  Edge cases: empty, one-token, page-boundary and ragged lengths, one and many
context splits, recipients (incl. the last layer), donors with several recipients."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import attention as orc
from paper_2410_18517_amd import inputs
from helpers import Case, rel_l2_rows, REL_L2_ATTENTION

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    yield binding
    binding.kvs_testing_force_split_tokens(0)


def _check_decode(kb, case, layers, seq_lens, tol):
    seq_lens = np.asarray(seq_lens, np.int32)
    worst = 0.0
    for layer in layers:
        q = case.q(layer)
        got = kb.kvs_decode_attention(case.store, layer, q.cuda(), seq_lens).cpu().numpy()
        want = orc.decode_attention(layer, case.share_map, case.K, case.V, inputs.to_oracle_array(q), seq_lens)
        assert np.isfinite(got).all()
        err = rel_l2_rows(got, want)
        worst = max(worst, err.max())
        assert err.max() <= tol, (layer, err.max())
    return worst


def test_tiny_config_fp32(kb):
    """4 layers, 4 query / 2 kv heads, d 64, one sequence of 128 tokens, fp32, layer 3 reads layer 1."""
    w = inputs.WORKLOADS["tiny"]
    share = inputs.make_share_map(w.L, w.n_shared, fixed=w.fixed_map)
    for paged in (True, False):
        case = Case(kb, w.L, w.Hq, w.Hkv, w.d, w.B, "f32", w.context, share, paged=paged, seed=1)
        assert case.store.desc.n_slots == 3
        _check_decode(kb, case, range(w.L), [w.context], 1e-5)
        # the recipient's output is attention over the donor's cache, not a cache of its own
        q3 = case.q(3)
        got = kb.kvs_decode_attention(case.store, 3, q3.cuda(), np.array([128], np.int32)).cpu().numpy()
        ident = np.arange(4, dtype=np.int32)
        want = orc.decode_attention(1, ident, case.K, case.V, inputs.to_oracle_array(q3), [128])
        assert rel_l2_rows(got, want).max() <= 1e-5


@pytest.mark.parametrize("d", [64, 128])
def test_fp32_ragged_and_gqa(kb, d):
    share = np.array([0, 0, 2, 2, 0], np.int32)               # layer 0 serves two recipients
    case = Case(kb, 5, 6, 2, d, 4, "f32", 150, share, seed=5)
    _check_decode(kb, case, range(5), [150, 0, 1, 77], 1e-5)


@pytest.mark.parametrize("Hq,Hkv,d", [(4, 4, 128), (8, 2, 128), (12, 2, 128), (16, 1, 128), (6, 2, 64), (5, 5, 64)])
def test_bf16_decode_shapes(kb, Hq, Hkv, d):
    L = 6
    share = np.array([0, 1, 0, 3, 1, 3], np.int32)            # last layer is a recipient
    case = Case(kb, L, Hq, Hkv, d, 3, "bf16", 400, share, seed=Hq * 10 + Hkv)
    _check_decode(kb, case, range(L), [400, 123, 257], REL_L2_ATTENTION)


@pytest.mark.parametrize("split_tokens", [0, 64, 128, 512])
def test_bf16_edge_lengths_and_splits(kb, split_tokens):
    kb.kvs_testing_force_split_tokens(split_tokens)
    try:
        share = np.array([0, 1, 1], np.int32)
        lens = [0, 1, 15, 16, 17, 63, 64, 65, 300, 333]
        case = Case(kb, 3, 8, 2, 128, len(lens), "bf16", 333, share, seed=21)
        _check_decode(kb, case, range(3), lens, REL_L2_ATTENTION)
        # lengths above the capacity are clamped to it
        q = case.q(0)
        a = kb.kvs_decode_attention(case.store, 0, q.cuda(), np.full(len(lens), 10 ** 6, np.int32))
        b = kb.kvs_decode_attention(case.store, 0, q.cuda(), np.full(len(lens), 336, np.int32))
        assert torch.equal(a, b)
    finally:
        kb.kvs_testing_force_split_tokens(0)


def test_many_splits_merge_is_exact_and_repeatable(kb):
    """128 splits per (sequence, kv head): the merge by the last-arriving workgroup must see every
    split's state.  The merge order is fixed, so repeated calls agree bit for bit."""
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, 8, 2, 128, 6, "bf16", 8192, share, seed=17)
    lens = np.array([8192, 8000, 4097, 64, 1, 0], np.int32)
    try:
        kb.kvs_testing_force_split_tokens(64)
        q = case.q(1)
        want = orc.decode_attention(1, share, case.K, case.V, inputs.to_oracle_array(q), lens)
        first = None
        for _ in range(25):
            got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens)
            first = got.clone() if first is None else first
            assert torch.equal(got, first)
        assert rel_l2_rows(first.cpu().numpy(), want).max() <= REL_L2_ATTENTION
        kb.kvs_testing_force_split_tokens(8192)                                    # one split: no merge at all
        single = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
        assert rel_l2_rows(single, want).max() <= REL_L2_ATTENTION
    finally:
        kb.kvs_testing_force_split_tokens(0)


# A decode launch sizes its context splits by the lengths it finds on the device: a batch far below
# the store's capacity, one long sequence among short ones, and a wide spread (with an empty
# sequence, a one-token one and a full one) each move the splits away from where the host's choice
# for full sequences would put them.  The plain call, the per-head lengths of a sparsified slot
# (each head of a sequence its own length) and the one-launch decode step all take that path.
@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("kind", ["spread", "short", "one_long", "long_last"])
@pytest.mark.parametrize("Hq,Hkv,B", [(16, 8, 16), (4, 2, 40)])      # up to 16 sequences: lengths read out of the lanes
def test_decode_splits_follow_the_lengths(kb, dtype, kind, Hq, Hkv, B):
    L, d, cap = 2, 128, 2048
    share = np.array([0, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, dtype, cap, share, paged=True, seed=97)
    rng = np.random.default_rng(97)
    if kind == "spread":
        lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
        lens[:4] = [cap, 0, 1, 16]
    elif kind == "short":
        lens = rng.integers(480, 520, size=B).astype(np.int32)
    else:
        lens = np.full(B, 40, np.int32)
        lens[5 if kind == "one_long" else B - 1] = cap
    q = case.q(1)
    qo = inputs.to_oracle_array(q)
    for _ in range(2):                                             # twice: counters are left at zero
        got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
        want = orc.decode_attention(1, share, case.K, case.V, qo, lens)
        assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    # per-head lengths: head g of sequence b keeps the first head_lens[b, g] tokens
    head_lens = np.stack([np.roll(lens, g) for g in range(Hkv)], axis=1).astype(np.int32)      # [B, Hkv]
    got = kb.kvs_decode_attention_per_head(case.store, 1, q.cuda(), head_lens[None]).cpu().numpy()
    group = Hq // Hkv
    for g in range(Hkv):
        want = orc.decode_attention(1, share, case.K, case.V, qo, head_lens[:, g])
        assert rel_l2_rows(got[:, g * group:(g + 1) * group], want[:, g * group:(g + 1) * group]).max() <= REL_L2_ATTENTION, g
    # the decode step that stores its own token (lengths count it, so at least one)
    step_lens = np.maximum(lens, 1)
    row_dt = case.row_dtype
    k_new = inputs.normal((B, 1, Hkv, d), 97, 700, dtype=row_dt)
    v_new = inputs.normal((B, 1, Hkv, d), 97, 701, dtype=row_dt)
    got = kb.kvs_decode_step(case.store, 0, q.cuda(), k_new.cuda(), v_new.cuda(), step_lens).cpu().numpy()
    ko, vo = inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new)
    if dtype == "fp8":
        from helpers import stored_fp8
        ko, vo = stored_fp8(ko), stored_fp8(vo)
    assert orc.append_kv(0, share, case.K, case.V, ko, vo, step_lens - 1)
    want = orc.decode_attention(0, share, case.K, case.V, qo, step_lens)
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION


# More than 64 sequences take the split kernel (the token-shared one keeps one sequence per lane): a
# ragged batch with empty and full sequences, the plain call twice on one workspace and the decode
# step that stores its own token.
@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,Hkv,B,cap", [(12, 2, 65, 700), (8, 8, 128, 300), (6, 1, 300, 130)])
def test_decode_more_than_64_sequences(kb, dtype, Hq, Hkv, B, cap):
    d = 128
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, dtype, cap, share, paged=True, seed=113)
    rng = np.random.default_rng(113)
    lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
    lens[:5] = [cap, 0, 1, 16, 17]
    q = case.q(1)
    qo = inputs.to_oracle_array(q)
    want = orc.decode_attention(1, share, case.K, case.V, qo, lens)
    for _ in range(2):
        got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
        assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    step_lens = np.maximum(lens, 1)
    k_new = inputs.normal((B, 1, Hkv, d), 113, 700, dtype=case.row_dtype)
    v_new = inputs.normal((B, 1, Hkv, d), 113, 701, dtype=case.row_dtype)
    got = kb.kvs_decode_step(case.store, 0, q.cuda(), k_new.cuda(), v_new.cuda(), step_lens).cpu().numpy()
    ko, vo = inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new)
    if dtype == "fp8":
        from helpers import stored_fp8
        ko, vo = stored_fp8(ko), stored_fp8(vo)
    assert orc.append_kv(0, share, case.K, case.V, ko, vo, step_lens - 1)
    want = orc.decode_attention(0, share, case.K, case.V, qo, step_lens)
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    # the rows the step stored are what a later call reads
    again = kb.kvs_decode_attention(case.store, 1, q.cuda(), step_lens).cpu().numpy()
    assert rel_l2_rows(again, want).max() <= REL_L2_ATTENTION


# Seeded random shapes and length patterns through the plain decode call: batch sizes on either side
# of 16 and 64 (how a launch reads the lengths), capacities off a multiple of the split sizes,
# contiguous and paged stores.
def test_randomised_decode_lengths(kb):
    rng = np.random.default_rng(20241018)
    for case_i in range(16):
        Hkv = int(rng.choice([1, 2, 4, 8]))
        group = int(rng.choice([1, 2, 4, 6]))
        d = int(rng.choice([64, 128]))
        B = int(rng.choice([1, 3, 16, 17, 64, 70]))
        cap = int(rng.choice([512, 1024, 2048])) + int(rng.choice([0, 16, 48]))
        dtype = str(rng.choice(["bf16", "fp8"]))
        kind = str(rng.choice(["uniform", "spread", "one_long", "zeros"]))
        if kind == "uniform":
            lens = np.full(B, rng.integers(1, cap + 1))
        elif kind == "spread":
            lens = rng.integers(0, cap + 1, size=B)
        elif kind == "one_long":
            lens = rng.integers(0, 64, size=B)
            lens[rng.integers(0, B)] = cap
        else:
            lens = np.zeros(B, np.int64)
            lens[rng.integers(0, B)] = rng.integers(0, cap + 1)
        lens = lens.astype(np.int32)
        share = np.array([0, 0], np.int32)
        case = Case(kb, 2, Hkv * group, Hkv, d, B, dtype, cap, share, paged=bool(rng.integers(0, 2)), seed=300 + case_i)
        q = case.q(1)
        got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
        want = orc.decode_attention(1, share, case.K, case.V, inputs.to_oracle_array(q), lens)
        assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION, (case_i, Hkv, group, d, B, cap, dtype, kind)
        del case


@pytest.mark.parametrize("gain", [0.05, 4.0, 24.0])
def test_bf16_flat_and_peaked_softmax(kb, gain):
    """Scores from nearly constant to widely spread (the running reference of the exponentials has
    to move many times, by small and by large steps), keys sorted so that the maximum keeps rising."""
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, 8, 2, 128, 3, "bf16", 1500, share, seed=23)
    lens = np.array([1500, 700, 33], np.int32)
    q = (case.q(1).float() * gain).to(torch.bfloat16)
    for split in (0, 256):
        kb.kvs_testing_force_split_tokens(split)
        got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
        want = orc.decode_attention(1, share, case.K, case.V, inputs.to_oracle_array(q), lens)
        assert np.isfinite(got).all()
        assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION, (gain, split)
    kb.kvs_testing_force_split_tokens(0)
    # rising scores: key j is a growing multiple of q's direction for head 0 of sequence 0
    k_up = torch.from_numpy(case.K[0].view(np.int16)).view(torch.bfloat16).clone()
    ramp = torch.linspace(-1.0, 1.0, 1500).view(1, 1500, 1, 1)
    k_up = (k_up.float() * 0.1 + ramp * q[:1, :1].float().reshape(1, 1, 1, 128)).to(torch.bfloat16)
    v = torch.from_numpy(case.V[0].view(np.int16)).view(torch.bfloat16)
    kb.kvs_append_kv(case.store, 0, k_up.expand(3, -1, 2, -1).contiguous().cuda(), v.contiguous().cuda(),
                     np.zeros(3, np.int32))
    Ko = [inputs.to_oracle_array(k_up.expand(3, -1, 2, -1).contiguous()), None]
    got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens).cpu().numpy()
    want = orc.decode_attention(1, share, Ko, case.V, inputs.to_oracle_array(q), lens)
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION


def test_bf16_unwritten_tail_cannot_leak(kb):
    """Rows past seq_len hold NaN bit patterns: they must not reach the output."""
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, 4, 2, 128, 2, "bf16", 64, share, seed=8, fill_tokens=64)
    junk = torch.full((2, 64, 2, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    kb.kvs_append_kv(case.store, 0, junk[:, :43].contiguous(), junk[:, :43].contiguous(), np.array([21, 21], np.int32))
    case.K[0] = np.ascontiguousarray(case.K[0][:, :21]); case.V[0] = np.ascontiguousarray(case.V[0][:, :21])
    _check_decode(kb, case, [0, 1], [21, 9], REL_L2_ATTENTION)


def test_decode_step_order_recipient_sees_current_token(kb):
    """One whole decode step: layers in order, own-cache layers append then attend, recipients
    attend to a donor that already holds this step's token."""
    L, Hq, Hkv, d, B = 5, 8, 2, 128, 3
    share = np.array([0, 1, 0, 1, 4], np.int32)
    lens0 = np.array([40, 7, 16], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "bf16", 48, share, seed=31, fill_tokens=40)
    Ko = [None if x is None else np.concatenate([x, np.zeros((B, 8, Hkv, d), x.dtype)], 1) for x in case.K]
    Vo = [None if x is None else np.concatenate([x, np.zeros((B, 8, Hkv, d), x.dtype)], 1) for x in case.V]
    for step in range(2):
        lens = lens0 + step + 1
        for layer in range(L):
            k_new = inputs.normal((B, 1, Hkv, d), 31, layer, step, 70)
            v_new = inputs.normal((B, 1, Hkv, d), 31, layer, step, 71)
            st = kb.kvs_append_kv(case.store, layer, k_new.cuda(), v_new.cuda(), lens - 1)
            wrote = orc.append_kv(layer, share, Ko, Vo, inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new), lens - 1)
            assert (st == kb.KVS_OK) == wrote and (st == kb.KVS_NOOP) == (share[layer] != layer)
            q = inputs.normal((B, Hq, d), 31, layer, step, 72)
            got = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens).cpu().numpy()
            want = orc.decode_attention(layer, share, Ko, Vo, inputs.to_oracle_array(q), lens)
            assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION


@pytest.mark.parametrize("dtype,Hq,Hkv,d,T_new", [("bf16", 4, 4, 128, 64), ("bf16", 8, 2, 128, 21),
                                                  ("bf16", 6, 1, 64, 33), ("f32", 4, 2, 64, 9)])
def test_causal_prefill(kb, dtype, Hq, Hkv, d, T_new):
    L, B, cap = 3, 3, 200
    share = np.array([0, 0, 2], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, dtype, cap, share, seed=41)
    tol = 1e-5 if dtype == "f32" else REL_L2_ATTENTION
    for start in ([0, 0, 0], [cap - T_new, 5, 100]):
        start = np.asarray(start, np.int32)
        for layer in range(L):
            q = case.q(layer, rows=T_new)
            got = kb.kvs_prefill_attention(case.store, layer, q.cuda(), start).cpu().numpy()
            want = orc.shared_attention(layer, share, case.K, case.V, inputs.to_oracle_array(q), start)
            assert np.isfinite(got).all()
            assert rel_l2_rows(got, want).max() <= tol, (layer, start)
    # The last prefill row is what the following decode step computes (the oracle's pins include that
    # identity): both calls are held to the oracle's decode result, each at the oracle tolerance.
    # (The two GPU results are not compared with each other: two values within tol of a third are
    # only within 2 tol of each other, and nothing in the method asks for more.)
    q = case.q(0, rows=T_new)
    begin = np.array([10, 20, 30], np.int32)
    pre = kb.kvs_prefill_attention(case.store, 0, q.cuda(), begin).cpu().numpy()
    dec = kb.kvs_decode_attention(case.store, 0, q[:, -1].contiguous().cuda(), begin + T_new).cpu().numpy()
    want = orc.decode_attention(0, share, case.K, case.V, inputs.to_oracle_array(q[:, -1].contiguous()), begin + T_new)
    assert rel_l2_rows(dec, want).max() <= tol
    assert rel_l2_rows(pre[:, -1], want).max() <= tol


# Shapes that reach each instantiation of the shared-page prefill kernel (a workgroup's wavefronts
# take separate columns and read every page pair from LDS): 256 columns per workgroup when one
# (sequence, kv head) has more than 128 query columns (rows x group size), 128 for 65 to 128, 64
# for exactly 64 (test_prefill_kernel_boundaries walks the limits); with few sequences x heads the
# context is split over workgroups as well (test_causal_prefill's small batches).  Ragged column counts, a group size of two,
# different start positions per sequence, a permuted page table, a recipient layer.
@pytest.mark.parametrize("d,Hq,Hkv,B,T_new", [(128, 16, 8, 16, 150),     # 300 columns -> 2 x 256-column workgroups, 8 wavefronts
                                              (128, 16, 8, 16, 100),     # 200 columns -> one 256-column workgroup, a quarter of it idle
                                              (64, 8, 8, 16, 300),       # head size 64, one query head per kv head
                                              (64, 16, 8, 16, 100)])
def test_shared_page_prefill_kernels(kb, d, Hq, Hkv, B, T_new):
    L, cap = 2, 416
    share = np.array([0, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=47)
    rng = np.random.default_rng(47)
    start = rng.integers(0, cap - T_new + 1, size=B).astype(np.int32)
    start[0], start[-1] = 0, cap - T_new
    q = case.q(1, rows=T_new)
    got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start).cpu().numpy()
    assert np.isfinite(got).all()
    # the same rows as a short chunk take the page-splitting kernel: both kernels are held to the
    # oracle (not to each other: two results within tol of a third are only within 2 tol of each other)
    tail = 8
    short = kb.kvs_prefill_attention(case.store, 1, q[:, -tail:].contiguous().cuda(), start + (T_new - tail)).cpu().numpy()
    assert np.isfinite(short).all()
    for b in (0, B // 2, B - 1):
        want = orc.shared_attention(1, share, [case.K[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                    inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
        assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, b
        assert rel_l2_rows(short[b:b + 1], want[:, -tail:]).max() <= REL_L2_ATTENTION, b


# Four or more 256-column blocks per (sequence, kv head): a workgroup takes the k-th longest and then
# the k-th shortest block (an odd number leaves the middle block to a workgroup of its own), three
# blocks keep one workgroup per block.  Ragged last block, a group size of two, different starts.
@pytest.mark.parametrize("Hq,Hkv,B,T_new", [(8, 8, 8, 800),        # 4 blocks, the last one with 32 columns
                                            (8, 8, 8, 1100),       # 5 blocks: two pairs and the middle block
                                            (16, 8, 6, 850),       # group 2: 1700 columns, 7 blocks
                                            (8, 8, 16, 700)])      # 3 blocks: one workgroup each
def test_prefill_many_column_blocks(kb, Hq, Hkv, B, T_new):
    d, L = 128, 2
    cap = T_new + 120
    share = np.array([0, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=53)
    rng = np.random.default_rng(53)
    start = rng.integers(0, cap - T_new + 1, size=B).astype(np.int32)
    start[0], start[-1] = 0, cap - T_new
    q = case.q(1, rows=T_new)
    got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start).cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, B // 2, B - 1):
        want = orc.shared_attention(1, share, [case.K[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                    inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
        assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, b


# Few (sequence, kv head) pairs: the shared-page kernels split the context over workgroups too, and
# the last workgroup of a column block to arrive merges the states.  By the host's own choice at a
# long context, and with a forced split of 4 or 8 pages at a short one; start positions that leave
# the later splits of a sequence without any visible key, or cut a split in the middle.
@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,Hkv,B,T_new,cap,split_tokens", [(8, 2, 3, 16, 2048, 0),      # 64 columns, 8 splits
                                                             (8, 2, 3, 30, 2048, 0),      # 120 columns -> the 128-column shape
                                                             (16, 2, 3, 40, 2048, 0),     # 320 columns -> 2 blocks of 256
                                                             (8, 2, 3, 16, 416, 64),      # 7 splits of 2 page pairs
                                                             (8, 1, 2, 31, 416, 128),     # 248 columns, 4 splits of 4 pairs
                                                             (4, 4, 3, 97, 416, 64)])     # one head per group, 128-column shape
def test_shared_page_prefill_with_context_splits(kb, dtype, Hq, Hkv, B, T_new, cap, split_tokens):
    d = 128
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, dtype, cap, share, paged=True, seed=67)
    start = np.array([0, cap // 3 + 5, cap - T_new][:B], np.int32)
    start[-1] = cap - T_new
    q = case.q(1, rows=T_new)
    assert kb.lib().kvs_testing_force_split_tokens(split_tokens) == kb.KVS_OK
    try:
        for _ in range(2):                                         # twice: the counters must be left at zero
            got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start).cpu().numpy()
            want = orc.shared_attention(1, share, [case.K[0], None], [case.V[0], None], inputs.to_oracle_array(q), start)
            assert np.isfinite(got).all()
            assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION
    finally:
        assert kb.lib().kvs_testing_force_split_tokens(0) == kb.KVS_OK


# A workspace sized for up to 33 rows must serve a call of 32: with 64 (sequence, kv head) pairs, 33
# rows x 4 heads take the 256-column shape with 4 context splits, 32 rows the 128-column shape with
# 8, which needs more partial states than either end of the range.
def test_workspace_for_a_row_range_serves_every_row_count(kb):
    Hq, Hkv, B, cap, d = 32, 8, 8, 2048, 128
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=71)
    need = kb.lib().kvs_workspace_bytes(C.byref(case.store.desc), B, 33)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    start = np.full(B, cap - 64, np.int32)
    for T_new in (33, 32, 16, 1):
        q = case.q(1, rows=T_new)
        got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start, workspace=ws).cpu().numpy()
        for b in (0, B - 1):
            want = orc.shared_attention(1, share, [case.K[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                        inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
            assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, (T_new, b)


# Column counts on either side of the limits at which the prefill kernels change hands (64, 128 and
# 256 columns per (sequence, kv head)): a last column block of a single column leaves wavefronts
# without any column.
@pytest.mark.parametrize("Hq,Hkv,B,T_new", [(8, 8, 64, 63), (8, 8, 64, 64), (8, 8, 64, 65), (8, 8, 64, 128), (8, 8, 64, 129),
                                            (16, 8, 32, 127), (16, 8, 32, 128), (16, 8, 32, 129)])
def test_prefill_kernel_boundaries(kb, Hq, Hkv, B, T_new):
    d, cap = 128, 208
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=57)
    rng = np.random.default_rng(57)
    start = rng.integers(0, cap - T_new + 1, size=B).astype(np.int32)
    start[0], start[-1] = 0, cap - T_new
    q = case.q(1, rows=T_new)
    got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start).cpu().numpy()
    assert np.isfinite(got).all()
    for b in (0, B // 3, B - 1):
        want = orc.shared_attention(1, share, [case.K[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                    inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
        assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, b


@pytest.mark.parametrize("Hq,Hkv,B,T_new", [(16, 8, 16, 160),      # 320 columns: the 8-wavefront shared-page kernel
                                            (8, 8, 64, 80)])       # 80 columns: the 4-wavefront one
def test_shared_page_prefill_rising_scores(kb, Hq, Hkv, B, T_new):
    """Keys that grow along the context in the direction of the queries: in the shared-page kernels
    the reference of the exponentials then moves again and again (the accumulators are rescaled on
    most page pairs), by steps from small to large, up to the causal edge of every row."""
    d, cap = 128, 400
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=53)
    rng = np.random.default_rng(53)
    start = rng.integers(0, cap - T_new + 1, size=B).astype(np.int32)
    start[0], start[-1] = 0, cap - T_new
    u = inputs.normal((1, 1, 1, d), 53, 777).float()
    u = u / u.norm()
    for gain in (3.0, 40.0):
        ramp = torch.linspace(0.0, 1.0, cap).view(1, cap, 1, 1)
        k = torch.from_numpy(case.K[0].view(np.int16)).view(torch.bfloat16).float() * 0.05 + gain * ramp * u
        k = k.to(torch.bfloat16).contiguous()
        v = torch.from_numpy(case.V[0].view(np.int16)).view(torch.bfloat16).contiguous()
        assert kb.kvs_append_kv(case.store, 0, k.cuda(), v.cuda(), np.zeros(B, np.int32)) == kb.KVS_OK
        q = (inputs.normal((B, T_new, Hq, d), 53, 778).float() * 0.05 + 4.0 * u.view(1, 1, 1, d)).to(torch.bfloat16)
        got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start).cpu().numpy()
        assert np.isfinite(got).all()
        Ko = [inputs.to_oracle_array(k), None]
        for b in (0, B // 2, B - 1):
            want = orc.shared_attention(1, share, [Ko[0][b:b + 1], None], [case.V[0][b:b + 1], None],
                                        inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
            assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, (gain, b)


def test_deep_model_layers_beyond_the_first_look_up(kb):
    """80 layers (the paper's largest model): the kernel's first look-up carries the slots of layers
    0..55 only, so a layer whose donor lies beyond them resolves its slot with a second look-up."""
    L, Hq, Hkv, d, B, cap = 80, 16, 2, 128, 2, 80
    share = np.arange(L, dtype=np.int32)
    share[79], share[70], share[57] = 60, 3, 56
    for dtype in ("bf16", "fp8", "f32"):
        case = Case(kb, L, Hq if dtype != "f32" else 4, Hkv, d if dtype != "f32" else 64, B, dtype, cap, share, seed=61,
                    fill_layers=[3, 56, 60, 78])
        lens = np.array([cap, 37], np.int32)
        tol = 1e-5 if dtype == "f32" else REL_L2_ATTENTION
        for layer in (79, 70, 57, 78, 60, 3):
            q = case.q(layer)
            got = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens).cpu().numpy()
            want = orc.decode_attention(layer, share, case.K, case.V, inputs.to_oracle_array(q), lens)
            assert rel_l2_rows(got, want).max() <= tol, (dtype, layer)
        q = case.q(79, rows=20)
        start = np.array([cap - 20, 3], np.int32)
        got = kb.kvs_prefill_attention(case.store, 79, q.cuda(), start).cpu().numpy()
        want = orc.shared_attention(79, share, case.K, case.V, inputs.to_oracle_array(q), start)
        assert rel_l2_rows(got, want).max() <= tol, (dtype, "prefill")


def test_randomised_shapes_maps_and_lengths(kb):
    """Seeded sweep over store types, head groupings, batch sizes, sharing maps, paging, split sizes
    and ragged lengths; every case is compared element by element with the oracle."""
    rng = np.random.default_rng(20241018)
    try:
        for case_id in range(24):
            dtype = "bf16" if case_id % 4 else "f32"
            d = int(rng.choice([64, 128]))
            Hkv = int(rng.choice([1, 2, 3, 8]))
            group = int(rng.choice([1, 2, 4, 7, 16] if dtype == "bf16" else [1, 3]))
            L = int(rng.integers(2, 7))
            B = int(rng.integers(1, 9))
            cap = int(rng.choice([40, 130, 517, 1200]))
            share = inputs.make_share_map(L, int(rng.integers(0, L)), 900 + case_id)
            case = Case(kb, L, Hkv * group, Hkv, d, B, dtype, cap, share, paged=bool(rng.integers(0, 2)),
                        seed=900 + case_id)
            lens = rng.integers(0, cap + 1, size=B).astype(np.int32)
            lens[rng.integers(0, B)] = cap
            kb.kvs_testing_force_split_tokens(int(rng.choice([0, 64, 256, 1024])))
            tol = 1e-5 if dtype == "f32" else REL_L2_ATTENTION
            for layer in rng.choice(L, size=min(L, 3), replace=False):
                q = case.q(int(layer))
                got = kb.kvs_decode_attention(case.store, int(layer), q.cuda(), lens).cpu().numpy()
                want = orc.decode_attention(int(layer), share, case.K, case.V, inputs.to_oracle_array(q), lens)
                assert np.isfinite(got).all()
                assert rel_l2_rows(got, want).max() <= tol, (case_id, dtype, d, Hkv, group, L, B, cap, int(layer))
            T_new = int(rng.integers(2, min(cap, 70)))
            start = rng.integers(0, cap - T_new + 1, size=B).astype(np.int32)
            layer = int(rng.integers(0, L))
            q = case.q(layer, rows=T_new)
            got = kb.kvs_prefill_attention(case.store, layer, q.cuda(), start).cpu().numpy()
            want = orc.shared_attention(layer, share, case.K, case.V, inputs.to_oracle_array(q), start)
            assert rel_l2_rows(got, want).max() <= tol, (case_id, "prefill", T_new)
    finally:
        kb.kvs_testing_force_split_tokens(0)
