"""GPU parity of the fused K/V projection + rotary embedding + append against the fp64 oracle.

The store holds bf16: a stored element must equal the oracle's exact value rounded to bf16, up to
the fp32 accumulation error of the contraction, i.e. within one bf16 unit (2^-8 relative, with a
small absolute floor for elements near zero).  Layers that read a donor's cache do nothing."""
import numpy as np
import pytest
import torch

from oracle import attention as orc
from oracle.projection import project_kv
from paper_2410_18517_amd import inputs
from helpers import rel_l2_rows, REL_L2_ATTENTION

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _rope_tables(positions, d, base=10000.0):
    inv = base ** (-np.arange(d // 2, dtype=np.float64) * 2.0 / d)
    ang = np.outer(np.arange(positions, dtype=np.float64), inv)
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def _bf16_round(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16)


# Up to 32 rows take the streaming kernel, more the tiled one.  Shapes 5-8 split the streaming
# kernel's contraction over 4, 4, 3 and 8 workgroups per output tile (the merge path), shapes 9-11
# the tiled kernel's over 2, 4 and 2 (head sizes 128 and 64, one and several row tiles with a
# ragged last one); the others finish inside one workgroup.
@pytest.mark.parametrize("Hq,Hkv,d,hidden,B,T_new,rope", [(8, 2, 128, 512, 3, 1, True), (4, 4, 64, 256, 2, 21, True),
                                                            (8, 8, 128, 1024, 5, 64, True), (4, 1, 128, 128, 4, 5, False),
                                                            (32, 8, 128, 4096, 4, 1, True), (8, 2, 128, 2048, 3, 1, True),
                                                            (8, 2, 128, 1536, 2, 16, True), (8, 1, 64, 4096, 2, 1, False),
                                                            (8, 2, 128, 2048, 2, 40, True), (8, 2, 64, 4096, 3, 50, True),
                                                            (4, 1, 128, 2048, 5, 60, False), (8, 2, 128, 1536, 2, 17, True)])
def test_project_append_parity(kb, Hq, Hkv, d, hidden, B, T_new, rope):
    _check_project_append(kb, Hq, Hkv, d, hidden, B, T_new, rope, 160)


# Enough 256-row tiles that a workgroup takes two head blocks at once (K|K, K|V with an odd number
# of kv heads, V|V): contractions of two and of six staged steps, a ragged last row tile.
@pytest.mark.parametrize("Hq,Hkv,d,hidden,B,T_new,rope", [(8, 8, 128, 384, 24, 250, True), (3, 3, 128, 128, 64, 255, True),
                                                            (8, 8, 128, 128, 25, 256, False)])
def test_project_append_parity_two_heads_per_workgroup(kb, Hq, Hkv, d, hidden, B, T_new, rope):
    assert Hkv * ((B * T_new + 255) // 256) >= 192
    _check_project_append(kb, Hq, Hkv, d, hidden, B, T_new, rope, 272)


# Into fp8 slots: the streaming kernel (with a split contraction), the tiled one and the one with
# two head blocks per workgroup.  A stored element is the bf16-rounded result rounded on to E4M3:
# within half an E4M3 step (2^-4 relative, 2^-10 below the normal range) plus the bf16 step of the
# oracle's unrounded value, exactly an E4M3 value, and nearly always the very code the oracle's own
# rounding chain gives (an accumulation error can only matter next to a rounding boundary).
@pytest.mark.parametrize("Hq,Hkv,d,hidden,B,T_new,rope,cap", [(8, 2, 128, 2048, 3, 1, True, 160), (8, 2, 64, 1024, 3, 50, True, 160),
                                                                (8, 8, 128, 384, 24, 250, True, 272)])
def test_project_append_into_fp8_slots(kb, Hq, Hkv, d, hidden, B, T_new, rope, cap):
    _check_project_append(kb, Hq, Hkv, d, hidden, B, T_new, rope, cap, dtype="fp8")


def _check_project_append(kb, Hq, Hkv, d, hidden, B, T_new, rope, cap, dtype="bf16"):
    L = 3
    share = np.array([0, 1, 1], np.int32)
    table = inputs.make_block_table(B, cap // 16, B * cap // 16 + 2, 61)
    store = kb.KVStore(share, Hq, Hkv, d, dtype, B * cap // 16 + 2, cap // 16, block_table=table, zero_fill=True)
    x = (inputs.normal((B, T_new, hidden), 61, 0, dtype="f32") / 4).to(torch.bfloat16)
    wk = (inputs.normal((Hkv * d, hidden), 61, 1, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    wv = (inputs.normal((Hkv * d, hidden), 61, 2, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    start = np.array([(7 * b + 3) % (cap - T_new + 1) for b in range(B)], np.int32)
    cos, sin = _rope_tables(cap, d) if rope else (None, None)
    dev = lambda t: None if t is None else torch.from_numpy(t).cuda()
    before = store.pool.clone()
    assert kb.kvs_project_append_kv(store, 2, x.cuda(), wk.cuda(), wv.cuda(), start, dev(cos), dev(sin)) == kb.KVS_NOOP
    torch.cuda.synchronize()
    assert torch.equal(before, store.pool)                       # a recipient layer computes and stores nothing
    assert kb.kvs_project_append_kv(store, 1, x.cuda(), wk.cuda(), wv.cuda(), start, dev(cos), dev(sin)) == kb.KVS_OK
    first = store.pool.clone()
    # again on the same workspace: the arrival counters were left at zero and the merge adds the
    # partial sums in a fixed order, so the stored bits repeat
    assert kb.kvs_project_append_kv(store, 1, x.cuda(), wk.cuda(), wv.cuda(), start, dev(cos), dev(sin)) == kb.KVS_OK
    assert torch.equal(first, store.pool)
    want_k, want_v = project_kv(inputs.to_oracle_array(x), inputs.to_oracle_array(wk), inputs.to_oracle_array(wv),
                                Hkv, d, start, cos, sin)
    same, total = 0, 0
    for layer in (1, 2):                                         # the recipient sees the donor's new rows
        for b in range(B):
            k, v = kb.kvs_gather_kv(store, layer, int(start[b]), T_new, B)
            for got, want in ((k[b], want_k[b]), (v[b], want_v[b])):
                got = got.float().cpu().numpy().astype(np.float64)
                if dtype == "fp8":
                    from oracle.fp8 import round_e4m3
                    assert np.array_equal(got, round_e4m3(got))
                    assert np.all(np.abs(got - want) <= (2.0 ** -4 + 2.0 ** -7) * np.abs(want) + 2.0 ** -10 + 2.0 ** -14), (layer, b)
                    chain = round_e4m3(_bf16_round(want).float().numpy().astype(np.float64))
                    same += int((got == chain).sum())
                    total += got.size
                    continue
                floor = 1e-2 * np.sqrt((want ** 2).mean())
                assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.maximum(np.abs(want), floor)), (layer, b)
    if dtype == "fp8":
        assert same >= 0.995 * total, (same, total)
    # slot 0 (layer 0) untouched
    k0, _ = kb.kvs_gather_kv(store, 0, 0, cap, B)
    assert float(k0.float().abs().max()) == 0.0


def test_projected_rows_feed_decode_attention(kb):
    """One decode step through the fused projection, then attention, against the oracle chain
    (project in fp64, round to bf16, attend in fp64)."""
    L, Hq, Hkv, d, hidden, B, cap = 2, 8, 2, 128, 512, 3, 96
    share = np.array([0, 0], np.int32)
    store = kb.KVStore(share, Hq, Hkv, d, "bf16", B * cap // 16, cap // 16)
    cos, sin = _rope_tables(cap, d)
    wk = (inputs.normal((Hkv * d, hidden), 62, 1, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    wv = (inputs.normal((Hkv * d, hidden), 62, 2, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    lens = np.array([96, 40, 17], np.int32)
    T0 = 95
    x0 = inputs.normal((B, T0, hidden), 62, 3)
    kb.kvs_project_append_kv(store, 0, x0.cuda(), wk.cuda(), wv.cuda(), np.zeros(B, np.int32),
                             torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda())
    x1 = inputs.normal((B, 1, hidden), 62, 4)
    kb.kvs_project_append_kv(store, 0, x1.cuda(), wk.cuda(), wv.cuda(), lens - 1,
                             torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda())
    K = np.zeros((B, cap, Hkv, d), np.uint16); V = np.zeros_like(K)
    k0, v0 = project_kv(inputs.to_oracle_array(x0), inputs.to_oracle_array(wk), inputs.to_oracle_array(wv), Hkv, d,
                        np.zeros(B, np.int32), cos, sin)
    k1, v1 = project_kv(inputs.to_oracle_array(x1), inputs.to_oracle_array(wk), inputs.to_oracle_array(wv), Hkv, d,
                        lens - 1, cos, sin)
    K[:, :T0] = inputs.to_oracle_array(_bf16_round(k0)); V[:, :T0] = inputs.to_oracle_array(_bf16_round(v0))
    for b in range(B):
        K[b, lens[b] - 1] = inputs.to_oracle_array(_bf16_round(k1[b, 0])); V[b, lens[b] - 1] = inputs.to_oracle_array(_bf16_round(v1[b, 0]))
    q = inputs.normal((B, Hq, d), 62, 5)
    got = kb.kvs_decode_attention(store, 1, q.cuda(), lens).cpu().numpy()
    want = orc.decode_attention(1, share, [K, None], [V, None], inputs.to_oracle_array(q), lens)
    assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION


def test_project_workspace_contract(kb):
    """Too small a workspace is refused before any launch; the stated size is accepted."""
    Hq, Hkv, d, hidden, B = 8, 2, 128, 2048, 2
    store = kb.KVStore(np.array([0], np.int32), Hq, Hkv, d, "bf16", B * 2, 2)
    need = kb.lib().kvs_project_workspace_bytes(store.desc, hidden, B, 1)
    assert need > 0
    x = inputs.normal((B, 1, hidden), 63, 0).cuda()
    wk = inputs.normal((Hkv * d, hidden), 63, 1).cuda()
    wv = inputs.normal((Hkv * d, hidden), 63, 2).cuda()
    small = torch.zeros(need - 1, dtype=torch.uint8, device="cuda")
    with pytest.raises(kb.KvsError) as err:
        kb.kvs_project_append_kv(store, 0, x, wk, wv, np.zeros(B, np.int32), workspace=small)
    assert err.value.status == kb.KVS_ERR_INVALID_ARG
    exact = torch.zeros(need, dtype=torch.uint8, device="cuda")
    assert kb.kvs_project_append_kv(store, 0, x, wk, wv, np.zeros(B, np.int32), workspace=exact) == kb.KVS_OK
    torch.cuda.synchronize()
    n_tiles = 2 * Hkv * (d // 32)
    assert int(exact[:4 * n_tiles].max()) == 0                  # counters back at zero
