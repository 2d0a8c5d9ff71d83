"""GPU: one workspace serves calls of different shapes in turn.

The arrival counters of the split merges sit in a region of fixed size at the workspace's start,
so the partial results of one call can never land where a later call of another batch size, row
count or kind keeps its counters (a counter that does not start at zero means that no workgroup
merges the splits, and the output keeps stale data without any error).  Every call below is
checked against the fp64 oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import attention as orc
from oracle.projection import project_kv
from paper_2410_18517_amd import inputs
from helpers import Case, rel_l2_rows, REL_L2_ATTENTION

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def test_decode_batches_and_split_prefill_share_one_workspace(kb):
    """Decode of 4 sequences, then of 16, then a whole-prompt prefill whose context is split, then
    the small decode again, all on one workspace (GQA shape: 8 kv heads, long context, so that each
    of the calls splits the context and publishes partial states)."""
    Hq, Hkv, d, B, cap = 32, 8, 128, 16, 4096
    share = np.array([0, 0], np.int32)
    case = Case(kb, 2, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=83)
    desc = C.byref(case.store.desc)
    need = max(kb.lib().kvs_workspace_bytes(desc, 4, 1), kb.lib().kvs_workspace_bytes(desc, 16, 1),
               kb.lib().kvs_workspace_bytes(desc, 1, 256))
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    lens = np.array([cap - 7 * b for b in range(B)], np.int32)

    def decode(nb):
        q = case.q(1)[:nb].contiguous()
        # the workspace is handed over as it is: nothing is cleared between the calls
        got = kb.kvs_decode_attention(case.store, 1, q.cuda(), lens[:nb], workspace=ws)
        want = orc.decode_attention(1, share, [case.K[0][:nb], None], [case.V[0][:nb], None],
                                    inputs.to_oracle_array(q), lens[:nb])
        assert rel_l2_rows(got.cpu().numpy(), want).max() <= REL_L2_ATTENTION, nb

    def prefill(nb, rows):
        q = case.q(1, rows=rows)[:nb].contiguous()
        start = np.full(nb, cap - rows, np.int32)
        got = kb.kvs_prefill_attention(case.store, 1, q.cuda(), start, workspace=ws).cpu().numpy()
        want = orc.shared_attention(1, share, [case.K[0][:nb], None], [case.V[0][:nb], None],
                                    inputs.to_oracle_array(q), start)
        assert rel_l2_rows(got, want).max() <= REL_L2_ATTENTION, (nb, rows)

    decode(4)
    decode(16)
    prefill(1, 256)          # 8 (sequence, kv head) pairs x 4 column blocks: the context is split
    decode(4)
    prefill(2, 40)
    decode(16)
    decode(1)


def test_projection_row_counts_share_one_workspace(kb):
    """A decode-step projection (its contraction split over workgroups), a 2048-row prefill chunk
    (more output tiles, also split) and the decode step again, on one workspace."""
    Hq, Hkv, d, hidden, B, cap = 8, 2, 128, 2048, 8, 512
    share = np.array([0, 1], np.int32)
    table = inputs.make_block_table(B, cap // 16, B * cap // 16 + 2, 91)
    store = kb.KVStore(share, Hq, Hkv, d, "bf16", B * cap // 16 + 2, cap // 16, block_table=table, zero_fill=True)
    wk = (inputs.normal((Hkv * d, hidden), 91, 1, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    wv = (inputs.normal((Hkv * d, hidden), 91, 2, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    need = max(kb.lib().kvs_project_workspace_bytes(C.byref(store.desc), hidden, B, T) for T in (1, 256))
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    for step, T_new in enumerate((1, 256, 1, 5, 256, 1)):
        x = (inputs.normal((B, T_new, hidden), 91, 10 + step, dtype="f32") / 4).to(torch.bfloat16)
        start = np.array([(3 * b + step) % (cap - T_new + 1) for b in range(B)], np.int32)
        assert kb.kvs_project_append_kv(store, 1, x.cuda(), wk.cuda(), wv.cuda(), start, workspace=ws) == kb.KVS_OK
        want_k, want_v = project_kv(inputs.to_oracle_array(x), inputs.to_oracle_array(wk), inputs.to_oracle_array(wv),
                                    Hkv, d, start, None, None)
        for b in range(B):
            k, v = kb.kvs_gather_kv(store, 1, int(start[b]), T_new, B)
            for got, want in ((k[b], want_k[b]), (v[b], want_v[b])):
                got = got.float().cpu().numpy().astype(np.float64)
                floor = 1e-2 * np.sqrt((want ** 2).mean())
                assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.maximum(np.abs(want), floor)), (step, T_new, b)


def test_check_store_reports_map_and_page_table_damage(kb):
    """kvs_check_store: zero counts for a sound store; a device map entry that differs from the host
    copy and page-table entries outside the pool are counted (the kernels themselves clamp them)."""
    share = np.array([0, 1, 1, 0], np.int32)
    B, cap = 3, 64
    table = inputs.make_block_table(B, cap // 16, B * cap // 16 + 1, 5)
    store = kb.KVStore(share, 4, 2, 64, "bf16", B * cap // 16 + 1, cap // 16, block_table=table)
    assert kb.kvs_check_store(store, B).tolist() == [0, 0]
    store.share_map[2] = 2                      # device copy only
    store.slot_of_layer[3] = 1
    assert kb.kvs_check_store(store, B).tolist() == [2, 0]
    store.block_table[1, 2] = -1
    store.block_table[2, 0] = B * cap // 16 + 1
    assert kb.kvs_check_store(store, B).tolist() == [2, 2]
    assert kb.kvs_check_store(store, 1).tolist() == [2, 0]      # only the first row of the table
    plain = kb.KVStore(share, 4, 2, 64, "bf16", B * cap // 16, cap // 16)
    assert kb.kvs_check_store(plain, B).tolist() == [0, 0]      # contiguous: no table to check
