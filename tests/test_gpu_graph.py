"""A whole decode step (every layer's kvs_decode_step) recorded once into a HIP graph and replayed
for several generated tokens: the sequence lengths live on the device and are advanced between
replays, the step's queries and new rows are copied into fixed buffers.  Every replay is checked
against the oracle, with eager launches and synchronisations of the same library between the
replays, so that anything a launch leaves behind (arrival counters, partial states) or any
host-side state baked into the recording would show."""
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
    return binding


# cap 1024: long enough for the context to be split, so the launches size their splits (and number
# their work items) from the device-side lengths, which change from replay to replay
@pytest.mark.parametrize("split,cap,T0", [(0, 96, 60), (64, 96, 60), (0, 1024, 1000)])
def test_decode_steps_replayed_from_a_graph(kb, split, cap, T0):
    L, Hq, Hkv, d, B = 4, 8, 2, 128, 3
    share = np.array([0, 1, 1, 0], np.int32)
    case = Case(kb, L, Hq, Hkv, d, B, "bf16", cap, share, paged=True, seed=91, fill_tokens=T0)
    K = [None if x is None else np.concatenate([x, np.zeros((B, cap - T0, Hkv, d), x.dtype)], 1) for x in case.K]
    V = [None if x is None else np.concatenate([x, np.zeros((B, cap - T0, Hkv, d), x.dtype)], 1) for x in case.V]
    lens = np.array([T0, 15, 31], np.int32)                    # before the first step; rows 15 and 31 end a page
    lens_dev = torch.from_numpy(lens.copy()).cuda()
    q_buf = torch.zeros((L, B, Hq, d), dtype=torch.bfloat16, device="cuda")
    k_buf = torch.zeros((L, B, 1, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_buf = torch.zeros_like(k_buf)
    out_buf = torch.zeros((L, B, Hq, d), dtype=torch.float32, device="cuda")
    assert kb.lib().kvs_testing_force_split_tokens(split) == kb.KVS_OK
    try:
        ws = case.store.workspace(B, 1)                         # sized for this split setting, before the recording
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            for layer in range(L):
                kb.kvs_decode_step(case.store, layer, q_buf[layer], k_buf[layer], v_buf[layer], lens_dev,
                                   out=out_buf[layer], workspace=ws)
        for step in range(4):
            lens += 1
            lens_dev += 1                                       # the only per-step state, and it is the device's
            qs = [inputs.normal((B, Hq, d), 91, step, layer, 500) for layer in range(L)]
            ks = [inputs.normal((B, 1, Hkv, d), 91, step, layer, 501) for layer in range(L)]
            vs = [inputs.normal((B, 1, Hkv, d), 91, step, layer, 502) for layer in range(L)]
            q_buf.copy_(torch.stack(qs)); k_buf.copy_(torch.stack(ks)); v_buf.copy_(torch.stack(vs))
            graph.replay()
            torch.cuda.synchronize()
            got = out_buf.cpu().numpy()
            for layer in range(L):
                orc.append_kv(layer, share, K, V, inputs.to_oracle_array(ks[layer]), inputs.to_oracle_array(vs[layer]), lens - 1)
            for layer in range(L):
                want = orc.decode_attention(layer, share, K, V, inputs.to_oracle_array(qs[layer]), lens)
                assert rel_l2_rows(got[layer], want).max() <= REL_L2_ATTENTION, (step, layer)
                # eager work of the same library on the same workspace between the replays
                eager = kb.kvs_decode_attention(case.store, layer, q_buf[layer], lens_dev, workspace=ws).cpu().numpy()
                assert rel_l2_rows(eager, want).max() <= REL_L2_ATTENTION, (step, layer)
    finally:
        assert kb.lib().kvs_testing_force_split_tokens(0) == kb.KVS_OK
