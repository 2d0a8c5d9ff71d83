"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times
(full batch, full store geometry, default split policy, permuted page table).  The store is
allocated at full size; only the layers that are sampled (recipients, their donors and layer 0)
are filled, since a layer's kernel touches no other slot.  For decode the oracle checks every
sequence and head of the sampled layers, element by element; for prefill sampled sequences."""
import numpy as np
import pytest
import torch

from oracle import attention as orc
from paper_2410_18517_amd import inputs
from helpers import Case, rel_l2_rows, REL_L2_ATTENTION, REL_DISTANCE

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2410_18517_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.kvs_testing_force_split_tokens(0)
    return binding


def _sample_layers(share):
    recipients = [l for l in range(len(share)) if share[l] != l]
    picked = [recipients[0], recipients[-1]] if recipients else []
    layers = sorted(set([0] + picked + [int(share[r]) for r in picked]))
    return layers, sorted(set(int(share[l]) for l in layers))


def _sub(case, layer_arrays, b):
    return [None if a is None else a[b:b + 1] for a in layer_arrays]


@pytest.mark.parametrize("name", ["tiny", "llama2-7b", "llama2-13b", "llama3-8b-32k", "gqa48-ragged"])
def test_decode_full_size_sampled(kb, name):
    w = inputs.WORKLOADS[name]
    share = inputs.make_share_map(w.L, w.n_shared, 1, fixed=w.fixed_map)
    lens = inputs.make_seq_lens(w, 1)
    layers, fill = _sample_layers(share)
    case = Case(kb, w.L, w.Hq, w.Hkv, w.d, w.B, w.dtype, w.context, share, paged=True, seed=100,
                fill_layers=fill, spare_blocks=0)
    assert case.store.desc.n_slots == w.L - w.n_shared
    tol = 1e-5 if w.dtype == "f32" else REL_L2_ATTENTION
    worst = 0.0
    for layer in layers:
        q = case.q(layer)
        got = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens).cpu().numpy()
        assert np.isfinite(got).all()
        # every sequence and head of the launch (the oracle walks a whole layer of the largest workload in 0.2 s)
        want = orc.decode_attention(layer, share, case.K, case.V, inputs.to_oracle_array(q), lens)
        err = rel_l2_rows(got, want)
        worst = max(worst, err.max())
        assert err.max() <= tol, (name, layer, np.unravel_index(np.argmax(err), err.shape), err.max())
    print(f"{name}: layers {layers}, all {w.B} sequences, max rel L2 {worst:.2e}")


def test_prefill_full_size_sampled(kb):
    """Llama-2-13B shape: a 64-row causal chunk at the end of a 2048-token context; own-cache layers
    append their 64 rows first, recipients read the donor's slot."""
    w = inputs.WORKLOADS["llama2-13b"]
    T_new = w.prefill_rows
    share = inputs.make_share_map(w.L, w.n_shared, 1)
    layers, fill = _sample_layers(share)
    case = Case(kb, w.L, w.Hq, w.Hkv, w.d, w.B, w.dtype, w.context, share, paged=True, seed=200,
                fill_layers=fill, fill_tokens=w.context - T_new, spare_blocks=0)
    start = np.full(w.B, w.context - T_new, np.int32)
    Ko = [None if x is None else np.concatenate([x, np.zeros((w.B, T_new, w.Hkv, w.d), x.dtype)], 1) for x in case.K]
    Vo = [None if x is None else np.concatenate([x, np.zeros((w.B, T_new, w.Hkv, w.d), x.dtype)], 1) for x in case.V]
    for layer in layers:                                  # layer order: donors before recipients
        k_new = inputs.normal((w.B, T_new, w.Hkv, w.d), 200, layer, 50)
        v_new = inputs.normal((w.B, T_new, w.Hkv, w.d), 200, layer, 51)
        st = kb.kvs_append_kv(case.store, layer, k_new.cuda(), v_new.cuda(), start)
        wrote = orc.append_kv(layer, share, Ko, Vo, inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new), start)
        assert (st == kb.KVS_OK) == wrote
        q = case.q(layer, rows=T_new)
        got = kb.kvs_prefill_attention(case.store, layer, q.cuda(), start).cpu().numpy()
        assert np.isfinite(got).all()
        for b in (0, w.B - 1):
            want = orc.shared_attention(layer, share, _sub(case, Ko, b), _sub(case, Vo, b),
                                        inputs.to_oracle_array(q[b:b + 1]), start[b:b + 1])
            assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, (layer, b)


def test_distance_full_size(kb):
    """Calibration of the 48-layer workload: 30 samples x 512 tokens x 8 kv heads x 128 (2.8 GiB)."""
    S, L, Hkv, T, d = 30, 48, 8, 512, 128
    kv = inputs.calibration_kv(S, L, Hkv, T, d, 300)
    dK2, dV2, D = (t.cpu().numpy().astype(np.float64) for t in kb.kvs_layer_distance(kv.cuda()))
    oK2, oV2, oD = orc.layer_distance(inputs.to_oracle_array(kv))
    for got, want in ((dK2, oK2), (dV2, oV2), (D, oD)):
        assert np.linalg.norm(got - want) <= REL_DISTANCE * np.linalg.norm(want)
    off = ~np.eye(L, dtype=bool)
    assert np.abs(D[off] / oD[off] - 1).max() <= 5 * REL_DISTANCE
    assert np.array_equal(D, D.T) and np.all(np.diag(D) == 0)
    from oracle import share_map as osm
    got = kb.kvs_build_share_map(D.astype(np.float32), 14)
    want = osm.build_share_map(D.astype(np.float32), L, 14)
    assert (got[0], got[1].tolist(), got[2].tolist(), got[3], got[4]) == want and got[3] == 34


def test_whole_prompt_prefill_full_size_sampled(kb):
    """Llama-2-13B shape, the whole 2048-token prompt prefilled in one call (32 column groups of 64
    rows per head): rows sampled from the first, a middle and the last group of two sequences."""
    w = inputs.WORKLOADS["llama2-13b"]
    T_new = w.context
    share = inputs.make_share_map(w.L, w.n_shared, 1)
    recipient = next(l for l in range(w.L) if share[l] != l)
    donor = int(share[recipient])
    case = Case(kb, w.L, w.Hq, w.Hkv, w.d, w.B, w.dtype, w.context, share, paged=True, seed=201,
                fill_layers=[donor], fill_tokens=T_new, spare_blocks=0)
    start = np.zeros(w.B, np.int32)
    for layer in (donor, recipient):
        q = case.q(layer, rows=T_new)
        got = kb.kvs_prefill_attention(case.store, layer, q.cuda(), start).cpu().numpy()
        assert np.isfinite(got).all()
        for b in (0, w.B - 1):
            for r0 in (0, 1000, T_new - 16):
                want = orc.shared_attention(layer, share, _sub(case, case.K, b), _sub(case, case.V, b),
                                            inputs.to_oracle_array(q[b:b + 1, r0:r0 + 16]), np.array([r0], np.int32))
                assert rel_l2_rows(got[b:b + 1, r0:r0 + 16], want).max() <= REL_L2_ATTENTION, (layer, b, r0)


def test_decode_full_size_fp8_slots(kb):
    """The 32k GQA workload with its slots kept in fp8: same launch configuration as the bf16 run,
    half the bytes; sampled sequences, all heads, against the oracle on the values as stored."""
    w = inputs.WORKLOADS["llama3-8b-32k"]
    share = inputs.make_share_map(w.L, w.n_shared, 1, fixed=w.fixed_map)
    lens = inputs.make_seq_lens(w, 1)
    layers, fill = _sample_layers(share)
    case = Case(kb, w.L, w.Hq, w.Hkv, w.d, w.B, "fp8", w.context, share, paged=True, seed=101,
                fill_layers=fill, spare_blocks=0)
    assert case.store.pool.numel() * 2 == (w.L - w.n_shared) * w.B * w.context * w.Hkv * w.d * 2 * 2
    for layer in layers:
        q = case.q(layer)
        got = kb.kvs_decode_attention(case.store, layer, q.cuda(), lens).cpu().numpy()
        assert np.isfinite(got).all()
        for b in (0, w.B - 1):
            want = orc.decode_attention(layer, share, _sub(case, case.K, b), _sub(case, case.V, b),
                                        inputs.to_oracle_array(q[b:b + 1]), lens[b:b + 1])
            assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, (layer, b)


@pytest.mark.parametrize("name", ["llama3-8b-32k", "gqa48-ragged"])
def test_decode_step_full_size_sampled(kb, name):
    """The one-launch decode step at full size: a donor layer stores its new row and attends, its
    recipient then attends to the same slot; sampled sequences against the oracle's append + attention."""
    w = inputs.WORKLOADS[name]
    share = inputs.make_share_map(w.L, w.n_shared, 1, fixed=w.fixed_map)
    lens = inputs.make_seq_lens(w, 1)
    recipient = next(l for l in range(w.L) if share[l] != l)
    donor = int(share[recipient])
    case = Case(kb, w.L, w.Hq, w.Hkv, w.d, w.B, w.dtype, w.context, share, paged=True, seed=102,
                fill_layers=[donor], spare_blocks=0)
    k_new = inputs.normal((w.B, 1, w.Hkv, w.d), 102, 700)
    v_new = inputs.normal((w.B, 1, w.Hkv, w.d), 102, 701)
    K, V = list(case.K), list(case.V)
    K[donor], V[donor] = K[donor].copy(), V[donor].copy()
    assert orc.append_kv(donor, share, K, V, inputs.to_oracle_array(k_new), inputs.to_oracle_array(v_new), lens - 1)
    seqs = sorted(set([int(np.argmax(lens)), int(np.argmin(lens))]))
    for layer in (donor, recipient):
        q = case.q(layer)
        got = kb.kvs_decode_step(case.store, layer, q.cuda(), k_new.cuda(), v_new.cuda(), lens).cpu().numpy()
        for b in seqs:
            want = orc.decode_attention(layer, share, [None if a is None else a[b:b + 1] for a in K],
                                        [None if a is None else a[b:b + 1] for a in V],
                                        inputs.to_oracle_array(q[b:b + 1]), lens[b:b + 1])
            assert rel_l2_rows(got[b:b + 1], want).max() <= REL_L2_ATTENTION, (layer, b)


def test_projection_full_size_sampled(kb):
    """The fused K/V projection at the shape bench.py times for a prefill chunk: 4 x 2048 rows,
    hidden 4096, 8 kv heads of 128 (64 staged contraction steps, the two-heads-per-workgroup
    kernel), rotary embedding, a permuted page table.  The fp64 oracle projects 96 sampled rows
    (first and last rows of tiles and sequences among them) and every stored channel of those rows
    is held to one bf16 unit of it."""
    from oracle.projection import project_kv
    Hq, Hkv, d, hidden, B, T = 32, 8, 128, 4096, 4, 2048
    cap = 4096
    share = np.array([0, 1, 1], np.int32)
    table = inputs.make_block_table(B, cap // 16, B * cap // 16, 67)
    store = kb.KVStore(share, Hq, Hkv, d, "bf16", B * cap // 16, cap // 16, block_table=table, zero_fill=True)
    x = (inputs.normal((B, T, hidden), 67, 0, dtype="f32") / 4).to(torch.bfloat16)
    wk = (inputs.normal((Hkv * d, hidden), 67, 1, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    wv = (inputs.normal((Hkv * d, hidden), 67, 2, dtype="f32") / np.sqrt(hidden)).to(torch.bfloat16)
    inv = 10000.0 ** (-np.arange(d // 2, dtype=np.float64) * 2.0 / d)
    ang = np.outer(np.arange(cap, dtype=np.float64), inv)
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    start = np.array([0, 2048, 1000, 37], np.int32)
    assert kb.kvs_project_append_kv(store, 1, x.cuda(), wk.cuda(), wv.cuda(), start, torch.from_numpy(cos).cuda(),
                                    torch.from_numpy(sin).cuda()) == kb.KVS_OK
    rng = np.random.default_rng(67)
    rows = sorted(set([0, 1, 255, 256, 2047] + rng.integers(0, T, size=19).tolist()))
    xo, wko, wvo = inputs.to_oracle_array(x), inputs.to_oracle_array(wk), inputs.to_oracle_array(wv)
    checked = 0
    for b in range(B):
        k_all, v_all = kb.kvs_gather_kv(store, 2, int(start[b]), T, B)        # through the recipient layer
        for i in rows:
            want_k, want_v = project_kv(xo[b:b + 1, i:i + 1], wko, wvo, Hkv, d, start[b:b + 1] + i, cos, sin)
            for got, want in ((k_all[b, i], want_k[0, 0]), (v_all[b, i], want_v[0, 0])):
                got = got.float().cpu().numpy().astype(np.float64)
                floor = 1e-2 * np.sqrt((want ** 2).mean())
                assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.maximum(np.abs(want), floor)), (b, i)
                checked += got.size
    assert checked >= 96 * 2 * Hkv * d
    k0, _ = kb.kvs_gather_kv(store, 0, 0, 64, B)                              # another layer's slot: untouched
    assert float(k0.float().abs().max()) == 0.0
