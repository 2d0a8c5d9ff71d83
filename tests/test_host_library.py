"""CPU-only checks of libkvs.so: exported symbols, the strategy walk (bit-exact against the
oracle on the same distance matrix) and every argument error that is decided before a HIP call."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import share_map as osm
from paper_2410_18517_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("kvs.h", "kvs_testing.h"))
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", body))
    declared -= {"kvs_accept_fn"}
    assert declared == set(kb.EXPORTS)
    lib = kb.lib()
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("L,C_", [(4, 1), (8, 3), (32, 8), (40, 12), (48, 14), (48, 18)])
@pytest.mark.parametrize("order", [0, 1])
def test_share_map_matches_oracle_bitwise(L, C_, order):
    rng = np.random.default_rng(L * 100 + C_)
    A = rng.random((L, L)).astype(np.float32)
    D = A + A.T
    np.fill_diagonal(D, 0)
    D[1, 3] = D[3, 1] = D[0, 2] = D[2, 0] = 0.5          # a tie
    st, share, slot, n_slots, n_shared = kb.kvs_build_share_map(D, C_, order)
    ost, oshare, oslot, on_slots, on_shared = osm.build_share_map(D, L, C_, ascending=bool(order))
    assert (st, share.tolist(), slot.tolist(), n_slots, n_shared) == (ost, oshare, oslot, on_slots, on_shared)
    assert kb.kvs_validate_share_map(share) == kb.KVS_OK
    s2, n2 = kb.kvs_slots_from_share_map(share)
    assert s2.tolist() == oslot and n2 == on_slots


def test_random_sharing_baseline_is_the_walk_over_a_random_ranking():
    """Sec. 5.3 compares against randomly chosen pairs at 25 % compression, three draws: a matrix of
    random values and no similarity test gives such a strategy, valid and different per draw."""
    L, C_ = 40, 10
    maps = []
    for seed in range(3):
        D = np.random.default_rng(seed).random((L, L)).astype(np.float32)
        st, share, slot, n_slots, n_shared = kb.kvs_build_share_map(D, C_, 0)
        assert st == kb.KVS_OK and n_shared == C_ and n_slots == L - C_
        assert kb.kvs_validate_share_map(share) == kb.KVS_OK
        assert share.tolist() == osm.build_share_map(D, L, C_)[1]
        maps.append(tuple(share.tolist()))
    assert len(set(maps)) == 3


def test_share_map_accept_callback_and_unreachable_target():
    D = np.array([[0, 1, 7, 8], [1, 0, 6, 9], [7, 6, 0, 5], [8, 9, 5, 0]], np.float32)
    calls = []
    def accept(m):
        calls.append(list(m))
        return len(calls) != 1                       # discard the first candidate only
    got = kb.kvs_build_share_map(D, 2, 0, accept)
    ocalls = []
    def oaccept(m):
        ocalls.append(list(m))
        return len(ocalls) != 1
    want = osm.build_share_map(D, 4, 2, accept=oaccept)
    assert calls == ocalls == [[0, 1, 2, 1], [0, 1, 2, 0], [0, 1, 0, 0]]
    assert (got[0], got[1].tolist(), got[2].tolist(), got[3], got[4]) == want
    st, share, _, n_slots, n_shared = kb.kvs_build_share_map(D, 3, 0, lambda m: False)
    assert st == kb.KVS_ERR_TARGET_UNREACHED and n_shared == 0 and share.tolist() == [0, 1, 2, 3] and n_slots == 4
    assert "exhausted" in kb.last_error()


def test_share_map_argument_errors():
    D = np.zeros((3, 3), np.float32)
    with pytest.raises(kb.KvsError) as e:
        kb.kvs_build_share_map(D, 3)
    assert e.value.status == kb.KVS_ERR_INVALID_ARG
    D[0, 2] = np.nan
    with pytest.raises(kb.KvsError):
        kb.kvs_build_share_map(D, 1)
    with pytest.raises(kb.KvsError):
        kb.kvs_build_share_map(np.zeros((3, 3), np.float32), 1, order=2)
    assert kb.kvs_validate_share_map([0, 0, 1]) == kb.KVS_ERR_BAD_MAP      # chain
    assert kb.kvs_validate_share_map([1, 1]) == kb.KVS_ERR_BAD_MAP         # donor nearer the output
    assert kb.kvs_validate_share_map([0, 0, 0, 3]) == kb.KVS_OK


def _desc(**kw):
    base = dict(L=4, n_slots=3, Hq=4, Hkv=2, head_dim=128, dtype=kb.KVS_BF16, block_tokens=16,
                num_blocks=8, max_blocks_per_seq=4)
    base.update(kw)
    return kb.kvs_desc(**base)


def test_store_and_workspace_sizes():
    lib = kb.lib()
    d = _desc()
    assert lib.kvs_store_bytes(C.byref(d)) == 3 * 8 * 2 * 2 * 16 * 128 * 2
    assert lib.kvs_store_bytes(C.byref(_desc(dtype=kb.KVS_F32, head_dim=64))) == 3 * 8 * 2 * 2 * 16 * 64 * 4
    assert lib.kvs_workspace_bytes(C.byref(d), 2, 1) > 0
    for bad in (dict(head_dim=96), dict(block_tokens=32), dict(Hq=5), dict(n_slots=5), dict(dtype=7),
                dict(Hq=34, Hkv=2), dict(num_blocks=0), dict(dtype=kb.KVS_F32, head_dim=320)):
        assert lib.kvs_store_bytes(C.byref(_desc(**bad))) == 0, bad
        assert kb.last_error()
    assert lib.kvs_workspace_bytes(C.byref(d), 0, 1) == 0
    assert lib.kvs_distance_workspace_bytes(129) == 0 and lib.kvs_distance_workspace_bytes(48) > 0
    assert lib.kvs_distance_workspace_bytes(128) > lib.kvs_distance_workspace_bytes(64)      # per pair block of layers
    # projection: the fixed 64 KiB counter region, then, when the contraction is split, one 256-thread
    # pair of floats per output tile (2*Hkv*(d/32) per 16 rows) and split
    big = _desc(Hq=32, Hkv=8)
    assert lib.kvs_project_workspace_bytes(C.byref(big), 4096, 4, 1) == 65536 + 4 * 64 * 256 * 8
    assert lib.kvs_project_workspace_bytes(C.byref(big), 128, 4, 1) == 65536        # nothing to split
    # more than 32 rows: 256-row tiles of a whole head, 512 threads x 64 accumulators per tile and split
    assert lib.kvs_project_workspace_bytes(C.byref(big), 4096, 64, 64) == 65536                  # enough tiles already
    assert lib.kvs_project_workspace_bytes(C.byref(big), 4096, 16, 64) == 65536 + 4 * 64 * 512 * 64 * 4
    assert lib.kvs_project_workspace_bytes(C.byref(big), 100, 4, 1) == 0
    assert lib.kvs_project_workspace_bytes(C.byref(_desc(dtype=kb.KVS_F32)), 4096, 4, 1) == 0


def test_workspace_covers_every_row_count_up_to_the_maximum():
    """Fewer rows can mean more context splits and so more partial states: the size for a range of
    row counts must not shrink when the range grows (33 rows against 32 at 64 (sequence, kv head)
    pairs is such a place: the kernel shape changes there and the splits halve)."""
    lib = kb.lib()
    for kw, B in ((dict(Hq=32, Hkv=8, max_blocks_per_seq=128, num_blocks=1024), 8),
                  (dict(Hq=32, Hkv=8, max_blocks_per_seq=2048, num_blocks=8192), 4),
                  (dict(Hq=40, Hkv=40, max_blocks_per_seq=128, num_blocks=2048), 16),
                  (dict(Hq=8, Hkv=1, max_blocks_per_seq=4096, num_blocks=4096), 1)):
        d = _desc(**kw)
        sizes = [lib.kvs_workspace_bytes(C.byref(d), B, r) for r in range(1, 300)]
        assert all(s > 0 for s in sizes)
        assert all(a <= b for a, b in zip(sizes, sizes[1:])), kw
    d = _desc(Hq=32, Hkv=8, max_blocks_per_seq=128, num_blocks=1024)
    assert lib.kvs_workspace_bytes(C.byref(d), 8, 33) == lib.kvs_workspace_bytes(C.byref(d), 8, 32)
    assert lib.kvs_workspace_bytes(C.byref(d), 8, 1 << 30) > 0          # beyond the capacity: as at the capacity


def _fake_store(share=(0, 1, 2, 1), slots=(0, 1, 2, 1), **kw):
    """A store whose device pointers are junk: valid only for calls that fail before any launch."""
    hs, hl = np.asarray(share, np.int32), np.asarray(slots, np.int32)
    st = kb.kvs_store(_desc(**kw), 0x1000, 0x1000, 0x1000, None, hs.ctypes.data, hl.ctypes.data)
    st._keep = (hs, hl)
    return st


def test_entry_points_reject_bad_arguments_without_touching_the_gpu():
    lib = kb.lib()
    st = _fake_store()
    p = C.c_void_p(0x1000)
    # append on a recipient layer is a no-op decided on the host
    assert lib.kvs_append_kv(C.byref(st), 3, p, p, p, 1, 1, None) == kb.KVS_NOOP
    assert lib.kvs_append_kv(C.byref(st), 4, p, p, p, 1, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_append_kv(C.byref(st), -1, p, p, p, 1, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_append_kv(C.byref(st), 0, None, p, p, 1, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_append_kv(C.byref(st), 0, p, p, p, 1, 0, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_append_kv(C.byref(st), 0, p, p, p, 1, 65, None) == kb.KVS_ERR_CAPACITY
    assert lib.kvs_append_kv(C.byref(st), 0, p, p, p, 3, 1, None) == kb.KVS_ERR_CAPACITY   # contiguous: 3*4 > 8 blocks
    assert lib.kvs_append_kv(None, 0, p, p, p, 1, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention(C.byref(st), 0, None, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention(C.byref(st), 9, p, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention(C.byref(st), 0, p, p, 0, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_prefill_attention(C.byref(st), 0, p, p, 1, 65, p, p, 1 << 30, None) == kb.KVS_ERR_CAPACITY
    assert lib.kvs_gather_kv(C.byref(st), 0, 60, 8, 1, p, p, None) == kb.KVS_ERR_CAPACITY
    assert lib.kvs_gather_kv(C.byref(st), 0, 0, 8, 1, None, p, None) == kb.KVS_ERR_INVALID_ARG
    # maps: chain, forward donor, slot disagreement, slot out of range
    for share, slots in (((0, 0, 1, 3), (0, 0, 0, 1)), ((1, 1, 2, 3), (0, 0, 1, 2)),
                         ((0, 1, 2, 1), (0, 1, 2, 2)), ((0, 1, 2, 1), (0, 1, 3, 1))):
        bad = _fake_store(share, slots)
        assert lib.kvs_decode_attention(C.byref(bad), 0, p, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_BAD_MAP
    assert lib.kvs_decode_attention(C.byref(_fake_store(head_dim=96)), 0, p, p, 1, p, p, 1 << 30, None) \
        == kb.KVS_ERR_UNSUPPORTED
    # split workspace too small (4 blocks per sequence, forced 64-token splits => 1 split... use more blocks)
    big = _fake_store(max_blocks_per_seq=64, num_blocks=64)
    assert lib.kvs_testing_force_split_tokens(64) == kb.KVS_OK
    try:
        assert lib.kvs_decode_attention(C.byref(big), 0, p, p, 1, p, p, 16, None) == kb.KVS_ERR_INVALID_ARG
        assert "workspace" in kb.last_error()
    finally:
        assert lib.kvs_testing_force_split_tokens(0) == kb.KVS_OK
    assert lib.kvs_testing_force_split_tokens(100) == kb.KVS_ERR_INVALID_ARG
    # fused projection: recipient layers are a host-side no-op; bad shapes and a missing workspace are errors
    proj = lambda layer, hidden=256, cos=None, sin=None, npos=0, B=1, T=1, ws=p, nws=1 << 30, x=p: \
        lib.kvs_project_append_kv(C.byref(st), layer, x, hidden, p, p, cos, sin, npos, p, B, T, ws, nws, None)
    assert proj(3) == kb.KVS_NOOP
    assert proj(4) == kb.KVS_ERR_INVALID_ARG
    assert proj(0, x=None) == kb.KVS_ERR_INVALID_ARG
    assert proj(0, hidden=200) == kb.KVS_ERR_UNSUPPORTED
    assert proj(0, cos=p) == kb.KVS_ERR_INVALID_ARG                      # one rotary table without the other
    assert proj(0, cos=p, sin=p, npos=63) == kb.KVS_ERR_CAPACITY         # tables shorter than the 64-token capacity
    assert proj(0, T=65) == kb.KVS_ERR_CAPACITY
    assert proj(0, B=0) == kb.KVS_ERR_INVALID_ARG
    assert proj(0, ws=None) == kb.KVS_ERR_INVALID_ARG
    assert proj(0, nws=8) == kb.KVS_ERR_INVALID_ARG and "workspace" in kb.last_error()
    assert lib.kvs_project_append_kv(C.byref(_fake_store(dtype=kb.KVS_F32, head_dim=64)), 0, p, 256, p, p, None, None, 0,
                                     p, 1, 1, p, 1 << 30, None) == kb.KVS_ERR_UNSUPPORTED
    # sparsified slots: per-head append and compaction are no-ops for recipients, bad arguments are errors
    assert lib.kvs_append_kv_per_head(C.byref(st), 3, p, p, p, 1, 1, None) == kb.KVS_NOOP
    assert lib.kvs_append_kv_per_head(C.byref(st), 0, p, p, None, 1, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_compact_kv(C.byref(st), 3, p, p, 8, 1, None) == kb.KVS_NOOP
    assert lib.kvs_compact_kv(C.byref(st), 0, None, p, 8, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_compact_kv(C.byref(st), 0, p, p, 0, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_compact_kv(C.byref(st), 0, p, p, 65, 1, None) == kb.KVS_ERR_CAPACITY
    assert lib.kvs_compact_kv(C.byref(st), 7, p, p, 8, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention_per_head(C.byref(st), 0, p, None, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention_per_head(C.byref(st), 0, None, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention_per_head(C.byref(st), 5, p, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    # the store check
    assert lib.kvs_check_store(C.byref(st), 1, None, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_check_store(C.byref(st), -1, p, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_check_store(None, 1, p, None) == kb.KVS_ERR_INVALID_ARG
    # the one-launch decode step
    assert lib.kvs_decode_step(C.byref(st), 0, p, None, p, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_step(C.byref(st), 0, None, p, p, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_step(C.byref(st), 4, p, p, p, p, 1, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_step(C.byref(st), 0, p, p, p, p, 1, p, None, 0, None) == kb.KVS_ERR_INVALID_ARG
    # distance
    assert lib.kvs_layer_distance(None, 1, 2, 8, 0, p, p, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_layer_distance(p, 1, 129, 8, 0, p, p, p, p, 1 << 30, None) == kb.KVS_ERR_UNSUPPORTED
    assert lib.kvs_layer_distance(p, 1, 2, 12, 0, p, p, p, p, 1 << 30, None) == kb.KVS_ERR_UNSUPPORTED
    assert lib.kvs_layer_distance(p, 0, 2, 8, 0, p, p, p, p, 1 << 30, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_layer_distance(p, 1, 2, 8, 0, p, p, p, p, 16, None) == kb.KVS_ERR_INVALID_ARG


def test_noalloc_entry_point_refuses_shapes_beyond_its_scratch():
    """Decided on the host, before the device is asked for anything: the built-in scratch has a fixed
    size, and a shape whose workspace need exceeds it is refused with the reason."""
    lib = kb.lib()
    assert lib.kvs_noalloc_scratch_bytes() == 8 << 20
    wide = kb.kvs_desc(2, 2, 16, 1, 128, kb.KVS_BF16, 16, 1 << 16, 1 << 16)
    assert 0 < lib.kvs_workspace_bytes(C.byref(wide), 64, 1) <= lib.kvs_noalloc_scratch_bytes()
    big = kb.kvs_store(wide, 1, 1, 1, None, 1, 1)                 # never dereferenced: the size check comes first
    assert lib.kvs_testing_force_split_tokens(64) == kb.KVS_OK    # 64-token splits of a 2^20-token context: far more partial states
    try:
        assert lib.kvs_workspace_bytes(C.byref(wide), 64, 1) > lib.kvs_noalloc_scratch_bytes()
        assert lib.kvs_decode_attention_noalloc(C.byref(big), 0, 1, 1, 64, 1, None) == kb.KVS_ERR_CAPACITY
        assert "scratch" in kb.last_error()
    finally:
        assert lib.kvs_testing_force_split_tokens(0) == kb.KVS_OK
    assert lib.kvs_decode_attention_noalloc(None, 0, 1, 1, 64, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention_noalloc(C.byref(big), 0, 1, 1, 0, 1, None) == kb.KVS_ERR_INVALID_ARG
    assert lib.kvs_decode_attention_noalloc(C.byref(kb.kvs_store(kb.kvs_desc(2, 2, 16, 1, 96, kb.KVS_BF16, 16, 64, 64), 1, 1, 1, None, 1, 1)),
                                            0, 1, 1, 1, 1, None) == kb.KVS_ERR_INVALID_ARG


def test_token_shares_of_a_decode_launch_partition_the_line():
    """The plan the decode kernel derives on the device, against brute force: n shares tile the line
    of octets without gap or overlap, share i begins at floor(total * i / n) (so the shares differ by
    at most one octet; a line shorter than n goes to the first workgroups, one octet each), and the
    owner look-up inverts them."""
    lib = kb.lib()
    first, count = C.c_int(0), C.c_int(0)
    for n in (1, 2, 7, 8, 256, 3000, 65535):
        for total in list(range(0, 40)) + [255, 256, 257, 511, 2720, 8192, 10240, 65537, (1 << 25) - 1]:
            # a line shorter than n: one octet for each of the first `total` workgroups, so that no empty share
            # lies between two that hold parts of one segment
            bound = (lambda i: total * i // n) if total >= n else (lambda i: min(i, total))
            probe = range(n) if n <= 256 else list(range(0, n, max(1, n // 97))) + [n - 1]
            sizes = []
            for i in probe:
                assert lib.kvs_testing_flat_share(i, n, total, C.byref(first), C.byref(count)) == kb.KVS_OK
                assert first.value == bound(i) and first.value + count.value == bound(i + 1)
                sizes.append(count.value)
            assert max(sizes) - min(sizes) <= 1
            step = max(1, total // 300)
            for o in list(range(0, total, step)) + [total - 1] * (total > 0):
                i = lib.kvs_testing_flat_owner(o, n, total)
                assert 0 <= i < n and bound(i) <= o < bound(i + 1), (n, total, o, i)
            assert lib.kvs_testing_flat_owner(total, n, total) == -1
    assert lib.kvs_testing_flat_share(3, 3, 10, C.byref(first), C.byref(count)) == kb.KVS_ERR_INVALID_ARG
