"""ctypes binding of libkvs.so: same names as the C ABI, argument marshalling only.

torch supplies device memory and the current stream; every step of the path (append, share-map
resolution, attention, combine, distance) runs in the library's HIP kernels.  There is no CPU or
torch fallback: if the shared library is missing or cannot be loaded, importing it raises.
"""
import ctypes as C
import os

import numpy as np
import torch  # imported before the library so both use the same HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
# KVS_LIBRARY names another build of the same library (the sanitizer run of tests/sanitize_cpu.py)
LIB_PATH = os.environ.get("KVS_LIBRARY") or os.path.join(_HERE, "libkvs.so")

KVS_OK, KVS_NOOP = 0, 1
KVS_ERR_INVALID_ARG, KVS_ERR_BAD_MAP, KVS_ERR_CAPACITY = -1, -2, -3
KVS_ERR_TARGET_UNREACHED, KVS_ERR_UNSUPPORTED, KVS_ERR_HIP = -4, -5, -6
KVS_F32, KVS_BF16, KVS_FP8 = 0, 1, 2
KVS_BLOCK_TOKENS = 16

EXPORTS = [
    "kvs_last_error", "kvs_build_share_map", "kvs_validate_share_map", "kvs_slots_from_share_map",
    "kvs_store_bytes", "kvs_workspace_bytes", "kvs_append_kv", "kvs_gather_kv",
    "kvs_decode_attention", "kvs_prefill_attention", "kvs_testing_force_split_tokens",
    "kvs_layer_distance", "kvs_distance_workspace_bytes", "kvs_avg_cos_sim", "kvs_cos_sim_workspace_bytes",
    "kvs_project_append_kv", "kvs_project_workspace_bytes",
    "kvs_compact_kv", "kvs_append_kv_per_head", "kvs_decode_attention_per_head", "kvs_decode_step",
    "kvs_check_store", "kvs_decode_attention_noalloc", "kvs_noalloc_scratch_bytes",
    "kvs_testing_flat_share", "kvs_testing_flat_owner", "kvs_testing_set_decode_workgroups",
]


class KvsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"kvs status {status}: {message}")
        self.status = status


class kvs_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("L", "n_slots", "Hq", "Hkv", "head_dim", "dtype",
                                         "block_tokens", "num_blocks", "max_blocks_per_seq")]


class kvs_store(C.Structure):
    _fields_ = [("desc", kvs_desc), ("pool", C.c_void_p), ("share_map", C.c_void_p),
                ("slot_of_layer", C.c_void_p), ("block_table", C.c_void_p),
                ("host_share_map", C.c_void_p), ("host_slot_of_layer", C.c_void_p)]


ACCEPT_FN = C.CFUNCTYPE(C.c_int, C.POINTER(C.c_int32), C.c_int, C.c_void_p)

_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(hipcc, gfx950). There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        L.kvs_last_error.restype = C.c_char_p
        L.kvs_store_bytes.restype = C.c_size_t
        L.kvs_store_bytes.argtypes = [C.POINTER(kvs_desc)]
        L.kvs_workspace_bytes.restype = C.c_size_t
        L.kvs_workspace_bytes.argtypes = [C.POINTER(kvs_desc), C.c_int, C.c_int]
        L.kvs_distance_workspace_bytes.restype = C.c_size_t
        L.kvs_distance_workspace_bytes.argtypes = [C.c_int]
        L.kvs_build_share_map.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, ACCEPT_FN, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_validate_share_map.argtypes = [C.c_void_p, C.c_int]
        L.kvs_slots_from_share_map.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.kvs_append_kv.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_int, C.c_int, C.c_void_p]
        L.kvs_append_kv_per_head.argtypes = L.kvs_append_kv.argtypes
        L.kvs_compact_kv.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.kvs_gather_kv.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_void_p, C.c_void_p, C.c_void_p]
        L.kvs_decode_attention.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                           C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvs_decode_attention_per_head.argtypes = L.kvs_decode_attention.argtypes
        L.kvs_decode_attention_noalloc.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                   C.c_void_p, C.c_void_p]
        L.kvs_noalloc_scratch_bytes.restype = C.c_size_t
        L.kvs_noalloc_scratch_bytes.argtypes = []
        L.kvs_decode_step.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvs_prefill_attention.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                            C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvs_testing_force_split_tokens.argtypes = [C.c_int]
        L.kvs_testing_flat_share.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.kvs_testing_flat_owner.argtypes = [C.c_int, C.c_int, C.c_int]
        L.kvs_testing_set_decode_workgroups.argtypes = [C.c_int]
        L.kvs_check_store.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_void_p]
        L.kvs_layer_distance.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_size_t, C.c_int, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvs_project_append_kv.argtypes = [C.POINTER(kvs_store), C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvs_project_workspace_bytes.restype = C.c_size_t
        L.kvs_project_workspace_bytes.argtypes = [C.POINTER(kvs_desc), C.c_int, C.c_int, C.c_int]
        L.kvs_cos_sim_workspace_bytes.restype = C.c_size_t
        L.kvs_cos_sim_workspace_bytes.argtypes = [C.c_int]
        L.kvs_avg_cos_sim.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_size_t, C.c_int, C.c_int, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
        _lib = L
    return _lib


def last_error() -> str:
    return lib().kvs_last_error().decode()


def _check(status, ok=(KVS_OK,)):
    if status not in ok:
        raise KvsError(status, last_error())
    return status


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


# ------------------------------------------------------------------ strategy (host)

def kvs_build_share_map(dist, target_shared, order=0, accept=None):
    """(status, share_map, slot_of_layer, n_slots, n_shared); raises only on invalid arguments."""
    dist = np.ascontiguousarray(dist, dtype=np.float32)
    L = dist.shape[0]
    share, slot = np.zeros(L, np.int32), np.zeros(L, np.int32)
    n_slots, n_shared = C.c_int32(0), C.c_int32(0)
    if accept is None:
        cb = C.cast(None, ACCEPT_FN)
    else:
        cb = ACCEPT_FN(lambda m, n, _u: int(bool(accept([m[i] for i in range(n)]))))
    st = lib().kvs_build_share_map(_np_ptr(dist), L, int(target_shared), int(order), cb, None,
                                   _np_ptr(share), _np_ptr(slot), C.byref(n_slots), C.byref(n_shared))
    _check(st, ok=(KVS_OK, KVS_ERR_TARGET_UNREACHED))
    return st, share, slot, n_slots.value, n_shared.value


def kvs_validate_share_map(share_map) -> int:
    m = _i32(share_map)
    return lib().kvs_validate_share_map(_np_ptr(m), len(m))


def kvs_slots_from_share_map(share_map):
    m = _i32(share_map)
    slot, n = np.zeros(len(m), np.int32), C.c_int32(0)
    _check(lib().kvs_slots_from_share_map(_np_ptr(m), len(m), _np_ptr(slot), C.byref(n)))
    return slot, n.value


def kvs_testing_force_split_tokens(tokens: int):
    _check(lib().kvs_testing_force_split_tokens(int(tokens)))


# ------------------------------------------------------------------ store

_TORCH_DTYPE = {KVS_F32: torch.float32, KVS_BF16: torch.bfloat16, KVS_FP8: torch.bfloat16}   # of rows and queries


class KVStore:
    """Device buffers of one slot-indexed paged KV store plus the kvs_store struct over them."""

    def __init__(self, share_map, Hq, Hkv, head_dim, dtype, num_blocks, max_blocks_per_seq,
                 block_table=None, device="cuda:0", zero_fill=False):
        self.device = torch.device(device)
        self.host_share_map = _i32(share_map)
        L = len(self.host_share_map)
        self.host_slot_of_layer, n_slots = kvs_slots_from_share_map(self.host_share_map)
        self.dtype = (KVS_FP8 if dtype in ("fp8", KVS_FP8) else
                      KVS_BF16 if dtype in ("bf16", KVS_BF16, torch.bfloat16) else KVS_F32)
        self.desc = kvs_desc(L, n_slots, Hq, Hkv, head_dim, self.dtype, KVS_BLOCK_TOKENS,
                             num_blocks, max_blocks_per_seq)
        nbytes = lib().kvs_store_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise KvsError(KVS_ERR_UNSUPPORTED, last_error())
        alloc = torch.zeros if zero_fill else torch.empty
        self.pool = alloc(nbytes, dtype=torch.uint8, device=self.device)
        self.share_map = torch.from_numpy(self.host_share_map).to(self.device)
        self.slot_of_layer = torch.from_numpy(self.host_slot_of_layer).to(self.device)
        self.block_table = None
        if block_table is not None:
            bt = _i32(block_table)
            assert bt.ndim == 2 and bt.shape[1] == max_blocks_per_seq
            self.block_table = torch.from_numpy(bt).to(self.device)
        self.c = kvs_store(self.desc, self.pool.data_ptr(), self.share_map.data_ptr(),
                           self.slot_of_layer.data_ptr(),
                           self.block_table.data_ptr() if self.block_table is not None else None,
                           self.host_share_map.ctypes.data, self.host_slot_of_layer.ctypes.data)
        self._ws = None

    @property
    def torch_dtype(self):
        return _TORCH_DTYPE[self.dtype]

    def workspace(self, B, rows):
        need = lib().kvs_workspace_bytes(C.byref(self.desc), int(B), int(rows))
        if need == 0:
            raise KvsError(KVS_ERR_INVALID_ARG, last_error())
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.zeros(need, dtype=torch.uint8, device=self.device)
        return self._ws


def _dev_i32(x, device):
    if isinstance(x, torch.Tensor):
        assert x.dtype == torch.int32 and x.is_cuda and x.is_contiguous()
        return x
    return torch.from_numpy(_i32(x)).to(device)


def kvs_append_kv(store: KVStore, layer, k_new, v_new, start_pos) -> int:
    """k_new, v_new: device [B, T_new, Hkv, d] of the store dtype. Returns KVS_OK or KVS_NOOP."""
    assert k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
    assert k_new.dtype == store.torch_dtype and v_new.dtype == store.torch_dtype
    B, T_new = k_new.shape[:2]
    assert tuple(k_new.shape) == (B, T_new, store.desc.Hkv, store.desc.head_dim) == tuple(v_new.shape)
    sp = _dev_i32(start_pos, store.device)
    assert sp.numel() == B
    return _check(lib().kvs_append_kv(C.byref(store.c), int(layer), k_new.data_ptr(), v_new.data_ptr(),
                                      sp.data_ptr(), B, T_new, _stream()), ok=(KVS_OK, KVS_NOOP))


def kvs_append_kv_per_head(store: KVStore, layer, k_new, v_new, pos) -> int:
    """As kvs_append_kv with a write position per (sequence, kv head): pos device/host int32 [B, Hkv]."""
    assert k_new.is_cuda and k_new.is_contiguous() and v_new.is_contiguous()
    assert k_new.dtype == store.torch_dtype and v_new.dtype == store.torch_dtype
    B, T_new = k_new.shape[:2]
    assert tuple(k_new.shape) == (B, T_new, store.desc.Hkv, store.desc.head_dim) == tuple(v_new.shape)
    sp = _dev_i32(pos, store.device)
    assert sp.numel() == B * store.desc.Hkv
    return _check(lib().kvs_append_kv_per_head(C.byref(store.c), int(layer), k_new.data_ptr(), v_new.data_ptr(),
                                               sp.data_ptr(), B, T_new, _stream()), ok=(KVS_OK, KVS_NOOP))


def kvs_compact_kv(store: KVStore, layer, keep_idx, keep_count) -> int:
    """keep_idx: int32 [B, Hkv, max_keep] increasing positions; keep_count: int32 [B, Hkv]."""
    idx = _dev_i32(keep_idx, store.device)
    cnt = _dev_i32(keep_count, store.device)
    B, Hkv, max_keep = idx.shape
    assert Hkv == store.desc.Hkv and tuple(cnt.shape) == (B, Hkv)
    return _check(lib().kvs_compact_kv(C.byref(store.c), int(layer), idx.data_ptr(), cnt.data_ptr(),
                                       int(max_keep), int(B), _stream()), ok=(KVS_OK, KVS_NOOP))


def kvs_project_append_kv(store: KVStore, layer, x, w_k, w_v, start_pos, rope_cos=None, rope_sin=None,
                          workspace=None) -> int:
    """x: device bf16 [B, T_new, hidden]; w_k, w_v: device bf16 [Hkv*d, hidden]; rope tables device fp32
    [positions, d/2] or None. Returns KVS_OK or KVS_NOOP."""
    for t in (x, w_k, w_v):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16
    B, T_new, hidden = x.shape
    n_out = store.desc.Hkv * store.desc.head_dim
    assert tuple(w_k.shape) == (n_out, hidden) == tuple(w_v.shape)
    positions = 0
    if rope_cos is not None:
        assert rope_cos.is_cuda and rope_cos.dtype == torch.float32 and rope_cos.is_contiguous()
        assert rope_sin is not None and rope_sin.shape == rope_cos.shape and rope_sin.dtype == torch.float32
        assert rope_cos.shape[1] == store.desc.head_dim // 2
        positions = rope_cos.shape[0]
    sp = _dev_i32(start_pos, store.device)
    assert sp.numel() == B
    if workspace is None:
        need = lib().kvs_project_workspace_bytes(C.byref(store.desc), int(hidden), int(B), int(T_new))
        if need == 0:
            raise KvsError(KVS_ERR_INVALID_ARG, last_error())
        ws = getattr(store, "_proj_ws", None)
        if ws is None or ws.numel() < need:
            ws = store._proj_ws = torch.zeros(need, dtype=torch.uint8, device=store.device)
        workspace = ws
    return _check(lib().kvs_project_append_kv(
        C.byref(store.c), int(layer), x.data_ptr(), int(hidden), w_k.data_ptr(), w_v.data_ptr(),
        rope_cos.data_ptr() if rope_cos is not None else None,
        rope_sin.data_ptr() if rope_sin is not None else None, int(positions),
        sp.data_ptr(), int(B), int(T_new), workspace.data_ptr(), workspace.numel(), _stream()), ok=(KVS_OK, KVS_NOOP))


def kvs_check_store(store: KVStore, B):
    """Device tensor int32 [2]: (map entries that differ from the host copies, page-table entries out of range)."""
    report = torch.empty(2, dtype=torch.int32, device=store.device)
    _check(lib().kvs_check_store(C.byref(store.c), int(B), report.data_ptr(), _stream()))
    return report


def kvs_gather_kv(store: KVStore, layer, t0, T, B):
    shape = (B, T, store.desc.Hkv, store.desc.head_dim)
    k = torch.empty(shape, dtype=store.torch_dtype, device=store.device)
    v = torch.empty(shape, dtype=store.torch_dtype, device=store.device)
    _check(lib().kvs_gather_kv(C.byref(store.c), int(layer), int(t0), int(T), int(B),
                               k.data_ptr(), v.data_ptr(), _stream()))
    return k, v


def kvs_decode_attention(store: KVStore, layer, q, seq_lens, out=None, workspace=None):
    """q: device [B, Hq, d] of the store dtype; seq_lens: device int32 [B]. Returns fp32 [B, Hq, d]."""
    assert q.is_cuda and q.is_contiguous() and q.dtype == store.torch_dtype
    B = q.shape[0]
    assert tuple(q.shape) == (B, store.desc.Hq, store.desc.head_dim)
    sl = _dev_i32(seq_lens, store.device)
    assert sl.numel() == B
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=store.device)
    ws = workspace if workspace is not None else store.workspace(B, 1)
    _check(lib().kvs_decode_attention(C.byref(store.c), int(layer), q.data_ptr(), sl.data_ptr(), B,
                                      out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return out


def kvs_decode_attention_noalloc(store: KVStore, layer, q, seq_lens, out):
    """kvs_decode_attention on the library's built-in scratch: no workspace; `out` is the caller's, fp32 [B, Hq, d]."""
    assert q.is_cuda and q.is_contiguous() and q.dtype == store.torch_dtype
    B = q.shape[0]
    assert tuple(q.shape) == (B, store.desc.Hq, store.desc.head_dim)
    assert out.is_cuda and out.is_contiguous() and out.dtype == torch.float32 and tuple(out.shape) == tuple(q.shape)
    sl = _dev_i32(seq_lens, store.device)
    assert sl.numel() == B
    _check(lib().kvs_decode_attention_noalloc(C.byref(store.c), int(layer), q.data_ptr(), sl.data_ptr(), B,
                                              out.data_ptr(), _stream()))
    return out


def kvs_decode_step(store: KVStore, layer, q, k_new, v_new, seq_lens, out=None, workspace=None):
    """Append of this step's token and decode attention in one call; seq_lens counts the new token."""
    assert q.is_cuda and q.is_contiguous() and q.dtype == store.torch_dtype
    B = q.shape[0]
    assert tuple(q.shape) == (B, store.desc.Hq, store.desc.head_dim)
    for t in (k_new, v_new):
        assert t.is_cuda and t.is_contiguous() and t.dtype == store.torch_dtype
        assert tuple(t.shape) == (B, 1, store.desc.Hkv, store.desc.head_dim)
    sl = _dev_i32(seq_lens, store.device)
    assert sl.numel() == B
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=store.device)
    ws = workspace if workspace is not None else store.workspace(B, 1)
    _check(lib().kvs_decode_step(C.byref(store.c), int(layer), q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                 sl.data_ptr(), B, out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return out


def kvs_decode_attention_per_head(store: KVStore, layer, q, kv_lens, out=None, workspace=None):
    """As kvs_decode_attention over a sparsified slot: kv_lens int32 [n_slots, B, Hkv]."""
    assert q.is_cuda and q.is_contiguous() and q.dtype == store.torch_dtype
    B = q.shape[0]
    assert tuple(q.shape) == (B, store.desc.Hq, store.desc.head_dim)
    kl = _dev_i32(kv_lens, store.device)
    assert tuple(kl.shape) == (store.desc.n_slots, B, store.desc.Hkv)
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=store.device)
    ws = workspace if workspace is not None else store.workspace(B, 1)
    _check(lib().kvs_decode_attention_per_head(C.byref(store.c), int(layer), q.data_ptr(), kl.data_ptr(), B,
                                               out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return out


def kvs_prefill_attention(store: KVStore, layer, q, start_pos, out=None, workspace=None):
    """q: device [B, T_new, Hq, d]; row i of sequence b sits at position start_pos[b] + i."""
    assert q.is_cuda and q.is_contiguous() and q.dtype == store.torch_dtype
    B, T_new = q.shape[:2]
    assert tuple(q.shape) == (B, T_new, store.desc.Hq, store.desc.head_dim)
    sp = _dev_i32(start_pos, store.device)
    assert sp.numel() == B
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=store.device)
    ws = workspace if workspace is not None else store.workspace(B, T_new)
    _check(lib().kvs_prefill_attention(C.byref(store.c), int(layer), q.data_ptr(), sp.data_ptr(), B, T_new,
                                       out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return out


# ------------------------------------------------------------------ calibration distance

def kvs_layer_distance(kv_samples, workspace=None):
    """kv_samples: device [S, L, 2, N] (bf16 or fp32). Returns fp32 (dK2, dV2, D), each [L, L]."""
    assert kv_samples.is_cuda and kv_samples.is_contiguous() and kv_samples.dim() == 4
    S, L, two, N = kv_samples.shape
    assert two == 2
    dtype = KVS_BF16 if kv_samples.dtype == torch.bfloat16 else KVS_F32
    assert kv_samples.dtype in (torch.bfloat16, torch.float32)
    need = lib().kvs_distance_workspace_bytes(int(L))
    if need == 0:
        raise KvsError(KVS_ERR_UNSUPPORTED, last_error())
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=kv_samples.device)
    outs = [torch.empty(L, L, dtype=torch.float32, device=kv_samples.device) for _ in range(3)]
    _check(lib().kvs_layer_distance(kv_samples.data_ptr(), S, L, N, dtype, outs[0].data_ptr(),
                                    outs[1].data_ptr(), outs[2].data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), _stream()))
    return tuple(outs)


# ------------------------------------------------------------------ similarity test

def kvs_avg_cos_sim(hidden_shared, hidden_original, mode=0, workspace=None):
    """hidden_*: device [S, N] (bf16 or fp32), same shape and dtype. Returns a device fp32 scalar tensor."""
    a, b = hidden_shared, hidden_original
    assert a.is_cuda and b.is_cuda and a.is_contiguous() and b.is_contiguous()
    assert a.shape == b.shape and a.dtype == b.dtype and a.dim() == 2
    assert a.dtype in (torch.bfloat16, torch.float32)
    S, N = a.shape
    need = lib().kvs_cos_sim_workspace_bytes(int(S))
    if need == 0:
        raise KvsError(KVS_ERR_INVALID_ARG, last_error())
    if workspace is None:
        workspace = torch.zeros(need, dtype=torch.uint8, device=a.device)
    out = torch.empty(1, dtype=torch.float32, device=a.device)
    _check(lib().kvs_avg_cos_sim(a.data_ptr(), b.data_ptr(), S, N, KVS_BF16 if a.dtype == torch.bfloat16 else KVS_F32,
                                 int(mode), out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    return out
