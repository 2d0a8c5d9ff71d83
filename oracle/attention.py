"""ctypes front end of the C oracle: shared-KV attention, append, layer distance.

Test infrastructure only.  The arithmetic lives in kvs_oracle.c; this file only marshals
numpy arrays.  A layer's cache is either contiguous, shape [B, T_cap, Hkv, d], or paged,
shape [num_blocks, block_tokens, Hkv, d] with a block table [B, max_blocks_per_seq].
Element type is float32, or uint16 holding bf16 bit patterns.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_shared_attention.restype = C.c_int
        L.orc_shared_attention.argtypes = [
            C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
            C.c_void_p, C.c_int, C.c_int, C.c_int64,
            C.c_void_p, C.c_int, C.c_void_p,
            C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
            C.c_void_p, C.c_void_p]
        L.orc_layer_distance.restype = C.c_int
        L.orc_layer_distance.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_num_threads.restype = C.c_int
        _LIB = L
    return _LIB


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"oracle arrays are float32 or uint16 (bf16 bits), got {a.dtype}")


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def shared_attention(layer, share_map, K_layers, V_layers, q, start_pos,
                     block_table=None, return_probs=False):
    """Attention of `layer` under `share_map` for q [B, T_new, Hq, d] (Sec. 3.2).

    Query row i of sequence b sees keys 0..start_pos[b]+i of the cache of layer
    share_map[layer].  Returns float64 [B, T_new, Hq, d] (and the softmax weights
    [B, T_new, Hq, T_cap] when asked).
    """
    share_map = np.ascontiguousarray(share_map, dtype=np.int32)
    L = share_map.shape[0]
    q = np.ascontiguousarray(q)
    B, T_new, Hq, d = q.shape
    start_pos = np.ascontiguousarray(start_pos, dtype=np.int32)
    assert start_pos.shape == (B,)
    ref = next(k for k in K_layers if k is not None)
    kv_code = _dtype_code(ref)
    Hkv = ref.shape[2]
    assert ref.shape[3] == d
    keep = []
    kp = (C.c_void_p * L)()
    vp = (C.c_void_p * L)()
    for l in range(L):
        for arr, dst in ((K_layers[l], kp), (V_layers[l], vp)):
            if arr is None:
                dst[l] = None
                continue
            assert arr.flags["C_CONTIGUOUS"] and arr.shape == ref.shape and arr.dtype == ref.dtype
            keep.append(arr)
            dst[l] = arr.ctypes.data
    if block_table is None:
        assert ref.shape[0] == B
        T_cap, bt, max_blocks, block_tokens = ref.shape[1], None, 0, 0
    else:
        bt = np.ascontiguousarray(block_table, dtype=np.int32)
        assert bt.shape[0] == B
        max_blocks, block_tokens = bt.shape[1], ref.shape[1]
        T_cap = max_blocks * block_tokens
        assert bt.min() >= 0 and bt.max() < ref.shape[0]
    out = np.zeros((B, T_new, Hq, d), dtype=np.float64)
    probs = np.zeros((B, T_new, Hq, T_cap), dtype=np.float64) if return_probs else None
    rc = lib().orc_shared_attention(
        int(layer), _ptr(share_map), L, C.cast(kp, C.c_void_p), C.cast(vp, C.c_void_p), kv_code,
        _ptr(bt), max_blocks, block_tokens, T_cap,
        _ptr(q), _dtype_code(q), _ptr(start_pos), B, T_new, Hq, Hkv, d,
        _ptr(out), _ptr(probs))
    if rc != 0:
        raise ValueError(f"orc_shared_attention rejected its arguments (rc={rc})")
    return (out, probs) if return_probs else out


def decode_attention(layer, share_map, K_layers, V_layers, q, seq_lens,
                     block_table=None, return_probs=False):
    """One decode step: q [B, Hq, d]; seq_lens counts the token appended this step."""
    q = np.ascontiguousarray(q)
    seq_lens = np.asarray(seq_lens, dtype=np.int64)
    r = shared_attention(layer, share_map, K_layers, V_layers, q[:, None],
                         (seq_lens - 1).astype(np.int32), block_table, return_probs)
    if return_probs:
        return r[0][:, 0], r[1][:, 0]
    return r[:, 0]


def append_kv(layer, share_map, K_layers, V_layers, k_new, v_new, start_pos, block_table=None):
    """Write k_new/v_new [B, T_new, Hkv, d] at positions start_pos[b]+i of `layer`'s cache.

    A layer whose cache is replaced by a donor's stores nothing (Sec. 3.2; the "Layer"
    column of the main results table counts only layers whose KV is computed).
    Returns True if rows were written.
    """
    if share_map[layer] != layer:
        return False
    K, V = K_layers[layer], V_layers[layer]
    B, T_new = k_new.shape[:2]
    for b in range(B):
        for i in range(T_new):
            j = int(start_pos[b]) + i
            if block_table is None:
                K[b, j] = k_new[b, i]
                V[b, j] = v_new[b, i]
            else:
                bs = K.shape[1]
                blk = int(block_table[b, j // bs])
                K[blk, j % bs] = k_new[b, i]
                V[blk, j % bs] = v_new[b, i]
    return True


def layer_distance(kv):
    """kv [S, L, 2, N] -> (dK2, dV2, D), each float64 [L, L] (Sec. 3.1.2)."""
    kv = np.ascontiguousarray(kv)
    S, L, two, N = kv.shape
    assert two == 2
    dK2 = np.zeros((L, L)); dV2 = np.zeros((L, L)); D = np.zeros((L, L))
    rc = lib().orc_layer_distance(_ptr(kv), _dtype_code(kv), S, L, N, _ptr(dK2), _ptr(dV2), _ptr(D))
    if rc != 0:
        raise ValueError(f"orc_layer_distance failed (rc={rc})")
    return dK2, dV2, D
