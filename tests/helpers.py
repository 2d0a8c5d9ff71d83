"""Shared scaffolding of the GPU parity tests: builds one workload on both sides.

The GPU store is filled through kvs_append_kv (so the layout transform is part of what is
tested); the oracle gets the same rounded values as plain contiguous arrays.
"""
import numpy as np
import torch

from paper_2410_18517_amd import inputs

REL_L2_ATTENTION = 5e-3      # max relative L2 error per output vector (bf16 and fp32 stores)
REL_DISTANCE = 1e-4          # relative Frobenius error of the fp32 distance matrix


def rel_l2_rows(got: np.ndarray, want: np.ndarray):
    """Per-vector relative L2 error over the last axis; zero rows must match exactly."""
    got = got.astype(np.float64)
    num = np.sqrt(((got - want) ** 2).sum(-1))
    den = np.sqrt((want ** 2).sum(-1))
    assert np.all(num[den == 0] == 0), "a row the oracle defines as zero is not zero"
    return np.where(den > 0, num / np.where(den > 0, den, 1), 0.0)


_FP8_LUT = None


def stored_fp8(bits: np.ndarray) -> np.ndarray:
    """What an fp8 slot holds of bf16 rows (bit patterns in, bit patterns of the stored values out):
    the storage oracle's rounding, applied to all 65536 bf16 patterns once and then looked up;
    every E4M3 value is exactly a bf16 value."""
    global _FP8_LUT
    if _FP8_LUT is None:
        from oracle.fp8 import round_e4m3
        with np.errstate(invalid="ignore"):                       # signalling NaN patterns among the inputs
            every = (np.arange(1 << 16, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
        _FP8_LUT = (round_e4m3(every).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    return _FP8_LUT[bits]


class Case:
    """One model-shaped workload: share map, page table, caches of the layers that keep one.
    dtype "fp8": rows and queries are bf16, the oracle-side arrays hold the values as stored."""

    def __init__(self, kb, L, Hq, Hkv, d, B, dtype, capacity, share_map, paged=True, seed=0,
                 fill_layers=None, fill_tokens=None, spare_blocks=3):
        self.kb, self.L, self.Hq, self.Hkv, self.d, self.B = kb, L, Hq, Hkv, d, B
        self.dtype, self.capacity, self.seed = dtype, capacity, seed
        self.row_dtype = "bf16" if dtype == "fp8" else dtype
        self.share_map = np.asarray(share_map, np.int32)
        self.max_blocks = (capacity + 15) // 16
        self.num_blocks = B * self.max_blocks + (spare_blocks if paged else 0)
        self.block_table = (inputs.make_block_table(B, self.max_blocks, self.num_blocks, seed)
                            if paged else None)
        self.store = kb.KVStore(self.share_map, Hq, Hkv, d, dtype, self.num_blocks, self.max_blocks,
                                block_table=self.block_table)
        self.K = [None] * L          # oracle-side arrays, [B, T_fill, Hkv, d]
        self.V = [None] * L
        fill_tokens = capacity if fill_tokens is None else fill_tokens
        own = [l for l in range(L) if self.share_map[l] == l]
        for l in (own if fill_layers is None else fill_layers):
            assert self.share_map[l] == l
            self.fill_layer(l, fill_tokens)

    def kv_chunk(self, layer, b, T):
        """The seeded K, V [T, Hkv, d] of (layer, sequence b); regenerable on demand."""
        k = inputs.normal((T, self.Hkv, self.d), self.seed, layer, b, 0, dtype=self.row_dtype)
        v = inputs.normal((T, self.Hkv, self.d), self.seed, layer, b, 1, dtype=self.row_dtype)
        return k, v

    def fill_layer(self, layer, T, keep_oracle_copy=True):
        chunks = inputs.parallel_map(lambda b: self.kv_chunk(layer, b, T), range(self.B))
        k = torch.stack([c[0] for c in chunks])
        v = torch.stack([c[1] for c in chunks])
        st = self.kb.kvs_append_kv(self.store, layer, k.cuda(), v.cuda(),
                                   torch.zeros(self.B, dtype=torch.int32, device="cuda"))
        assert st == self.kb.KVS_OK
        if keep_oracle_copy:
            self.K[layer] = inputs.to_oracle_array(k)
            self.V[layer] = inputs.to_oracle_array(v)
            if self.dtype == "fp8":
                self.K[layer], self.V[layer] = stored_fp8(self.K[layer]), stored_fp8(self.V[layer])

    def q(self, layer, rows=None):
        shape = (self.B, self.Hq, self.d) if rows is None else (self.B, rows, self.Hq, self.d)
        return inputs.normal(shape, self.seed, layer, 9999, dtype=self.row_dtype)
