"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Only data generation lives here: shapes, random draws, rounding of the draws to the storage
type, sharing strategies and page tables drawn from a seed.  None of the method's arithmetic
(attention, distances, strategy search) is in this module, and it imports neither the GPU
binding nor the CPU oracle.

The workloads stand in for the models the paper evaluates (Llama-2 7B/13B, InternLM2-20B;
Sec. 4.1) and for its calibration set (30 sentences of equal length, Sec. 4.3): only the
tensor shapes are taken from them; the contents are synthetic.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

SEED_BASE = 20241018
BLOCK_TOKENS = 16


@dataclass(frozen=True)
class Workload:
    name: str
    L: int                    # layers
    Hq: int                   # query heads
    Hkv: int                  # key/value heads
    d: int                    # head dimension
    B: int                    # sequences in the batch
    context: int              # tokens per sequence (upper bound when ragged)
    dtype: str                # "f32" or "bf16"
    n_shared: int             # layers that read a donor's cache
    min_context: Optional[int] = None   # set => seq lens uniform in [min_context, context]
    paged: bool = True
    prefill_rows: int = 0
    fixed_map: Optional[tuple] = None   # ((recipient, donor), ...) when the strategy is given

    @property
    def group(self):
        return self.Hq // self.Hkv

    @property
    def max_blocks_per_seq(self):
        return (self.context + BLOCK_TOKENS - 1) // BLOCK_TOKENS


WORKLOADS = {
    # 4 layers, 4/2 heads, d 64, fp32, one sequence of 128 tokens, layer 3 reads layer 1
    "tiny": Workload("tiny", 4, 4, 2, 64, 1, 128, "f32", 1, fixed_map=((3, 1),)),
    # Llama-2-7B shape
    "llama2-7b": Workload("llama2-7b", 32, 32, 32, 128, 8, 4096, "bf16", 8),
    # Llama-2-13B shape, plus a 64-row causal prefill chunk
    "llama2-13b": Workload("llama2-13b", 40, 40, 40, 128, 16, 2048, "bf16", 12, prefill_rows=64),
    # Llama-3-8B GQA shape at 32k context
    "llama3-8b-32k": Workload("llama3-8b-32k", 32, 32, 8, 128, 4, 32768, "bf16", 10),
    # 48 layers, group-of-6 GQA, ragged lengths (InternLM2-20B-like)
    "gqa48-ragged": Workload("gqa48-ragged", 48, 48, 8, 128, 32, 8192, "bf16", 14,
                             min_context=1024),
}


def _gen(*key) -> torch.Generator:
    """A CPU generator whose seed is a fixed function of SEED_BASE and the integer key."""
    s = SEED_BASE
    for k in key:
        s = (s * 1000003 + int(k) + 12345) % (2 ** 62)
    g = torch.Generator(device="cpu")
    g.manual_seed(s)
    return g


def normal(shape, *key, dtype="bf16") -> torch.Tensor:
    """N(0,1) draws as a CPU tensor of the storage type (bf16: rounded to nearest even)."""
    x = torch.randn(*shape, generator=_gen(*key), dtype=torch.float32)
    return x.to(torch.bfloat16) if dtype == "bf16" else x


def to_oracle_array(t: torch.Tensor) -> np.ndarray:
    """CPU view the oracle reads: float32 as is, bf16 as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.to(torch.float32).numpy()


def make_share_map(L: int, n_shared: int, *key, fixed=None) -> np.ndarray:
    """share_map[l] = donor layer of l (l itself if l keeps its own cache).

    Recipients are drawn among layers 1..L-1; each donor is drawn uniformly among the
    lower-indexed layers that keep their own cache, so donor < recipient and no donor is
    itself a recipient.
    """
    m = np.arange(L, dtype=np.int32)
    if fixed is not None:
        for r, dn in fixed:
            m[r] = dn
        return m
    g = _gen(*key, 77)
    perm = torch.randperm(L - 1, generator=g).numpy() + 1
    recipients = np.sort(perm[:n_shared])
    rset = set(int(r) for r in recipients)
    for r in recipients:
        cands = [l for l in range(int(r)) if l not in rset]
        m[r] = cands[int(torch.randint(len(cands), (1,), generator=g))]
    return m


def slots_of(share_map: np.ndarray):
    """Slot numbering used to size stores in the harness: own-cache layers in layer order."""
    L = len(share_map)
    slot = np.zeros(L, dtype=np.int32)
    n = 0
    for l in range(L):
        if share_map[l] == l:
            slot[l] = n
            n += 1
    for l in range(L):
        if share_map[l] != l:
            slot[l] = slot[share_map[l]]
    return slot, n


def make_block_table(B: int, max_blocks_per_seq: int, num_blocks: int, *key) -> np.ndarray:
    """[B, max_blocks_per_seq] distinct physical page ids: a seeded permutation, not identity."""
    assert num_blocks >= B * max_blocks_per_seq
    perm = torch.randperm(num_blocks, generator=_gen(*key, 991)).numpy().astype(np.int32)
    return perm[:B * max_blocks_per_seq].reshape(B, max_blocks_per_seq).copy()


def make_seq_lens(w: Workload, *key) -> np.ndarray:
    if w.min_context is None:
        return np.full(w.B, w.context, dtype=np.int32)
    g = _gen(*key, 313)
    return torch.randint(w.min_context, w.context + 1, (w.B,), generator=g).numpy().astype(np.int32)


def calibration_kv(S, L, Hkv, T, d, *key, noise=1.0, dtype="bf16") -> torch.Tensor:
    """Calibration caches [S, L, 2, Hkv*T*d] with per-layer scale and per-channel offsets.

    x = a_l * (beta_{l,kv,c} + noise * eps): a_l log-uniform in [0.5, 4], beta ~ N(0,1) per
    (layer, K|V, channel c < d), eps ~ N(0,1) iid.  Plain N(0,1) data would make all layer
    pairs equidistant; real caches differ in scale and channel offsets, which this imitates.
    """
    g = _gen(*key, 555)
    a = torch.exp(torch.empty(L).uniform_(np.log(0.5), np.log(4.0), generator=g))
    beta = torch.randn(L, 2, d, generator=g)
    out = torch.empty(S, L, 2, Hkv * T * d, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)

    def one_sample(s):
        if noise:
            eps = torch.randn(L, 2, Hkv * T, d, generator=_gen(*key, 556, s))
        else:
            eps = torch.zeros(L, 2, Hkv * T, d)
        x = a.view(L, 1, 1, 1) * (beta.view(L, 2, 1, d) + noise * eps)
        out[s] = x.reshape(L, 2, Hkv * T * d).to(out.dtype)

    parallel_map(one_sample, range(S))
    return out


def parallel_map(fn, items, workers=16):
    """Run independent draws on host threads (each has its own generator, so order is irrelevant)."""
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return list(ex.map(fn, items))
