// Device-side helpers shared by the kernels that address the paged, slot-indexed KV store
// (gfx950): the strategy's layer -> donor -> slot substitution (paper Sec. 3.2), the page table
// and the in-page operand order of the bf16 store.
#pragma once
#include <hip/hip_runtime.h>

#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kPageTokens = 16;

__device__ __forceinline__ int resolve_slot(const StoreView& st)
{
    // the strategy's substitution: a layer reads the cache of its donor (itself if none)
    int donor = st.share_map[st.layer];
    donor = donor < 0 ? 0 : (donor >= st.L ? st.L - 1 : donor);
    const int slot = st.slot_of_layer[donor];
    return slot < 0 ? 0 : (slot >= st.n_slots ? st.n_slots - 1 : slot);
}

// Physical block of logical page `page` of sequence b.
__device__ __forceinline__ int block_of(const StoreView& st, int b, int page)
{
    const size_t idx = (size_t)b * st.max_blocks_per_seq + page;
    return st.block_table ? st.block_table[idx] : (int)idx;   // contiguous: the host checked B * max_blocks <= num_blocks
}

// Same, forced into the pool: a corrupt table entry must not turn into a wild read.
__device__ __forceinline__ int safe_block_of(const StoreView& st, int b, int page)
{
    const int blk = block_of(st, b, page);
    return blk < 0 ? 0 : (blk >= st.num_blocks ? st.num_blocks - 1 : blk);
}

// Element offset of the K page of (slot, block, kv head); the V page follows it.
__device__ __forceinline__ size_t page_offset(const StoreView& st, int slot, int blk, int g)
{
    return (((size_t)slot * st.num_blocks + blk) * st.Hkv + g) * 2 * (size_t)(kPageTokens * st.head_dim);
}

// In-page element index of (token t, channel c) for the bf16 store.
__device__ __forceinline__ int k_index_bf16(int t, int c)
{
    return (((c >> 5) * 4 + ((c & 31) >> 3)) * 16 + t) * 8 + (c & 7);
}
__device__ __forceinline__ int v_index_bf16(int t, int c)
{
    return ((((c >> 5) * 4 + (t >> 2)) * 16 + (c & 15)) * 2 + ((c >> 4) & 1)) * 4 + (t & 3);
}

}  // namespace
}  // namespace kvs
