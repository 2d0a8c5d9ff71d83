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

// The same for a page index that is uniform over the wavefront, as a scalar load whatever the
// compiler can prove about the stores around it: the table is read through the constant address
// space (no launch writes it).  A vector load would join the queue of the page loads in flight,
// and waiting for it would drain them.
__device__ __forceinline__ int safe_block_of_uniform(const StoreView& st, int b, int page)
{
    typedef const int __attribute__((address_space(4))) * table_ptr;
    const size_t idx = (size_t)b * st.max_blocks_per_seq + page;
    const int blk = st.block_table ? reinterpret_cast<table_ptr>(reinterpret_cast<size_t>(st.block_table))[idx] : (int)idx;
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

// The same for the fp8 store (one byte per element).  A lane's 16-byte load covers two 32-deep
// contraction steps of K (8 channels each), or four 16-channel tiles of V (4 tokens each).
__device__ __forceinline__ int k_index_fp8(int t, int c)
{
    return ((((c >> 6) * 4 + ((c & 31) >> 3)) * 16 + t) * 16) + ((c >> 5) & 1) * 8 + (c & 7);
}
__device__ __forceinline__ int v_index_fp8(int t, int c)
{
    return ((((c >> 6) * 4 + (t >> 2)) * 16 + (c & 15)) * 16) + ((c >> 4) & 3) * 4 + (t & 3);
}

// bf16 bit pattern -> E4M3 code: round to nearest, ties to even, saturating at +-448; NaN -> NaN.
// Integer arithmetic on the bit pattern (exponent rebias 127 -> 7 is -120; 7 -> 3 mantissa bits),
// so the result does not depend on any conversion instruction's mode.
__device__ __forceinline__ unsigned bf16_to_e4m3(unsigned h)
{
    const unsigned sign = (h >> 8) & 0x80u, mag = h & 0x7fffu;
    if (mag > 0x7f80u) return sign | 0x7fu;                       // NaN
    if (mag >= 0x43e0u) return sign | 0x7eu;                      // >= 448 (and infinity): saturate
    if (mag >= (121u << 7)) {                                     // >= 2^-6: normal in the target
        const unsigned r = (mag + 7u + ((mag >> 4) & 1u)) >> 4;   // drop 4 mantissa bits, nearest even; may carry
        return sign | (r - (120u << 3));
    }
    // below 2^-6 the target is m * 2^-9, m = 0..8 (8 is the code of 2^-6 itself)
    const float f = __uint_as_float(mag << 16) * 512.f;
    return sign | (unsigned)__builtin_rintf(f);
}

// E4M3 code -> bf16 bit pattern (exact).
__device__ __forceinline__ unsigned e4m3_to_bf16(unsigned b)
{
    const unsigned sign = (b & 0x80u) << 8, em = b & 0x7fu;
    if (em == 0x7fu) return sign | 0x7fc0u;
    const unsigned e = em >> 3, m = em & 7u;
    if (e) return sign | ((e + 120u) << 7) | (m << 4);
    if (!m) return sign;
    const unsigned p = 31u - __builtin_clz(m);                    // m * 2^-9 = 2^(p-9) * (m / 2^p)
    return sign | ((p + 118u) << 7) | ((m << (7u - p)) & 0x7fu);
}

}  // namespace
}  // namespace kvs
