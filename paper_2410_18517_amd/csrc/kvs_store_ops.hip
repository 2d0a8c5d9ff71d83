// Moving rows into, out of and inside the paged KV store (gfx950): append (one row per decode
// step, or page-wise for prefill chunks), gather, and the in-place compaction of a slot after an
// intra-layer method dropped tokens.  A layer that reads a donor's cache (paper Sec. 3.2) never
// gets here for writes: the host returns before any launch.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kvs_device.h"
#include "kvs_internal.h"

namespace kvs {
namespace {

// ------------------------------------------------------------------ append / gather
// One thread moves 8 consecutive channels (bf16) or 4 (fp32) of one (sequence, row, kv head).
template <bool kToStore>
__global__ void copy_rows_kernel(CopyArgs a)
{
    const StoreView& st = a.st;
    const int D = st.head_dim;
    const int per = st.dtype == 0 ? 4 : 8;       // rows are bf16 for the bf16 and fp8 stores, fp32 for the fp32 store
    const int chunks = D / per;
    const long total = (long)a.B * a.T * st.Hkv * chunks;
    const long tid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= total) return;
    const int ch = (int)(tid % chunks);
    const int g = (int)((tid / chunks) % st.Hkv);
    const int i = (int)((tid / ((long)chunks * st.Hkv)) % a.T);
    const int b = (int)(tid / ((long)chunks * st.Hkv * a.T));
    const long pos = (long)(a.start_pos ? a.start_pos[a.pos_per_head ? b * st.Hkv + g : b] + a.pos_bias : a.t0) + i;
    if (pos < 0 || pos >= (long)st.max_blocks_per_seq * kPageTokens) return;
    const int slot = resolve_slot(st);
    const int blk = block_of(st, b, (int)(pos / kPageTokens));
    if (blk < 0 || blk >= st.num_blocks) return;
    const int t = (int)(pos % kPageTokens);
    const size_t page = page_offset(st, slot, blk, g);
    const size_t row = (((size_t)b * a.T + i) * st.Hkv + g) * D + (size_t)ch * per;
    if (st.dtype == 2) {
        // fp8 store: 8 channels of a row are 8 bytes of the K page (one store) and 8 single bytes of
        // the V page; quantisation and its inverse are the integer routines of kvs_device.h
        unsigned char* kp = static_cast<unsigned char*>(st.pool) + page;
        unsigned char* vp = kp + kPageTokens * D;
        unsigned short* kr = static_cast<unsigned short*>(a.k) + row;
        unsigned short* vr = static_cast<unsigned short*>(a.v) + row;
        const int c0 = ch * 8;
        if (kToStore) {
            const uint4 kk = *reinterpret_cast<const uint4*>(kr), vv = *reinterpret_cast<const uint4*>(vr);
            const unsigned kw[4] = {kk.x, kk.y, kk.z, kk.w}, vw[4] = {vv.x, vv.y, vv.z, vv.w};
            unsigned lo = 0, hi = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                lo |= bf16_to_e4m3((kw[e >> 1] >> ((e & 1) * 16)) & 0xffffu) << (8 * e);
                hi |= bf16_to_e4m3((kw[2 + (e >> 1)] >> ((e & 1) * 16)) & 0xffffu) << (8 * e);
            }
            *reinterpret_cast<uint2*>(kp + k_index_fp8(t, c0)) = make_uint2(lo, hi);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                vp[v_index_fp8(t, c0 + e)] = (unsigned char)bf16_to_e4m3((vw[e >> 1] >> ((e & 1) * 16)) & 0xffffu);
        } else {
            const uint2 kb = *reinterpret_cast<const uint2*>(kp + k_index_fp8(t, c0));
            unsigned kw[4] = {0, 0, 0, 0}, vw[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned kbyte = ((e < 4 ? kb.x : kb.y) >> (8 * (e & 3))) & 0xffu;
                kw[e >> 1] |= e4m3_to_bf16(kbyte) << ((e & 1) * 16);
                vw[e >> 1] |= e4m3_to_bf16(vp[v_index_fp8(t, c0 + e)]) << ((e & 1) * 16);
            }
            *reinterpret_cast<uint4*>(kr) = make_uint4(kw[0], kw[1], kw[2], kw[3]);
            *reinterpret_cast<uint4*>(vr) = make_uint4(vw[0], vw[1], vw[2], vw[3]);
        }
    } else if (st.dtype == 1) {
        unsigned short* pool = static_cast<unsigned short*>(st.pool);
        unsigned short* kp = pool + page;
        unsigned short* vp = kp + kPageTokens * D;
        unsigned short* kr = static_cast<unsigned short*>(a.k) + row;
        unsigned short* vr = static_cast<unsigned short*>(a.v) + row;
        const int c0 = ch * 8;
        if (kToStore) {
            *reinterpret_cast<uint4*>(kp + k_index_bf16(t, c0)) = *reinterpret_cast<const uint4*>(kr);
            const uint4 vv = *reinterpret_cast<const uint4*>(vr);
            const unsigned w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                vp[v_index_bf16(t, c0 + e)] = (unsigned short)(w[e >> 1] >> ((e & 1) * 16));
        } else {
            *reinterpret_cast<uint4*>(kr) = *reinterpret_cast<const uint4*>(kp + k_index_bf16(t, c0));
            unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                w[e >> 1] |= (unsigned)vp[v_index_bf16(t, c0 + e)] << ((e & 1) * 16);
            *reinterpret_cast<uint4*>(vr) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    } else {
        float* pool = static_cast<float*>(st.pool);
        float* kp = pool + page + (size_t)t * D + ch * 4;
        float* vp = kp + kPageTokens * D;
        float* kr = static_cast<float*>(a.k) + row;
        float* vr = static_cast<float*>(a.v) + row;
        if (kToStore) {
            *reinterpret_cast<float4*>(kp) = *reinterpret_cast<const float4*>(kr);
            *reinterpret_cast<float4*>(vp) = *reinterpret_cast<const float4*>(vr);
        } else {
            *reinterpret_cast<float4*>(kr) = *reinterpret_cast<const float4*>(kp);
            *reinterpret_cast<float4*>(vr) = *reinterpret_cast<const float4*>(vp);
        }
    }
}

// Append of several rows per sequence to a bf16 or fp8 store (prefill chunks, store fills): one
// workgroup per (sequence, kv head, page touched).  K rows go straight to their operand-order
// position, one 16-byte (fp8: 8-byte) piece per thread.  V rows are staged in LDS and leave as whole
// 16-byte operand chunks (bf16: four tokens x two channels; fp8: four tokens x four channels)
// wherever all four tokens of the chunk are being written; the ragged first and last tokens of the
// append fall back to single elements.  A whole-page append therefore writes each page in full-width
// stores instead of 2-byte (1-byte) scatters.  fp8: the rows are rounded to E4M3 by the integer
// routine every other writer of that store uses.
template <bool kFp8>
__global__ __launch_bounds__(256) void append_pages_kernel(CopyArgs a)
{
    using Elem = std::conditional_t<kFp8, unsigned char, unsigned short>;
    const StoreView& st = a.st;
    const int D = st.head_dim;                    // 64 or 128
    const int g = blockIdx.y, b = blockIdx.z;
    const long start = (long)a.start_pos[a.pos_per_head ? b * st.Hkv + g : b] + a.pos_bias;
    const long cap = (long)st.max_blocks_per_seq * kPageTokens;
    if (start < 0 || start >= cap) return;
    const long end = start + a.T < cap ? start + a.T : cap;
    const long page = start / kPageTokens + blockIdx.x;
    const long tok0 = page * kPageTokens;
    if (tok0 >= end) return;
    const int t_lo = (int)(start > tok0 ? start - tok0 : 0);
    const int t_hi = (int)(end - tok0 < kPageTokens ? end - tok0 : kPageTokens);
    const int blk = block_of(st, b, (int)page);
    if (blk < 0 || blk >= st.num_blocks) return;
    Elem* kp = static_cast<Elem*>(st.pool) + page_offset(st, resolve_slot(st), blk, g);
    Elem* vp = kp + kPageTokens * D;
    __shared__ Elem vs[kPageTokens][128 + 8];

    const int chunks = D / 8;                     // 8-channel pieces per row
    const int t = threadIdx.x / 16, ch = threadIdx.x % 16;
    if (t >= t_lo && t < t_hi && ch < chunks) {
        const size_t row = (((size_t)b * a.T + (size_t)(tok0 + t - start)) * st.Hkv + g) * D + (size_t)ch * 8;
        const uint4 kk = *reinterpret_cast<const uint4*>(static_cast<const unsigned short*>(a.k) + row);
        const uint4 vv = *reinterpret_cast<const uint4*>(static_cast<const unsigned short*>(a.v) + row);
        if constexpr (kFp8) {
            const unsigned kw[4] = {kk.x, kk.y, kk.z, kk.w}, vw[4] = {vv.x, vv.y, vv.z, vv.w};
            unsigned k8[2] = {0, 0}, v8[2] = {0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                k8[e >> 2] |= bf16_to_e4m3((kw[e >> 1] >> ((e & 1) * 16)) & 0xffffu) << (8 * (e & 3));
                v8[e >> 2] |= bf16_to_e4m3((vw[e >> 1] >> ((e & 1) * 16)) & 0xffffu) << (8 * (e & 3));
            }
            *reinterpret_cast<uint2*>(kp + k_index_fp8(t, ch * 8)) = make_uint2(k8[0], k8[1]);
            *reinterpret_cast<uint2*>(&vs[t][ch * 8]) = make_uint2(v8[0], v8[1]);
        } else {
            *reinterpret_cast<uint4*>(kp + k_index_bf16(t, ch * 8)) = kk;
            *reinterpret_cast<uint4*>(&vs[t][ch * 8]) = vv;
        }
    }
    __syncthreads();
    if constexpr (kFp8) {
        // output chunk o: channels (o/64)*64 + {0,16,32,48} + o%16, tokens 4*((o/16)%4) .. +3
        for (int o = threadIdx.x; o < D; o += 256) {
            const int cp = o / 64, quad = (o / 16) % 4, dl = o % 16;
            unsigned char e[16];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) e[j * 4 + i] = vs[quad * 4 + i][cp * 64 + j * 16 + dl];
            unsigned char* dst = vp + (size_t)o * 16;
            if (quad * 4 >= t_lo && quad * 4 + 4 <= t_hi) {
                unsigned w[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    w[j] = e[j * 4] | (unsigned)e[j * 4 + 1] << 8 | (unsigned)e[j * 4 + 2] << 16 | (unsigned)e[j * 4 + 3] << 24;
                *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (quad * 4 + i >= t_lo && quad * 4 + i < t_hi) dst[j * 4 + i] = e[j * 4 + i];
            }
        }
    } else {
        // output chunk o: channels (o/64)*32 + {0,16} + o%16, tokens 4*((o/16)%4) .. +3
        for (int o = threadIdx.x; o < D * 2; o += 256) {
            const int cp = o / 64, quad = (o / 16) % 4, dl = o % 16;
            unsigned short e[8];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) e[j * 4 + i] = vs[quad * 4 + i][cp * 32 + j * 16 + dl];
            unsigned short* dst = vp + (size_t)o * 8;
            if (quad * 4 >= t_lo && quad * 4 + 4 <= t_hi) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(e[0] | (unsigned)e[1] << 16, e[2] | (unsigned)e[3] << 16,
                                                            e[4] | (unsigned)e[5] << 16, e[6] | (unsigned)e[7] << 16);
            } else {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (quad * 4 + i >= t_lo && quad * 4 + i < t_hi) dst[j * 4 + i] = e[j * 4 + i];
            }
        }
    }
}

// In-place compaction of a slot after token eviction: for every (sequence, kv head) the tokens
// at the increasing positions keep_idx[0 .. count) move to positions 0 .. count.  A workgroup
// owns one (kv head, sequence) and one of the 16-byte channel pieces of its rows (pieces never
// interact, so they spread over workgroups) and walks the destination in chunks of 1024 tokens:
// thread t loads the piece of K and of V of the source tokens keep_idx[chunk + t + 256 u],
// u = 0 .. 3, the workgroup meets at a barrier, then the pieces are stored at chunk + t + 256 u.  Because
// keep_idx[j] >= j, a chunk reads only positions at or behind its own start and writes only its
// own positions, so chunks never touch each other's data and one barrier per chunk is enough.
// kKind: the store's type code (0 fp32: a piece is 4 channels; 1 bf16, 2 fp8: 8 channels, whose keys
// are one contiguous run in the page and whose values are eight separate elements).
constexpr int kCompactTokens = 256;    // tokens one pass of the workgroup's threads covers
constexpr int kCompactPasses = 4;      // passes per chunk: a thread moves this many tokens between two barriers
template <int kKind>
__global__ __launch_bounds__(256) void compact_kernel(CompactArgs a)
{
    const StoreView& st = a.st;
    const int D = st.head_dim;
    constexpr bool kBf16 = kKind == 1, kFp8 = kKind == 2;
    constexpr int per = kKind == 0 ? 4 : 8;
    const int g = blockIdx.x, b = blockIdx.y;
    const int ch = blockIdx.z;                                 // the workgroup's piece of the rows
    const int tt = threadIdx.x;
    const int cap = st.max_blocks_per_seq * kPageTokens;
    int count = a.keep_count[b * st.Hkv + g];
    const int most = a.max_keep < cap ? a.max_keep : cap;
    count = count < 0 ? 0 : (count > most ? most : count);
    const int32_t* idx = a.keep_idx + ((size_t)b * st.Hkv + g) * a.max_keep;
    const int slot = resolve_slot(st);
    // A chunk is kCompactPasses * kCompactTokens destination positions: the walk is a chain of
    // dependent round trips (index, page-table entry, data, barrier, store), so the more tokens a
    // thread has in flight per barrier the fewer such chains a (sequence, kv head) takes.
    for (int c0 = 0; c0 < count; c0 += kCompactPasses * kCompactTokens) {
        uint4 kreg[kCompactPasses], vreg[kCompactPasses];
        int dblk[kCompactPasses];
        bool ok[kCompactPasses];
#pragma unroll
        for (int u = 0; u < kCompactPasses; ++u) {
            const int j = c0 + u * kCompactTokens + tt;
            const bool active = j < count && ch * per < D;
            int src = active ? idx[j] : 0;
            src = src < 0 ? 0 : (src >= cap ? cap - 1 : src);
            const int sblk = block_of(st, b, src / kPageTokens);
            dblk[u] = block_of(st, b, (j < cap ? j : cap - 1) / kPageTokens);
            ok[u] = active && sblk >= 0 && sblk < st.num_blocks && dblk[u] >= 0 && dblk[u] < st.num_blocks;
            const int ts = src % kPageTokens;
            kreg[u] = make_uint4(0, 0, 0, 0);
            vreg[u] = make_uint4(0, 0, 0, 0);
            if (ok[u]) {
                if (kBf16) {
                    const unsigned short* kp = static_cast<const unsigned short*>(st.pool) + page_offset(st, slot, sblk, g);
                    const unsigned short* vp = kp + kPageTokens * D;
                    kreg[u] = *reinterpret_cast<const uint4*>(kp + k_index_bf16(ts, ch * 8));
                    unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int e = 0; e < 8; ++e) w[e >> 1] |= (unsigned)vp[v_index_bf16(ts, ch * 8 + e)] << ((e & 1) * 16);
                    vreg[u] = make_uint4(w[0], w[1], w[2], w[3]);
                } else if (kFp8) {
                    const unsigned char* kp = static_cast<const unsigned char*>(st.pool) + page_offset(st, slot, sblk, g);
                    const unsigned char* vp = kp + kPageTokens * D;
                    const uint2 k8 = *reinterpret_cast<const uint2*>(kp + k_index_fp8(ts, ch * 8));
                    kreg[u] = make_uint4(k8.x, k8.y, 0, 0);
                    unsigned w[2] = {0, 0};
#pragma unroll
                    for (int e = 0; e < 8; ++e) w[e >> 2] |= (unsigned)vp[v_index_fp8(ts, ch * 8 + e)] << ((e & 3) * 8);
                    vreg[u] = make_uint4(w[0], w[1], 0, 0);
                } else {
                    const float* kp = static_cast<const float*>(st.pool) + page_offset(st, slot, sblk, g) + (size_t)ts * D + ch * 4;
                    kreg[u] = *reinterpret_cast<const uint4*>(kp);
                    vreg[u] = *reinterpret_cast<const uint4*>(kp + kPageTokens * D);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kCompactPasses; ++u) {
            if (!ok[u]) continue;
            const int td = (c0 + u * kCompactTokens + tt) % kPageTokens;
            if (kBf16) {
                unsigned short* kp = static_cast<unsigned short*>(st.pool) + page_offset(st, slot, dblk[u], g);
                unsigned short* vp = kp + kPageTokens * D;
                *reinterpret_cast<uint4*>(kp + k_index_bf16(td, ch * 8)) = kreg[u];
                const unsigned w[4] = {vreg[u].x, vreg[u].y, vreg[u].z, vreg[u].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) vp[v_index_bf16(td, ch * 8 + e)] = (unsigned short)(w[e >> 1] >> ((e & 1) * 16));
            } else if (kFp8) {
                unsigned char* kp = static_cast<unsigned char*>(st.pool) + page_offset(st, slot, dblk[u], g);
                unsigned char* vp = kp + kPageTokens * D;
                *reinterpret_cast<uint2*>(kp + k_index_fp8(td, ch * 8)) = make_uint2(kreg[u].x, kreg[u].y);
                const unsigned w[2] = {vreg[u].x, vreg[u].y};
#pragma unroll
                for (int e = 0; e < 8; ++e) vp[v_index_fp8(td, ch * 8 + e)] = (unsigned char)(w[e >> 2] >> ((e & 3) * 8));
            } else {
                float* kp = static_cast<float*>(st.pool) + page_offset(st, slot, dblk[u], g) + (size_t)td * D + ch * 4;
                *reinterpret_cast<uint4*>(kp) = kreg[u];
                *reinterpret_cast<uint4*>(kp + kPageTokens * D) = vreg[u];
            }
        }
    }
}

// Debug aid: the kernels resolve slots and pages from the device copies of the maps and clamp
// whatever they find into the pool, so a device map that differs from the host copies the checks
// and the no-op decisions use, or a page-table entry outside the pool, stays silent.  One workgroup
// counts both kinds of entries and writes the two counts.
__global__ __launch_bounds__(1024) void check_store_kernel(CheckArgs a)
{
    const StoreView& st = a.st;
    int bad_map = 0, bad_block = 0;
    for (int l = threadIdx.x; l < st.L; l += blockDim.x)
        bad_map += (st.share_map[l] != a.host_share_map[l]) + (st.slot_of_layer[l] != a.host_slot_of_layer[l]);
    if (st.block_table) {
        const size_t n = (size_t)a.B * st.max_blocks_per_seq;
        for (size_t i = threadIdx.x; i < n; i += blockDim.x) {
            const int blk = st.block_table[i];
            bad_block += blk < 0 || blk >= st.num_blocks;
        }
    }
    __shared__ int s_map, s_block;
    if (threadIdx.x == 0) s_map = s_block = 0;
    __syncthreads();
    if (bad_map) atomicAdd(&s_map, bad_map);
    if (bad_block) atomicAdd(&s_block, bad_block);
    __syncthreads();
    if (threadIdx.x == 0) {
        a.report[0] = s_map;
        a.report[1] = s_block;
    }
}

}  // namespace

int launch_check_store(const CheckArgs& a, void* stream)
{
    hipLaunchKernelGGL(check_store_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

int launch_append(const CopyArgs& a, void* stream)
{
    if (a.st.dtype != 0 && a.T >= 4) {
        // pages a sequence's rows can touch: T rows starting anywhere inside a page
        const dim3 grid((unsigned)((a.T + kPageTokens - 1) / kPageTokens + 1), a.st.Hkv, a.B);
        if (a.st.dtype == 1) hipLaunchKernelGGL(append_pages_kernel<false>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
        else hipLaunchKernelGGL(append_pages_kernel<true>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
        return (int)hipGetLastError();
    }
    const int per = a.st.dtype == 0 ? 4 : 8;
    const long total = (long)a.B * a.T * a.st.Hkv * (a.st.head_dim / per);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(copy_rows_kernel<true>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

int launch_compact(const CompactArgs& a, void* stream)
{
    const int pieces = a.st.head_dim / (a.st.dtype == 0 ? 4 : 8);
    const dim3 grid(a.st.Hkv, a.B, pieces);
    if (a.st.dtype == 1)
        hipLaunchKernelGGL(compact_kernel<1>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    else if (a.st.dtype == 2)
        hipLaunchKernelGGL(compact_kernel<2>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    else
        hipLaunchKernelGGL(compact_kernel<0>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

int launch_gather(const CopyArgs& a, void* stream)
{
    const int per = a.st.dtype == 0 ? 4 : 8;
    const long total = (long)a.B * a.T * a.st.Hkv * (a.st.head_dim / per);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(copy_rows_kernel<false>, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

}  // namespace kvs
