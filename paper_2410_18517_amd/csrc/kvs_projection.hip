// Key/value projection fused with the append (gfx950).  This is the work a sharing strategy
// removes for every layer that reads a donor's cache (paper Sec. 3.2; the abstract's "KV cache
// computation"): such layers never reach this kernel.  For the others
//     k = x . Wk^T,  v = x . Wv^T,  k <- rope(k),  store <- round_bf16(k), round_bf16(v)
// in one pass: the projected rows never exist in HBM in row-major form.
//
// Work split: a workgroup owns 16 rows of x (a row is one token of one sequence) and, of
// either K or V, one head's channels [c0, c0+16) and [c0+half, c0+half+16) -- the two ends of
// the rotary pairs (c, c + head_dim/2), so the rotation needs no other workgroup.  Its four
// wavefronts split the contraction over `hidden`; each streams its slice of x (A operand) and of
// the two 16-row weight strips (B operands) in 16-byte pieces straight into
// v_mfma_f32_16x16x32_bf16, and the four partial tiles meet in LDS.  A decode step (a handful
// of rows) is a weight-streaming problem bounded by HBM; to put enough workgroups on it the
// contraction is also split across workgroups (grid.z): each publishes its partial tile with
// device-scope stores and the last to arrive at a tile adds them in a fixed order and finishes
// (same no-wait protocol as the attention splits).  A prefill chunk re-reads the strips from
// L2 once per 16 rows.
#include <hip/hip_runtime.h>

#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kPageTokens = 16;
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kUnroll = 4;             // contraction steps (of 32) whose loads are issued together

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;

__device__ __forceinline__ unsigned short round_bf16(float x)
{
    floatx2 f = {x, 0.f};
    return (unsigned short)(__builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2)) & 0xffffu);
}

// In-page element index of (token t, channel c): the store's operand order (see kvs.h).
__device__ __forceinline__ int k_index(int t, int c) { return (((c >> 5) * 4 + ((c & 31) >> 3)) * 16 + t) * 8 + (c & 7); }
__device__ __forceinline__ int v_index(int t, int c)
{
    return ((((c >> 5) * 4 + (t >> 2)) * 16 + (c & 15)) * 2 + ((c >> 4) & 1)) * 4 + (t & 3);
}

__global__ __launch_bounds__(kThreads) void project_append_bf16_kernel(ProjectArgs a)
{
    const StoreView& st = a.st;
    const int D = st.head_dim, half = D / 2;
    const int tiles_per_head = half / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int quad = lane >> 4, l16 = lane & 15;
    const int tile = blockIdx.x % tiles_per_head;
    const int head = (blockIdx.x / tiles_per_head) % st.Hkv;
    const int is_v = blockIdx.x / (tiles_per_head * st.Hkv);
    const int c0 = tile * 16;
    const int M = a.B * a.T;
    const int m0 = blockIdx.y * 16;

    const unsigned short* x = static_cast<const unsigned short*>(a.x);
    const unsigned short* w = static_cast<const unsigned short*>(is_v ? a.w_v : a.w_k);
    const int slice = a.hidden / (kWaves * a.k_splits);  // contraction range of this wavefront
    const int k_lo = (blockIdx.z * kWaves + wave) * slice;
    const bool row_ok = m0 + l16 < M;
    const unsigned short* xa = x + (size_t)(row_ok ? m0 + l16 : 0) * a.hidden + k_lo + quad * 8;
    const unsigned short* wb0 = w + ((size_t)head * D + c0 + l16) * a.hidden + k_lo + quad * 8;
    const unsigned short* wb1 = wb0 + (size_t)half * a.hidden;

    // Where this thread's (row, channel pair) of the finished tile goes, and its rotation: the
    // dependent look-ups are issued now so that they travel under the weight stream.
    const int r = threadIdx.x / 16, c = threadIdx.x % 16;
    const int m = m0 + r;
    bool writes = m < M;
    int b = 0, blk = 0, slot = 0;
    long pos = 0;
    float cs = 1.f, sn = 0.f;
    if (writes) {
        b = m / a.T;
        pos = (long)a.start_pos[b] + m % a.T;
        writes = pos >= 0 && pos < (long)st.max_blocks_per_seq * kPageTokens;
    }
    if (writes) {
        if (!is_v && a.rope_cos) {
            cs = a.rope_cos[(size_t)pos * half + c0 + c];
            sn = a.rope_sin[(size_t)pos * half + c0 + c];
        }
        int donor = st.share_map[st.layer];
        donor = donor < 0 ? 0 : (donor >= st.L ? st.L - 1 : donor);
        slot = st.slot_of_layer[donor];
        slot = slot < 0 ? 0 : (slot >= st.n_slots ? st.n_slots - 1 : slot);
        const size_t bidx = (size_t)b * st.max_blocks_per_seq + (size_t)(pos / kPageTokens);
        blk = st.block_table ? st.block_table[bidx] : (int)bidx;
        writes = blk >= 0 && blk < st.num_blocks;
    }

    floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < slice; k += 32 * kUnroll) {
        uint4 fa[kUnroll], f0[kUnroll], f1[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int kk = k + 32 * u;
            const bool in = kk < slice;
            fa[u] = in && row_ok ? *reinterpret_cast<const uint4*>(xa + kk) : make_uint4(0, 0, 0, 0);
            f0[u] = in ? *reinterpret_cast<const uint4*>(wb0 + kk) : make_uint4(0, 0, 0, 0);
            f1[u] = in ? *reinterpret_cast<const uint4*>(wb1 + kk) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[u]),
                                                           __builtin_bit_cast(bf16x8, f0[u]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[u]),
                                                           __builtin_bit_cast(bf16x8, f1[u]), acc1, 0, 0, 0);
        }
    }
    // lane holds column l16 of rows 4*quad .. 4*quad+3 of both strips
    __shared__ float part[kWaves][2][16][17];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        part[wave][0][quad * 4 + i][l16] = acc0[i];
        part[wave][1][quad * 4 + i][l16] = acc1[i];
    }
    __syncthreads();

    // one thread per (row, channel pair): sum the four slices, rotate, round, store
    float lo = 0.f, hi = 0.f;
#pragma unroll
    for (int wv = 0; wv < kWaves; ++wv) {
        lo += part[wv][0][r][c];
        hi += part[wv][1][r][c];
    }
    if (a.k_splits > 1) {
        // partial tiles: [k split][column workgroup][row workgroup][256 threads] pairs of floats
        const size_t tile_id = (size_t)blockIdx.x * gridDim.y + blockIdx.y;
        const size_t n_tiles = (size_t)gridDim.x * gridDim.y;
        float* mine = a.partials + ((blockIdx.z * n_tiles + tile_id) * kThreads + threadIdx.x) * 2;
        const floatx2 pv = {lo, hi};
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(mine), __builtin_bit_cast(unsigned long long, pv),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __shared__ int s_is_last;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the device-scope stores are acknowledged
        __syncthreads();
        if (threadIdx.x == 0) {
            const int arrived = atomicAdd(a.counters + tile_id, 1);
            s_is_last = arrived == a.k_splits - 1;
            if (s_is_last) atomicExch(a.counters + tile_id, 0);
        }
        __syncthreads();
        if (!s_is_last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        lo = hi = 0.f;
        for (int ks0 = 0; ks0 < a.k_splits; ks0 += 4) {  // four loads in flight, added in split order
            unsigned long long wd[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                wd[u] = ks0 + u < a.k_splits
                            ? __hip_atomic_load(reinterpret_cast<const unsigned long long*>(
                                                    a.partials + (((ks0 + u) * n_tiles + tile_id) * kThreads + threadIdx.x) * 2),
                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                            : 0ull;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const floatx2 v2 = __builtin_bit_cast(floatx2, wd[u]);
                lo += v2[0];
                hi += v2[1];
            }
        }
    }
    if (!writes) return;
    if (!is_v && a.rope_cos) {
        const float rl = lo * cs - hi * sn, rh = hi * cs + lo * sn;
        lo = rl;
        hi = rh;
    }
    unsigned short* page = static_cast<unsigned short*>(st.pool) +
                           ((((size_t)slot * st.num_blocks + blk) * st.Hkv + head) * 2 + is_v) * (size_t)(kPageTokens * D);
    const int t = (int)(pos % kPageTokens);
    if (is_v) {
        page[v_index(t, c0 + c)] = round_bf16(lo);
        page[v_index(t, c0 + c + half)] = round_bf16(hi);
    } else {
        page[k_index(t, c0 + c)] = round_bf16(lo);
        page[k_index(t, c0 + c + half)] = round_bf16(hi);
    }
}

}  // namespace

// Workgroups per launch aimed at.  The contraction is split across workgroups only as far as
// each wavefront keeps at least 128 elements of it.
constexpr long kTargetWorkgroups = 256;                  // one per compute unit measured fastest
int project_k_splits(int Hkv, int head_dim, int hidden, int rows)
{
    const long tiles = 2L * Hkv * (head_dim / 32) * ((rows + 15) / 16);
    long want = (kTargetWorkgroups + tiles - 1) / tiles;
    const long most = hidden / (kWaves * 128);
    want = want > most ? most : want;
    want = want < 1 ? 1 : want;
    while (hidden % (kWaves * 32 * want) != 0) --want;    // every wavefront gets whole steps of 32
    return (int)want;
}

size_t project_workspace_bytes(int Hkv, int head_dim, int hidden, int rows)
{
    const size_t tiles = (size_t)2 * Hkv * (head_dim / 32) * ((rows + 15) / 16);
    const size_t counters = (tiles * sizeof(int32_t) + 255) / 256 * 256;
    const int ks = project_k_splits(Hkv, head_dim, hidden, rows);
    return counters + (ks > 1 ? (size_t)ks * tiles * kThreads * 2 * sizeof(float) : 0);
}

int launch_project_append(ProjectArgs a, void* workspace, void* stream)
{
    const int tiles_per_head = a.st.head_dim / 32;
    const unsigned col_wgs = 2u * a.st.Hkv * tiles_per_head;
    const unsigned row_wgs = (unsigned)((a.B * a.T + 15) / 16);
    a.k_splits = project_k_splits(a.st.Hkv, a.st.head_dim, a.hidden, a.B * a.T);
    const size_t tiles = (size_t)col_wgs * row_wgs;
    a.counters = static_cast<int32_t*>(workspace);
    a.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + (tiles * sizeof(int32_t) + 255) / 256 * 256);
    hipLaunchKernelGGL(project_append_bf16_kernel, dim3(col_wgs, row_wgs, a.k_splits), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

}  // namespace kvs
