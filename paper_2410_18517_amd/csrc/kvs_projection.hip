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
// (same no-wait protocol as the attention splits).
//
// A prefill chunk (more than 32 rows) is a matrix product bounded by the matrix cores and takes
// a tiled kernel instead: a workgroup of eight wavefronts owns 256 rows and one whole head of
// K or V (or, with enough rows, two adjacent heads); the 256 x 64 pieces of x and of the weight
// rows go from global memory straight into LDS (global_load_lds_dwordx4), with the 16-byte pieces
// of a row XOR-swizzled by the row index so that the operand reads of a wavefront fall on
// distinct banks without padding; each wavefront keeps a block of accumulators whose columns
// again hold both ends of the rotary pairs.
#include <hip/hip_runtime.h>

#include "kvs_device.h"
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kUnroll = 4;             // contraction steps (of 32) whose loads are issued together

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned short round_bf16(float x)
{
    floatx2 f = {x, 0.f};
    return (unsigned short)(__builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2)) & 0xffffu);
}

// One projected element into its page (`page_off`: element offset of the page in the pool), in
// the store's operand order.  bf16 store: rounded to bf16.  fp8 store: that bf16 value rounded on
// to E4M3, exactly what an append of the bf16 row would store.
__device__ __forceinline__ void store_projected(void* pool, size_t page_off, bool fp8, int is_v, int t, int c, float x)
{
    const unsigned short h = round_bf16(x);
    if (fp8)
        static_cast<unsigned char*>(pool)[page_off + (is_v ? v_index_fp8(t, c) : k_index_fp8(t, c))] = (unsigned char)bf16_to_e4m3(h);
    else
        static_cast<unsigned short*>(pool)[page_off + (is_v ? v_index_bf16(t, c) : k_index_bf16(t, c))] = h;
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
    const size_t page_off = ((((size_t)slot * st.num_blocks + blk) * st.Hkv + head) * 2 + is_v) * (size_t)(kPageTokens * D);
    const int t = (int)(pos % kPageTokens);
    const bool fp8 = st.dtype == 2;                              // the store's type code: 1 bf16, 2 fp8
    store_projected(st.pool, page_off, fp8, is_v, t, c0 + c, lo);
    store_projected(st.pool, page_off, fp8, is_v, t, c0 + c + half, hi);
}

// ---- tiled kernel for many rows ------------------------------------------------------------

constexpr int kTileRows = 256;         // rows of x per workgroup
constexpr int kTiledThreads = 2 * kTileRows;   // a wavefront per 64 rows x half of the head's rotary pairs
constexpr int kStageRows = kTiledThreads / 8;  // rows staged by one pass of the workgroup (8 threads per row)
constexpr int kTileK = 64;             // contraction depth staged per step
constexpr int kLdsRow = kTileK;        // elements per staged row; 16-byte piece q of row r sits at piece q ^ (r & 7)

template <int D>
__global__ __launch_bounds__(kTiledThreads) void project_append_tiled_kernel(ProjectArgs a)
{
    constexpr int NT = D / 32;         // 16-column accumulator tiles per wavefront: NT/2 low, NT/2 high channels
    constexpr int half = D / 2;
    constexpr int kBChunks = D * (kTileK / 8) / kTiledThreads;          // 16-byte pieces of the weight tile per thread
    constexpr int kAChunks = kTileRows * (kTileK / 8) / kTiledThreads;  // and of the x tile
    const StoreView& st = a.st;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int quad = lane >> 4, l16 = lane & 15;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroups go to the eight XCDs round-robin by their linear index, and each XCD has its own
    // L2.  The grid is (8, tiles per XCD, splits), so blockIdx.x is the XCD; the output tiles,
    // listed row tile by row tile, are dealt out in eight consecutive runs: the head blocks of a
    // row tile meet in one L2 and fetch its x rows from memory once.
    const int n_blocks = 2 * st.Hkv;
    const int M = a.B * a.T;
    const int n_row_tiles = (M + kTileRows - 1) / kTileRows;
    const int tile = blockIdx.x * gridDim.y + blockIdx.y;
    if (tile >= n_blocks * n_row_tiles) return;                    // padding of the last run
    const int head_block = tile % n_blocks;
    const int row_tile = tile / n_blocks;
    const int head = head_block % st.Hkv;
    const int is_v = head_block / st.Hkv;
    const int m0 = row_tile * kTileRows;

    __shared__ __attribute__((aligned(16))) unsigned short sa[3][kTileRows][kLdsRow];
    __shared__ __attribute__((aligned(16))) unsigned short sb[3][D][kLdsRow];

    const unsigned short* x = static_cast<const unsigned short*>(a.x);
    const unsigned short* w = static_cast<const unsigned short*>(is_v ? a.w_v : a.w_k) + (size_t)head * D * a.hidden;
    const int k_len = a.hidden / a.k_splits;
    const int k_begin = blockIdx.z * k_len;
    const int n_steps = k_len / kTileK;

    // Where each of the tile's rows will be stored: looked up once, by one thread per row, while
    // the first tiles load (the epilogue then has no chain of dependent global loads per row).
    __shared__ long long row_page[kTileRows];                      // element offset of the row's page, -1: dropped
    __shared__ int row_pos[kTileRows];
    if (threadIdx.x < kTileRows) {
        const int m = m0 + threadIdx.x;
        long long off = -1;
        long pos = 0;
        if (m < M) {
            const int b = m / a.T;
            pos = (long)a.start_pos[b] + m % a.T;
            if (pos >= 0 && pos < (long)st.max_blocks_per_seq * kPageTokens) {
                int donor = st.share_map[st.layer];
                donor = donor < 0 ? 0 : (donor >= st.L ? st.L - 1 : donor);
                int slot = st.slot_of_layer[donor];
                slot = slot < 0 ? 0 : (slot >= st.n_slots ? st.n_slots - 1 : slot);
                const size_t bidx = (size_t)b * st.max_blocks_per_seq + (size_t)(pos / kPageTokens);
                const int blk = st.block_table ? st.block_table[bidx] : (int)bidx;
                if (blk >= 0 && blk < st.num_blocks)
                    off = (long long)(((((size_t)slot * st.num_blocks + blk) * st.Hkv + head) * 2 + is_v) *
                                      (size_t)(kPageTokens * D));
            }
        }
        row_page[threadIdx.x] = off;
        row_pos[threadIdx.x] = off < 0 ? 0 : (int)pos;
    }

    // Staging goes from global memory straight into LDS (global_load_lds_dwordx4: lane L of a
    // wavefront fetches 16 bytes from its own address and the hardware writes them at the
    // wavefront's LDS base + 16 L), so the tiles in flight occupy no registers and no LDS store
    // instructions are issued.  LDS piece p = 512 j + thread of a tile is piece p % 8 of row p / 8;
    // the swizzle (piece q of row r sits at q ^ (r & 7)) is applied on the global side: the lane
    // fetches the piece that belongs where it writes.  Rows past the last one re-read the last row;
    // their accumulators are never stored.
    const int s_row = threadIdx.x >> 3;                            // + 64 j
    const int s_col = ((threadIdx.x & 7) ^ (s_row & 7)) * 8;       // 64 j keeps row & 7
    const int wave_row = __builtin_amdgcn_readfirstlane(wave * 8); // first LDS row the wavefront writes in a pass
    const unsigned short* src_a[kAChunks];
    const unsigned short* src_b[kBChunks];
#pragma unroll
    for (int j = 0; j < kAChunks; ++j) {
        const int m = m0 + s_row + kStageRows * j;
        src_a[j] = x + (size_t)(m < M ? m : M - 1) * a.hidden + k_begin + s_col;
    }
#pragma unroll
    for (int j = 0; j < kBChunks; ++j) src_b[j] = w + (size_t)(s_row + kStageRows * j) * a.hidden + k_begin + s_col;

    floatx4 acc[4][NT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // The load is written as assembly: seen as an LDS write by the compiler, every LDS read after it
    // would be made to wait for it (the two cannot be told apart by address), which would undo the
    // prefetch; the waits that matter are spelled out at the barrier instead.
#define KVS_LOAD_TO_LDS(gptr, lds_ptr)                                                               \
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"                    \
                 :: "v"(gptr), "s"((unsigned)(size_t)(lds_ptr)) : "memory")
#define KVS_FETCH(step, buf)                                                                         \
    _Pragma("unroll") for (int j = 0; j < kAChunks; ++j)                                             \
        KVS_LOAD_TO_LDS(src_a[j] + (step) * kTileK, &sa[buf][wave_row + kStageRows * j][0]);         \
    _Pragma("unroll") for (int j = 0; j < kBChunks; ++j)                                             \
        KVS_LOAD_TO_LDS(src_b[j] + (step) * kTileK, &sb[buf][wave_row + kStageRows * j][0]);
#define KVS_READ(buf, kk, fa, fb)                                                                    \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
        fa[i] = *reinterpret_cast<const bf16x8*>(&sa[buf][wm * 64 + i * 16 + l16][((kk) + quad * 8) ^ ((l16 & 7) * 8)]); \
    _Pragma("unroll") for (int j = 0; j < NT; ++j) {                                                 \
        const int col = (j < NT / 2 ? 0 : half) + wn * (D / 4) + (j % (NT / 2)) * 16 + l16;          \
        fb[j] = *reinterpret_cast<const bf16x8*>(&sb[buf][col][((kk) + quad * 8) ^ ((l16 & 7) * 8)]); \
    }
#define KVS_MULTIPLY(fa, fb)                                                                         \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
        _Pragma("unroll") for (int j = 0; j < NT; ++j)                                               \
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    // Matrix instructions in fours, each four followed by two LDS reads: the order the scheduler
    // is held to, so that operand reads travel under arithmetic instead of being waited for
    // right where they are issued.
#define KVS_FOURS_WITH_READS                                                                         \
    if constexpr (NT == 4) {                                                                         \
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                              \
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); /* matrix instructions */             \
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0); /* LDS reads */                       \
        }                                                                                            \
    }

    // A step is two half-steps of 32 along the contraction, and the workgroup's barrier sits
    // between them, not at the step's end.  Three LDS buffers rotate.  Step s
    //   - starts the loads of the tiles of step s+2 into buffer (s+2)%3, whose last readers waited
    //     for their data before the barrier of step s-1,
    //   - multiplies its first half (operands already in registers) while it reads its second
    //     half's operands from buffer s%3,
    //   - waits until its own loads of step s+1 (issued a step ago) have landed; barrier;
    //   - multiplies its second half while it reads the first half's operands of step s+1.
    // Every LDS read has sixteen matrix instructions to hide behind and every global load two
    // steps.  The last two steps re-load the last tiles into a free buffer, which nobody reads, so
    // that every step is the same straight-line code.  The barrier is the bare instruction with the
    // waits spelled out: a fence would also wait for the loads that were only just issued.
    constexpr int kLoads = kAChunks + kBChunks;                    // global loads a thread issues per step
    // vmcnt(kLoads): all but this step's loads have landed; lgkmcnt(0): this wavefront's LDS reads are done
#define KVS_WAIT_OLDER asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(kLoads) : "memory")
#define KVS_STEP(step, b0, b1, b2)                                                                   \
    {                                                                                                \
        const int ahead = (step) + 2 < n_steps ? (step) + 2 : n_steps - 1;                           \
        KVS_FETCH(ahead, b2)                                                                         \
        KVS_READ(b0, 32, fa1, fb1)                                                                   \
        KVS_MULTIPLY(fa0, fb0)                                                                       \
        if constexpr (NT == 4) __builtin_amdgcn_sched_group_barrier(0x020, kLoads, 0);               \
        KVS_FOURS_WITH_READS                                                                         \
        KVS_WAIT_OLDER;                                                                              \
        __builtin_amdgcn_s_barrier();                                                                \
        KVS_READ(b1, 0, fa0, fb0)                                                                    \
        KVS_MULTIPLY(fa1, fb1)                                                                       \
        KVS_FOURS_WITH_READS                                                                         \
    }
    bf16x8 fa0[4], fb0[NT], fa1[4], fb1[NT];
    KVS_FETCH(0, 0)
    KVS_FETCH(1, 1)
    KVS_WAIT_OLDER;                                                // the tiles of step 0 have landed
    __builtin_amdgcn_s_barrier();
    KVS_READ(0, 0, fa0, fb0)
    int b0 = 0, b1 = 1, b2 = 2;
    for (int step = 0; step < n_steps; ++step) {
        KVS_STEP(step, b0, b1, b2)
        const int t = b0;
        b0 = b1;
        b1 = b2;
        b2 = t;
    }
    // the last steps' spare loads must have landed before this workgroup's LDS can be handed on
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef KVS_STEP
#undef KVS_WAIT_OLDER
#undef KVS_FOURS_WITH_READS
#undef KVS_READ
#undef KVS_FETCH
#undef KVS_LOAD_TO_LDS
#undef KVS_MULTIPLY

    // lane holds, of tile (i, j), column l16 and rows 4*quad .. 4*quad+3
    if (a.k_splits > 1) {
        const size_t tile_id = (size_t)head_block * n_row_tiles + row_tile;
        const size_t n_tiles = (size_t)n_blocks * n_row_tiles;
        constexpr int kPairs = 4 * NT * 2;                         // 64-bit pieces of a thread's accumulators
        unsigned long long* mine = reinterpret_cast<unsigned long long*>(a.partials) +
                                   (blockIdx.z * n_tiles + tile_id) * (size_t)(kPairs * kTiledThreads) + threadIdx.x;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const floatx2 pv = {acc[i][j][2 * h], acc[i][j][2 * h + 1]};
                    __hip_atomic_store(mine + (size_t)((i * NT + j) * 2 + h) * kTiledThreads,
                                       __builtin_bit_cast(unsigned long long, pv), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
        __shared__ int s_is_last;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0): the device-scope stores are acknowledged
        __syncthreads();
        if (threadIdx.x == 0) {
            const int arrived = atomicAdd(a.counters + tile_id, 1);
            s_is_last = arrived == a.k_splits - 1;
            if (s_is_last) atomicExch(a.counters + tile_id, 0);
        }
        __syncthreads();
        if (!s_is_last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int ks = 0; ks < a.k_splits; ++ks) {                  // split order: the sum does not depend on arrival
            const unsigned long long* theirs = reinterpret_cast<const unsigned long long*>(a.partials) +
                                               (ks * n_tiles + tile_id) * (size_t)(kPairs * kTiledThreads) + threadIdx.x;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const floatx2 v2 = __builtin_bit_cast(
                            floatx2, __hip_atomic_load(theirs + (size_t)((i * NT + j) * 2 + h) * kTiledThreads, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT));
                        acc[i][j][2 * h] += v2[0];
                        acc[i][j][2 * h + 1] += v2[1];
                    }
        }
    }

    const bool rotate = !is_v && a.rope_cos;
    const bool fp8 = st.dtype == 2;                              // the store's type code: 1 bf16, 2 fp8
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = wm * 64 + i * 16 + quad * 4 + r;
            const long long off = row_page[row];                   // written before the first barrier
            const int pos = row_pos[row];
            const int t = pos % kPageTokens;
#pragma unroll
            for (int j = 0; j < NT / 2; ++j) {
                const int c = wn * (D / 4) + j * 16 + l16;
                float lo = acc[i][j][r], hi = acc[i][j + NT / 2][r];
                if (rotate) {                                      // dropped rows read table row 0
                    const float cs = a.rope_cos[(size_t)pos * half + c], sn = a.rope_sin[(size_t)pos * half + c];
                    const float rl = lo * cs - hi * sn, rh = hi * cs + lo * sn;
                    lo = rl;
                    hi = rh;
                }
                if (off >= 0) {
                    store_projected(st.pool, (size_t)off, fp8, is_v, t, c, lo);
                    store_projected(st.pool, (size_t)off, fp8, is_v, t, c + half, hi);
                }
            }
        }
}

// ---- tiled kernel for very many rows: two heads per workgroup -------------------------------
//
// With 256 x 128 output tiles the x and weight tiles that cross from L2 into the compute units
// (3.1 GB for 8192 rows at hidden 4096, 16 heads) take longer than the arithmetic.  This variant
// gives a workgroup 256 rows and two adjacent head blocks of the list [K heads, V heads]: a third
// fewer bytes per flop, three operand reads per eight matrix instructions instead of four, and
// one barrier per 64 matrix instructions of a wavefront instead of 32.  A wavefront owns
// 128 rows x (32 + 32) channels, the two ends of the rotary pairs of one head block.  Two LDS
// buffers of 64 KiB; a step runs in four quarters of sixteen matrix instructions (contraction
// half x row half), every quarter reading the operands of the next one:
//   q0  rows 0-63,  k 0-31    | reads x rows 64-127, k 0-31
//   q1  rows 64-127, k 0-31   | reads weights k 32-63 and x rows 0-63, k 32-63
//   q2  rows 0-63,  k 32-63   | reads x rows 64-127, k 32-63; then waits for the next step's tiles, barrier
//   q3  rows 64-127, k 32-63  | starts the loads of step + 2 into the buffer just freed; reads the
//                             | first operands of step + 1 from the other buffer
// head_dim 128 only, no contraction split (it is chosen when the tiles alone fill the chip).
constexpr int kPairCols = 256;

__global__ __launch_bounds__(kTiledThreads) void project_append_pair_kernel(ProjectArgs a)
{
    constexpr int D = 128, half = D / 2;
    constexpr int kChunks = kTileRows * (kTileK / 8) / kTiledThreads;   // 16-byte pieces per thread of either tile: 4
    const StoreView& st = a.st;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int quad = lane >> 4, l16 = lane & 15;
    const int wm = wave >> 2, wn = wave & 3;
    // grid (8, tiles per XCD): blockIdx.x is the XCD, which takes a run of consecutive output
    // tiles of the list ordered row tile by row tile (see the kernel above)
    const int n_pairs = st.Hkv;
    const int M = a.B * a.T;
    const int tile = blockIdx.x * gridDim.y + blockIdx.y;
    if (tile >= n_pairs * ((M + kTileRows - 1) / kTileRows)) return;   // padding of the last run
    const int pair = tile % n_pairs;
    const int row_tile = tile / n_pairs;
    const int hb = pair * 2 + (wn >> 1);                           // this wavefront's head block
    const int strip = wn & 1;
    const int is_v = hb >= st.Hkv;
    const int head = is_v ? hb - st.Hkv : hb;
    const int m0 = row_tile * kTileRows;

    __shared__ __attribute__((aligned(16))) unsigned short sa[2][kTileRows][kLdsRow];
    __shared__ __attribute__((aligned(16))) unsigned short sb[2][kPairCols][kLdsRow];
    __shared__ long long row_block[kTileRows];                     // slot * num_blocks + block of the row's page, -1: dropped
    __shared__ int row_pos[kTileRows];

    const unsigned short* x = static_cast<const unsigned short*>(a.x);
    const int n_steps = a.hidden / kTileK;                         // even: hidden is a multiple of 128

    if (threadIdx.x < kTileRows) {
        const int m = m0 + threadIdx.x;
        long long blk_of_row = -1;
        long pos = 0;
        if (m < M) {
            const int b = m / a.T;
            pos = (long)a.start_pos[b] + m % a.T;
            if (pos >= 0 && pos < (long)st.max_blocks_per_seq * kPageTokens) {
                int donor = st.share_map[st.layer];
                donor = donor < 0 ? 0 : (donor >= st.L ? st.L - 1 : donor);
                int slot = st.slot_of_layer[donor];
                slot = slot < 0 ? 0 : (slot >= st.n_slots ? st.n_slots - 1 : slot);
                const size_t bidx = (size_t)b * st.max_blocks_per_seq + (size_t)(pos / kPageTokens);
                const int blk = st.block_table ? st.block_table[bidx] : (int)bidx;
                if (blk >= 0 && blk < st.num_blocks) blk_of_row = (long long)slot * st.num_blocks + blk;
            }
        }
        row_block[threadIdx.x] = blk_of_row;
        row_pos[threadIdx.x] = blk_of_row < 0 ? 0 : (int)pos;
    }

    // staging as in the kernel above: piece p = 512 j + thread is piece p % 8 of row p / 8, swizzled
    // on the global side; weight rows 0-127 of the tile are the first head block, 128-255 the second
    const int s_row = threadIdx.x >> 3;
    const int s_col = ((threadIdx.x & 7) ^ (s_row & 7)) * 8;
    const int wave_row = __builtin_amdgcn_readfirstlane(wave * 8);
    const unsigned short* src_a[kChunks];
    const unsigned short* src_b[kChunks];
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
        const int m = m0 + s_row + kStageRows * j;
        src_a[j] = x + (size_t)(m < M ? m : M - 1) * a.hidden + s_col;
        const int blk = pair * 2 + j / 2;                          // rows 64 j .. 64 j + 63 of the weight tile
        const unsigned short* wbase = blk >= st.Hkv ? static_cast<const unsigned short*>(a.w_v) + (size_t)(blk - st.Hkv) * D * a.hidden
                                                    : static_cast<const unsigned short*>(a.w_k) + (size_t)blk * D * a.hidden;
        src_b[j] = wbase + (size_t)(s_row + kStageRows * (j % 2)) * a.hidden + s_col;
    }

    floatx4 acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

#define KVS_LOAD_TO_LDS(gptr, lds_ptr)                                                               \
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"                    \
                 :: "v"(gptr), "s"((unsigned)(size_t)(lds_ptr)) : "memory")
#define KVS_FETCH(step, buf)                                                                         \
    _Pragma("unroll") for (int j = 0; j < kChunks; ++j)                                              \
        KVS_LOAD_TO_LDS(src_a[j] + (step) * kTileK, &sa[buf][wave_row + kStageRows * j][0]);         \
    _Pragma("unroll") for (int j = 0; j < kChunks; ++j)                                              \
        KVS_LOAD_TO_LDS(src_b[j] + (step) * kTileK, &sb[buf][wave_row + kStageRows * j][0]);
#define KVS_READ_A(buf, kk, rh, fa)                                                                  \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
        fa[i] = *reinterpret_cast<const bf16x8*>(&sa[buf][wm * 128 + (rh) * 64 + i * 16 + l16][((kk) + quad * 8) ^ ((l16 & 7) * 8)]);
#define KVS_READ_B(buf, kk, fb)                                                                      \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                  \
        const int col = (wn >> 1) * D + (j < 2 ? 0 : half) + strip * 32 + (j % 2) * 16 + l16;        \
        fb[j] = *reinterpret_cast<const bf16x8*>(&sb[buf][col][((kk) + quad * 8) ^ ((l16 & 7) * 8)]); \
    }
#define KVS_MULTIPLY(rh, fa, fb)                                                                     \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
            acc[(rh) * 4 + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[(rh) * 4 + i][j], 0, 0, 0);
#define KVS_SPREAD_READS(per_four)                                                                   \
    _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                                  \
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);                                           \
        __builtin_amdgcn_sched_group_barrier(0x100, per_four, 0);                                    \
    }
    // all of this wavefront's loads have landed and its LDS reads are done
#define KVS_WAIT_ALL asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory")
#define KVS_STEP(step, buf)                                                                          \
    {                                                                                                \
        KVS_READ_A(buf, 0, 1, fa1)                                                                   \
        KVS_MULTIPLY(0, fa0, fb0)                                                                    \
        KVS_SPREAD_READS(1)                                                                          \
        KVS_READ_B(buf, 32, fb1)                                                                     \
        KVS_READ_A(buf, 32, 0, fa0)                                                                  \
        KVS_MULTIPLY(1, fa1, fb0)                                                                    \
        KVS_SPREAD_READS(2)                                                                          \
        KVS_READ_A(buf, 32, 1, fa1)                                                                  \
        KVS_MULTIPLY(0, fa0, fb1)                                                                    \
        KVS_SPREAD_READS(1)                                                                          \
        KVS_WAIT_ALL;                                                                                \
        __builtin_amdgcn_s_barrier();                                                                \
        if ((step) + 2 < n_steps) { KVS_FETCH((step) + 2, buf) }                                     \
        KVS_READ_B(1 - (buf), 0, fb0)                                                                \
        KVS_READ_A(1 - (buf), 0, 0, fa0)                                                             \
        KVS_MULTIPLY(1, fa1, fb1)                                                                    \
        KVS_SPREAD_READS(2)                                                                          \
    }
    bf16x8 fa0[4], fa1[4], fb0[4], fb1[4];
    KVS_FETCH(0, 0)
    KVS_WAIT_ALL;
    __builtin_amdgcn_s_barrier();
    KVS_FETCH(1, 1)
    KVS_READ_B(0, 0, fb0)
    KVS_READ_A(0, 0, 0, fa0)
    for (int step = 0; step < n_steps; step += 2) {
        KVS_STEP(step, 0)
        KVS_STEP(step + 1, 1)
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef KVS_STEP
#undef KVS_WAIT_ALL
#undef KVS_SPREAD_READS
#undef KVS_MULTIPLY
#undef KVS_READ_B
#undef KVS_READ_A
#undef KVS_FETCH
#undef KVS_LOAD_TO_LDS

    // lane holds, of tile (i, j), column l16 and rows 4*quad .. 4*quad+3
    const bool rotate = !is_v && a.rope_cos;
    const bool fp8 = st.dtype == 2;                              // the store's type code: 1 bf16, 2 fp8
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = wm * 128 + i * 16 + quad * 4 + r;
            const long long rb = row_block[row];
            const int pos = row_pos[row];
            const size_t page_off = (((size_t)(rb < 0 ? 0 : rb) * st.Hkv + head) * 2 + is_v) * (size_t)(kPageTokens * D);
            const int t = pos % kPageTokens;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = strip * 32 + j * 16 + l16;
                float lo = acc[i][j][r], hi = acc[i][j + 2][r];
                if (rotate) {                                      // dropped rows read table row 0
                    const float cs = a.rope_cos[(size_t)pos * half + c], sn = a.rope_sin[(size_t)pos * half + c];
                    const float rl = lo * cs - hi * sn, rh = hi * cs + lo * sn;
                    lo = rl;
                    hi = rh;
                }
                if (rb >= 0) {
                    store_projected(st.pool, page_off, fp8, is_v, t, c, lo);
                    store_projected(st.pool, page_off, fp8, is_v, t, c + half, hi);
                }
            }
        }
}

}  // namespace

// Which kernel a call takes and how far its contraction is split across workgroups.
namespace {
constexpr long kTargetWorkgroups = 256;                  // one per compute unit measured fastest
constexpr int kTiledFromRows = 33;                       // more rows than this: the tiled kernel

constexpr long kPairFromTiles = 192;                     // two-head tiles that fill the chip by themselves

struct ProjectPlan {
    bool tiled;
    bool pair;                   // two head blocks per workgroup
    int k_splits;
    size_t tiles;                // output tiles = arrival counters
    size_t partial_bytes;        // per tile and split
};

ProjectPlan plan_project(int Hkv, int head_dim, int hidden, int rows)
{
    ProjectPlan p;
    p.tiled = rows >= kTiledFromRows;
    p.pair = p.tiled && head_dim == 128 && (long)Hkv * ((rows + kTileRows - 1) / kTileRows) >= kPairFromTiles;
    if (p.pair) {
        p.tiles = (size_t)Hkv * ((rows + kTileRows - 1) / kTileRows);
        p.partial_bytes = 0;
        p.k_splits = 1;
        return p;
    }
    long most;                   // splits that leave every workgroup enough contraction
    int unit;                    // the contraction of one split is a multiple of this
    if (p.tiled) {
        p.tiles = (size_t)2 * Hkv * ((rows + kTileRows - 1) / kTileRows);
        p.partial_bytes = (size_t)kTiledThreads * 4 * (head_dim / 32) * 4 * sizeof(float);
        most = hidden / 1024;
        unit = 2 * kTileK;       // an even number of staged steps
    } else {
        p.tiles = (size_t)2 * Hkv * (head_dim / 32) * ((rows + 15) / 16);
        p.partial_bytes = (size_t)kThreads * 2 * sizeof(float);
        most = hidden / (kWaves * 128);
        unit = kWaves * 32;      // every wavefront gets whole steps of 32
    }
    long want = (kTargetWorkgroups + (long)p.tiles - 1) / (long)p.tiles;
    want = want > most ? most : want;
    want = want < 1 ? 1 : want;
    while (hidden % (unit * want) != 0) --want;
    p.k_splits = (int)want;
    return p;
}

}  // namespace

// The contraction is split only while the output tiles are fewer than kTargetWorkgroups, so the
// counters in use (one per tile) always fit the fixed counter region at the workspace's start.
static_assert(kTargetWorkgroups <= (long)kMaxCounters, "one arrival counter per output tile of a split contraction");

size_t project_workspace_bytes(int Hkv, int head_dim, int hidden, int rows)
{
    const ProjectPlan p = plan_project(Hkv, head_dim, hidden, rows);
    return kCounterRegionBytes + (p.k_splits > 1 ? (size_t)p.k_splits * p.tiles * p.partial_bytes : 0);
}

int launch_project_append(ProjectArgs a, void* workspace, void* stream)
{
    const int rows = a.B * a.T;
    const ProjectPlan p = plan_project(a.st.Hkv, a.st.head_dim, a.hidden, rows);
    a.k_splits = p.k_splits;
    a.counters = static_cast<int32_t*>(workspace);
    a.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kCounterRegionBytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (p.pair) {
        const dim3 grid(8, (unsigned)((p.tiles + 7) / 8), 1);
        hipLaunchKernelGGL(project_append_pair_kernel, grid, dim3(kTiledThreads), 0, s, a);
    } else if (p.tiled) {
        const dim3 grid(8, (unsigned)((p.tiles + 7) / 8), p.k_splits);
        if (a.st.head_dim == 128)
            hipLaunchKernelGGL(project_append_tiled_kernel<128>, grid, dim3(kTiledThreads), 0, s, a);
        else
            hipLaunchKernelGGL(project_append_tiled_kernel<64>, grid, dim3(kTiledThreads), 0, s, a);
    } else {
        const dim3 grid(2u * a.st.Hkv * (a.st.head_dim / 32), (unsigned)((rows + 15) / 16), p.k_splits);
        hipLaunchKernelGGL(project_append_bf16_kernel, grid, dim3(kThreads), 0, s, a);
    }
    return (int)hipGetLastError();
}

}  // namespace kvs
