// Attention over the slot-indexed, paged KV store (gfx950): the fp32 reference-precision kernel,
// the bf16 split-context MFMA kernel with its split combine, and the shared-page prefill kernels.
//
// The operation is the ordinary attention of the host model after the sharing strategy has
// redirected a layer to its donor's cache (paper Sec. 3.2): the only method-specific step in
// the kernels is the two-level lookup slot_of_layer[share_map[layer]], done on the device.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kvs_attn_tiles.h"
#include "kvs_device.h"
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kWaves = 4;              // wavefronts per workgroup of the bf16 kernel
constexpr int kThreads = kWaves * 64;
constexpr int kMinAdaptivePages = 16;  // a split sized on the device never gets fewer pages than this

// ------------------------------------------------------------------ fp32 store
// One wavefront per (sequence, query row, query head); the whole context in one pass.
// Lanes own tokens for the scores and channels for the weighted sum.
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

__global__ __launch_bounds__(64) void attn_f32_kernel(AttnArgs a)
{
    const StoreView& st = a.st;
    const int D = st.head_dim;                       // 64, 128, 192 or 256
    const int h = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x;
    const int group = st.Hq / st.Hkv;
    const int g = h / group;
    const long cap = (long)st.max_blocks_per_seq * kPageTokens;
    long n = (long)a.lens[a.lens_per_head ? b * st.Hkv + g : b] + a.lens_bias + r;
    n = n < 0 ? 0 : (n > cap ? cap : n);
    const size_t row = (((size_t)b * a.T_new + r) * st.Hq + h) * D;
    __shared__ float qs[256];
    const float* q = static_cast<const float*>(a.q) + row;
    for (int c = lane; c < D; c += 64) qs[c] = q[c];
    __syncthreads();
    const int slot = resolve_slot(st);
    const float* pool = static_cast<const float*>(st.pool);
    const float scale_log2 = 1.44269504088896340736f / sqrtf((float)D);
    float m = -INFINITY, l = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    for (long j0 = 0; j0 < n; j0 += 64) {
        const long j = j0 + lane;
        float z = -INFINITY;
        if (j < n) {
            const int blk = safe_block_of(st, b, (int)(j / kPageTokens));
            const float* kp = pool + page_offset(st, slot, blk, g) + (size_t)(j % kPageTokens) * D;
            float dot = 0.f;
            for (int c = 0; c < D; ++c) dot = fmaf(qs[c], kp[c], dot);
            z = dot * scale_log2;
        }
        const float m_new = fmaxf(m, wave_max(z));     // finite: the tile holds token j0 < n
        const float alpha = exp2f(m - m_new);
        const float p = exp2f(z - m_new);
        l = l * alpha + wave_sum(p);
        m = m_new;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] *= alpha;
        const int cnt = (int)((n - j0) < 64 ? (n - j0) : 64);
        for (int t = 0; t < cnt; ++t) {
            const float pt = __shfl(p, t);
            const long jj = j0 + t;
            const int blk = safe_block_of(st, b, (int)(jj / kPageTokens));
            const float* vp = pool + page_offset(st, slot, blk, g) + (size_t)kPageTokens * D +
                              (size_t)(jj % kPageTokens) * D;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (lane + 64 * e < D) o[e] = fmaf(pt, vp[lane + 64 * e], o[e]);
        }
    }
    const float inv = n > 0 ? 1.f / l : 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (lane + 64 * e < D) a.out[row + lane + 64 * e] = o[e] * inv;
}

// ------------------------------------------------------------------ bf16 store, MFMA
//
// Work split: grid = (Hkv, B, n_splits * n_col_groups).  A workgroup owns one kv head of one
// sequence, NT tiles of 16 query columns (a column is a (query row, head-in-group) pair; a
// decode step has one row, so one tile holds the whole GQA group) and a contiguous range of
// pages.  Its four wavefronts take pages round-robin, each streaming its pages from HBM
// straight into MFMA operand registers (the store's in-page order is the operand order) with
// kPrefetch pages in flight, and keeps a private online-softmax state.  The states merge
// through LDS at the end; with more than one split the merged, unnormalised state goes to
// the partials buffer, and the last workgroup to finish a (sequence, kv head, column group)
// folds its splits into the output.  The host sizes the grid from the store's capacity (it
// never sees the lengths); a decode launch then sizes the page range of a split by the lengths
// it finds on the device, so that a batch far below the capacity still spreads over as many
// workgroups as a full one.  (Decode launches with one length per sequence and at most 64
// sequences do not come here: kvs_decode.hip shares their pages out by tokens.)
//
// MFMA roles.  Scores: S[token][column] = K_page(16 x D) . Q^T(D x 16) with
// v_mfma_f32_16x16x32_bf16; lane l holds the scores of column l%16 for tokens 4*(l/16)..+3 of
// the page.  Two pages give a lane eight probabilities, which is exactly a B operand of the
// same instruction (contraction over 32 tokens: slots 0-3 from the first page, 4-7 from the
// second), and the V pages are stored so that a lane's registers are the matching A operand:
// O^T[channel][column] += V^T(16 x 32 tokens) . P^T(32 tokens x 16 columns) without any data
// leaving its registers.
template <int D, int NT, int kPrefetch, bool kFp8>
__global__ __launch_bounds__(kThreads) void attn_bf16_kernel(AttnArgs a)
{
    // kPrefetch: pages each wavefront keeps in flight (consumed in pairs)
    constexpr int KS = D / 32;   // k-steps of the score MFMA = 1-KiB chunks per page
    constexpr int DT = D / 16;   // 16-channel tiles of the output
    const StoreView& st = a.st;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int quad = lane >> 4, col = lane & 15;
    // Workgroup ids go round-robin over the chip's eight XCDs, so the fastest-varying index
    // must be one whose every value carries work: the kv head.  A split index there would
    // park whole XCDs on the empty splits of short sequences.
    //
    // Which (sequence, split) a workgroup takes: the grid says it (blockIdx.y = sequence,
    // blockIdx.z = split, and column group), with a fixed (or, a.adaptive == 1, device-sized) page
    // range per split; workgroups past a sequence's last split leave at once.
    const int g = blockIdx.x;
    const int b = blockIdx.y, split = NT == 1 ? (int)blockIdx.z : (int)blockIdx.z % a.n_splits;
    const int cgrp = NT == 1 ? 0 : (int)blockIdx.z / a.n_splits;
    const int group = st.Hq / st.Hkv;
    const int ncols = a.T_new * group;
    const int cap = st.max_blocks_per_seq * kPageTokens;
    const int guessed_first = split * a.pages_per_split + wave;

    // Start-up look-ups in one round trip: a single vector load in which lane 0 fetches the
    // sequence length, lane 1 the layer's donor, lanes 2..7 the page-table entries of the first
    // pages (index clamped into the table, so they can be fetched before the length says how
    // many are used) and lanes 8..63 the slots of layers 0..55; the values are then read out of
    // the lanes.  Only a donor beyond layer 55 costs a second, dependent look-up.  The first
    // pages are those of the split the host would give full sequences.
    static_assert(kPrefetch <= 6, "lanes 2..7 carry the first page-table entries");
    static_assert(NT > 1 || kPrefetch * kWaves <= kMinAdaptivePages, "a split sized on the device holds the first pages of every wavefront");
    int first_page[kPrefetch];
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        const int pg = guessed_first + j * kWaves;
        first_page[j] = pg < st.max_blocks_per_seq ? pg : st.max_blocks_per_seq - 1;
    }
    const int32_t* look = nullptr;
    if (lane == 0) look = a.lens + (a.lens_per_head ? b * st.Hkv + g : b);
    else if (lane == 1) look = st.share_map + st.layer;
    else if (lane < 8) {
        int pg = first_page[0];
#pragma unroll
        for (int j = 1; j < kPrefetch; ++j) pg = lane - 2 == j ? first_page[j] : pg;
        if (st.block_table && lane - 2 < kPrefetch) look = st.block_table + (size_t)b * st.max_blocks_per_seq + pg;
    } else if (lane - 8 < st.L) look = st.slot_of_layer + (lane - 8);
    const int looked = look ? *look : 0;
    // A decode launch sizes its splits by the lengths it finds (a.adaptive): every workgroup reads
    // all of them, in the same round trip as the look-ups above, and derives the same pages per
    // split further down.
    const bool carries_new = NT == 1 && a.k_new != nullptr;
    const bool adaptive = NT == 1 && a.adaptive;
    const int n_len = a.lens_per_head ? a.B * st.Hkv : a.B;
    int len_sum = 0, len_longest = 0;             // in pages, this lane's share of the lengths
    if (adaptive) {
        for (int i = lane; i < n_len; i += 64) {
            const int raw = a.lens[i];
            int n = raw + a.lens_bias - (carries_new ? 1 : 0);
            n = n < 0 ? 0 : (n > cap ? cap : n);
            const int pg = (n + kPageTokens - 1) / kPageTokens;
            len_sum += pg;
            len_longest = pg > len_longest ? pg : len_longest;
        }
    }
    const int len_raw = __builtin_amdgcn_readlane(looked, 0);
    const int donor_raw = __builtin_amdgcn_readlane(looked, 1);
    int first_blk[kPrefetch];
#pragma unroll
    for (int j = 0; j < kPrefetch; ++j) {
        int blk = st.block_table ? __builtin_amdgcn_readlane(looked, 2 + j) : b * st.max_blocks_per_seq + first_page[j];
        first_blk[j] = blk < 0 ? 0 : (blk >= st.num_blocks ? st.num_blocks - 1 : blk);
    }

    // the strategy's substitution: this layer reads the slot of its donor (itself if none)
    const int donor = donor_raw < 0 ? 0 : (donor_raw >= st.L ? st.L - 1 : donor_raw);
    const int slot_raw = donor < 56 ? __builtin_amdgcn_readlane(looked, 8 + donor) : st.slot_of_layer[donor];
    const int slot = slot_raw < 0 ? 0 : (slot_raw >= st.n_slots ? st.n_slots - 1 : slot_raw);

    // What depends on the sequence: the columns of this lane, one per tile, with their query
    // fragments (B operand of the score MFMA), and the keys its rows see.
    bool col_ok[NT];
    int col_row[NT];
    bf16x8 qf[NT][KS];
    const unsigned short* qbase = static_cast<const unsigned short*>(a.q);
    int n0, n_min, n_max, pages_total, new_pos;
    bool has_new;
    int n_col[NT];
    auto sequence_setup = [&]() {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const int cidx = (cgrp * NT + ct) * 16 + col;
            col_ok[ct] = cidx < ncols;
            col_row[ct] = col_ok[ct] ? cidx / group : 0;
            const int hc = col_ok[ct] ? cidx % group : 0;
            const size_t q_off = (((size_t)b * a.T_new + col_row[ct]) * st.Hq + g * group + hc) * D;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                uint4 w = make_uint4(0, 0, 0, 0);
                if (col_ok[ct]) w = *reinterpret_cast<const uint4*>(qbase + q_off + s * 32 + quad * 8);
                qf[ct][s] = __builtin_bit_cast(bf16x8, w);
            }
        }
        // A decode step that carries its own new token (k_new, v_new): the pages hold the tokens before
        // it, the token itself joins the softmax in the merge below (split 0) and is written to its
        // place in the store on the side -- no separate append launch, and nothing here waits for the write.
        new_pos = len_raw - 1;
        has_new = carries_new && new_pos >= 0 && new_pos < cap;
        // keys visible to query row 0; row r sees n0 + r
        n0 = len_raw + a.lens_bias - (carries_new ? 1 : 0);
        n0 = n0 < 0 ? 0 : n0;
        if (n0 > cap - (a.T_new - 1)) n0 = cap - (a.T_new - 1);
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) n_col[ct] = n0 + col_row[ct];
        // rows covered by the workgroup bound the pages it needs
        const int c_lo = cgrp * NT * 16;
        int c_hi = c_lo + NT * 16 - 1;
        if (c_hi > ncols - 1) c_hi = ncols - 1;
        n_min = n0 + c_lo / group;          // fewest keys any of its rows sees
        n_max = n0 + c_hi / group;          // most keys, = tokens certainly stored
        pages_total = (n_max + kPageTokens - 1) / kPageTokens;
    };
    sequence_setup();

    // Where the launch does not size its splits itself, or this sequence fills its table (then the
    // sizing below most likely ends at the host's figure), the first pages go out at once, for the
    // split the host would give full sequences (what the look-up above fetched the page-table
    // entries for) ...
    const void* pool = st.pool;
    using Raw = std::conditional_t<kFp8, PageRegs8<D>, PageRegs<D>>;    // a page as it sits in the store
    Raw buf[kPrefetch];
    const bool guess_early = !adaptive || pages_total + 4 * a.want_splits > st.max_blocks_per_seq;
    if (guess_early) {
        int hi = guessed_first - wave + a.pages_per_split;
        if (hi > pages_total) hi = pages_total;
        const int guessed_pages = guessed_first < hi ? (hi - guessed_first + kWaves - 1) / kWaves : 0;
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j)
            if (j < guessed_pages) load_page(buf[j], pool, page_offset(st, slot, first_blk[j], g), lane);
    }
    // ... and while they travel the launch's pages per split are worked out from all its lengths:
    // the mean length shared out as the host shares out a full sequence, so that about as many
    // workgroups carry keys whatever the lengths are.  Every workgroup derives the same number.
    int pps = a.pages_per_split;
    if (adaptive) {
        int sum = len_sum, longest = len_longest;
        if (n_len <= 16) {                       // one length per lane: read the lanes out, add on the scalar side
            sum = 0;
            longest = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int pg = __builtin_amdgcn_readlane(len_sum, i);
                sum += pg;
                longest = pg > longest ? pg : longest;
            }
        } else {                                 // lanes from n_len on hold zero: lane 0 ends with all of it
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                if (off >= n_len) continue;
                sum += __shfl_xor(sum, off);
                const int other = __shfl_xor(longest, off);
                longest = other > longest ? other : longest;
            }
            sum = __builtin_amdgcn_readfirstlane(sum);
            longest = __builtin_amdgcn_readfirstlane(longest);
        }
        const int sharers = n_len * a.want_splits;
        pps = ((sum + sharers - 1) / sharers + 3) & ~3;
        // the grid has a.n_splits split indices per sequence: the longest must fit
        const int fit = ((longest + a.n_splits - 1) / a.n_splits + 3) & ~3;
        pps = pps > fit ? pps : fit;
        pps = pps > kMinAdaptivePages ? pps : kMinAdaptivePages;
    }
    const int page_lo = split * pps;
    const int my_first = page_lo + wave;
    int page_hi = page_lo + pps;
    if (page_hi > pages_total) page_hi = pages_total;
    const int my_pages = my_first < page_hi ? (page_hi - my_first + kWaves - 1) / kWaves : 0;
    // Splits that hold keys for this (sequence, column group).  Workgroups past them leave at
    // once; if there is at most one, split 0 writes the output itself and no state is published.
    const int live_splits = (pages_total + pps - 1) / pps;
    if (split > 0 && split >= live_splits) return;
    // Where nothing was guessed, or the lengths moved this split, its own first pages are loaded (a split
    // that starts where it was guessed to has the same first pages: neither size is below
    // kPrefetch pages per wavefront, so only the sequence's end can cut them short).
    if (!guess_early || my_first != guessed_first) {
#pragma unroll
        for (int j = 0; j < kPrefetch; ++j)
            if (j < my_pages)
                load_page(buf[j], pool, page_offset(st, slot, safe_block_of(st, b, my_first + j * kWaves), g), lane);
    }

    const float scale_log2 = 1.44269504088896340736f * (D == 128 ? 0.08838834764831845f : 0.125f);
    float m[NT], l[NT];
    floatx4 o[NT][DT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        m[ct] = -INFINITY;
        l[ct] = 0.f;
#pragma unroll
        for (int c = 0; c < DT; ++c) o[ct][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // Pages are consumed two at a time: 32 tokens fill the contraction depth of the 16x16x32
    // MFMA for P.V as well, two independent score chains overlap, and one softmax update
    // (one column maximum, one reference test) serves both pages.  A wavefront with an odd
    // page count pairs its last page with an absent one whose scores are masked and whose
    // operand registers are zero.
    static_assert(kPrefetch % 2 == 0, "buffers are used in pairs");
    const int my_pairs = (my_pages + 1) / 2;
    for (int p0 = 0; p0 < my_pairs; p0 += kPrefetch / 2) {
#pragma unroll
        for (int jj = 0; jj < kPrefetch / 2; ++jj) {
            const int pr = p0 + jj;
            if (pr >= my_pairs) break;
            Raw& pa = buf[2 * jj];
            Raw& pb = buf[2 * jj + 1];
            const int ka = 2 * pr, kb = ka + 1;
            const bool have_b = kb < my_pages;
            const int page_a = my_first + ka * kWaves, page_b = my_first + kb * kWaves;
            const int tok_a = page_a * kPageTokens, tok_b = page_b * kPageTokens;

            if constexpr (kFp8) {
                PageRegs<D> wa, wb;                                   // widened to bf16 operands
                widen<D>(pa, wa);
                widen<D>(pb, wb);                                     // an absent page is zeroed by consume_pair
                consume_pair<D, NT>(wa, wb, have_b, tok_a, tok_b, n_min, n_max, n_col, qf, m, l, o, quad, scale_log2);
            } else {
                consume_pair<D, NT>(pa, pb, have_b, tok_a, tok_b, n_min, n_max, n_col, qf, m, l, o, quad, scale_log2);
            }
            if (ka + kPrefetch < my_pages)
                load_page(pa, pool, page_offset(st, slot, safe_block_of(st, b, page_a + kPrefetch * kWaves), g), lane);
            if (kb + kPrefetch < my_pages)
                load_page(pb, pool, page_offset(st, slot, safe_block_of(st, b, page_b + kPrefetch * kWaves), g), lane);
        }
    }

    __shared__ float lds_new_score[16];               // log2-domain score of the step's own token, per column
    const bool adds_new = has_new && split == 0;
    // the new row as the store will hold it: as given (bf16 store), rounded to E4M3 (fp8 store)
    auto as_stored = [](unsigned short h) -> float {
        const unsigned w = kFp8 ? e4m3_to_bf16(bf16_to_e4m3(h)) : h;
        return __uint_as_float(w << 16);
    };
    if (adds_new) {
        const unsigned short* k_row = static_cast<const unsigned short*>(a.k_new) + ((size_t)b * st.Hkv + g) * D;
        const unsigned short* v_row = static_cast<const unsigned short*>(a.v_new) + ((size_t)b * st.Hkv + g) * D;
        // its place in the store, for the steps to come (this launch masks that position)
        const int blk = block_of(st, b, new_pos / kPageTokens);
        if (blk >= 0 && blk < st.num_blocks) {
            const int t = new_pos % kPageTokens;
            if constexpr (kFp8) {
                unsigned char* kp = static_cast<unsigned char*>(st.pool) + page_offset(st, slot, blk, g);
                unsigned char* vp = kp + kPageTokens * D;
                if ((int)threadIdx.x < D / 8) {
                    const uint4 w = *reinterpret_cast<const uint4*>(k_row + threadIdx.x * 8);
                    const unsigned kw[4] = {w.x, w.y, w.z, w.w};
                    unsigned lo = 0, hi = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        lo |= bf16_to_e4m3((kw[e >> 1] >> ((e & 1) * 16)) & 0xffffu) << (8 * e);
                        hi |= bf16_to_e4m3((kw[2 + (e >> 1)] >> ((e & 1) * 16)) & 0xffffu) << (8 * e);
                    }
                    *reinterpret_cast<uint2*>(kp + k_index_fp8(t, threadIdx.x * 8)) = make_uint2(lo, hi);
                }
                if ((int)threadIdx.x < D) vp[v_index_fp8(t, threadIdx.x)] = (unsigned char)bf16_to_e4m3(v_row[threadIdx.x]);
            } else {
                unsigned short* kp = static_cast<unsigned short*>(st.pool) + page_offset(st, slot, blk, g);
                unsigned short* vp = kp + kPageTokens * D;
                if ((int)threadIdx.x < D / 8)
                    *reinterpret_cast<uint4*>(kp + k_index_bf16(t, threadIdx.x * 8)) =
                        *reinterpret_cast<const uint4*>(k_row + threadIdx.x * 8);
                if ((int)threadIdx.x < D) vp[v_index_bf16(t, threadIdx.x)] = v_row[threadIdx.x];
            }
        }
        // q . k_new for the 16 columns: a wavefront takes four columns, sixteen lanes each
        constexpr int CH = D / 16;
        const int cc = wave * 4 + quad, part = col;
        float dot = 0.f;
        if (cc < ncols) {
            const unsigned short* qr = qbase + (((size_t)b * a.T_new) * st.Hq + g * group + cc) * D + part * CH;
#pragma unroll
            for (int e = 0; e < CH; ++e)
                dot += __uint_as_float((unsigned)qr[e] << 16) * as_stored(k_row[part * CH + e]);
        }
#pragma unroll
        for (int o_ = 8; o_ > 0; o_ >>= 1) dot += __shfl_xor(dot, o_);
        const float scale = 1.44269504088896340736f * (D == 128 ? 0.08838834764831845f : 0.125f);
        if (part == 0) lds_new_score[cc] = cc < ncols ? dot * scale : -INFINITY;   // read after the merge's barrier
    }

    // merge the four wavefront states, one column tile at a time
    __shared__ float lds_o[kWaves][16][D + 4];
    __shared__ float lds_m[kWaves][16];
    __shared__ float lds_l[kWaves][16];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const float lsum = column_sum(l[ct]);
        if (ct > 0) __syncthreads();
        if (quad == 0) {
            lds_m[wave][col] = m[ct];
            lds_l[wave][col] = lsum;
        }
#pragma unroll
        for (int c = 0; c < DT; ++c)
            *reinterpret_cast<floatx4*>(&lds_o[wave][col][c * 16 + quad * 4]) = o[ct][c];
        __syncthreads();
        for (int idx = threadIdx.x; idx < 16 * (D / 4); idx += kThreads) {
            const int cc = idx / (D / 4);
            const int d4 = (idx % (D / 4)) * 4;
            const int cidx = (cgrp * NT + ct) * 16 + cc;
            if (cidx >= ncols) continue;
            float mw[kWaves], M = -INFINITY;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { mw[w] = lds_m[w][cc]; M = fmaxf(M, mw[w]); }
            const float m_new_tok = adds_new ? lds_new_score[cc] : -INFINITY;
            M = fmaxf(M, m_new_tok);
            const float M_use = M == -INFINITY ? 0.f : M;
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
            float lt = 0.f;
            if (adds_new) {                                   // weight 2^(score - M), value row v_new
                const unsigned short* v_row = static_cast<const unsigned short*>(a.v_new) + ((size_t)b * st.Hkv + g) * D + d4;
                const float wgt = __builtin_amdgcn_exp2f(m_new_tok - M_use);
                acc = wgt * floatx4{as_stored(v_row[0]), as_stored(v_row[1]), as_stored(v_row[2]), as_stored(v_row[3])};
                lt = wgt;
            }
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float wgt = __builtin_amdgcn_exp2f(mw[w] - M_use);
                acc += wgt * *reinterpret_cast<const floatx4*>(&lds_o[w][cc][d4]);
                lt += wgt * lds_l[w][cc];
            }
            const int r = cidx / group, hc = cidx % group;
            const size_t row = ((size_t)b * a.T_new + r) * st.Hq + g * group + hc;
            if (live_splits <= 1) {
                const float inv = lt > 0.f ? 1.f / lt : 0.f;
                *reinterpret_cast<floatx4*>(a.out + row * D + d4) = acc * inv;
            } else {
                float* part = a.partials + (row * a.n_splits + split) * (size_t)(D + 2);     // one record per (row, split)
                // (D + 2) floats per record keeps 8-byte alignment only: store as pairs
                publish_pair(part + d4, acc[0], acc[1]);
                publish_pair(part + d4 + 2, acc[2], acc[3]);
                if (d4 == 0) publish_pair(part + D, M, lt);
            }
        }
    }
    if (live_splits <= 1) return;

    const int n_col_groups = gridDim.z / a.n_splits;
    if (!arrived_last(a.counters + ((size_t)b * st.Hkv + g) * n_col_groups + cgrp, live_splits)) return;
    merge_splits<D>(a, b, g, cgrp * NT * 16, NT * 16, ncols, group, live_splits, kThreads, a.n_splits, 1, 0);
}

// ------------------------------------------------------------------ wide prefill
// Prefill with many query columns per (sequence, kv head).  The kernel above gives a workgroup
// 64 columns and lets its wavefronts share out the pages, so every 64 columns stream the whole
// prefix again: 64 flops per byte, which the memory system, not the matrix cores, then bounds.
// Here the wavefronts of a workgroup each take their own columns (256 per workgroup as 8 x 32, or
// 64 as 4 x 16 when a head has fewer) and all consume the same page pair.  The pair is fetched
// once per workgroup (each thread a few 16-byte pieces, a few pairs ahead, in registers) and laid
// into LDS in operand order: keys as the plain image of the two pages (the in-page order is the
// operand order, so a lane's operand is the 16 bytes at its own index); values the same in the
// small variant, and in the large one with the two pages' halves interleaved, so that a lane reads
// the eight-token operand of the value product in one piece.  Each wavefront reads them back after
// a barrier.  A wavefront owns its columns for all the pairs of its workgroup: no state is merged
// inside a workgroup.  grid.z = column blocks x context splits: with one split the output is
// written normalised; with several (few sequences x heads, long context: the host splits the pairs
// over workgroups to fill the chip) every workgroup publishes its columns' states and the last to
// arrive merges them.  Causality: a wavefront skips the pairs that lie beyond the last key any of
// its columns sees.
// NT 16-column tiles per wavefront, WAVES wavefronts: NT * 16 * WAVES columns per workgroup.
// kReadOnce: one column block per (sequence, kv head), so that every page is read exactly once per
// launch and is streamed past the caches (nontemporal loads); with several blocks the later ones
// find it in L2.  A template parameter, not a test of the grid size inside the kernel: a load
// chosen by a run-time condition between the two kinds is folded into one plain load.
// kFp8: the slots hold E4M3 bytes.  A page is fetched as it is stored (half the bytes, half the
// registers in flight) and widened to bf16 once, by the thread that lays it into LDS; LDS holds the
// bf16 page and everything downstream is the same code.
template <int D, int NT, int WAVES, bool kReadOnce, bool kFp8>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(NT == 1 ? (kFp8 ? 3 : 4) : 2)))
void attn_bf16_wide_kernel(AttnArgs a)
{
    constexpr int KS = D / 32, DT = D / 16;
    constexpr int kWideThreads = WAVES * 64, kWideCols = WAVES * NT * 16;
    // The large variant lays the values into LDS as the eight-token operands of a page pair (no
    // register shuffling before the value product); the small one, tight on registers at three
    // wavefronts per SIMD, keeps the plain page image and concatenates in registers.
    constexpr bool kCatV = NT > 1;
    constexpr int kPageVecs = kPageTokens * D * 2 * 2 / 16;        // 16-byte pieces of one bf16 page (K then V)
    constexpr int kRawVecs = kFp8 ? kPageVecs / 2 : kPageVecs;     // and of the page as the store holds it
    const StoreView& st = a.st;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int quad = lane >> 4, col = lane & 15;
    // later column blocks see more keys (causality) and run longer: they are started first, so
    // that the launch does not end on its longest workgroups
    int g, b, n_cblk, split, turns = 1, cblk_first, cblk_second = 0;
    if (NT == 2 && !kReadOnce && a.col_blocks > 0) {               // (only that variant is ever launched so)
        // 1-D grid, no context split: workgroup ids go round-robin over the eight XCDs, so ids
        // 8 k + x, k = 0, 1, ... are consecutive on XCD x.  The workgroups of one (sequence, kv head)
        // take consecutive k: they run side by side on one XCD, walk the same pages at about the same
        // time, and all but the first find a page in that XCD's L2.  Either a workgroup per column
        // block, or (col_paired) a workgroup takes the k-th longest block and then the k-th shortest,
        // so that the workgroups of the launch do the same amount of work.
        n_cblk = a.col_blocks;
        split = 0;
        const int per = a.col_paired ? (n_cblk + 1) / 2 : n_cblk;  // workgroups per (sequence, kv head)
        const int xcd = (int)blockIdx.x % 8, k = (int)blockIdx.x / 8;
        const int bg = (k / per) * 8 + xcd;
        if (bg >= a.B * st.Hkv) return;                            // padding of the last round
        g = bg % st.Hkv;
        b = bg / st.Hkv;
        // block i of a prompt walks about i + 1 times the pairs of block 0: an even number of blocks pairs
        // i with n - 1 - i; an odd number leaves the longest block by itself and pairs the others so that
        // every pair is as long as it (exactly so when the chunk starts the sequence)
        const int which = k % per, odd = n_cblk & 1;
        cblk_first = n_cblk - 1 - which;
        cblk_second = which - odd;
        turns = a.col_paired && cblk_second >= 0 ? 2 : 1;
    } else {
        // grid (kv head, sequence, column blocks x context splits), the split index fastest
        g = blockIdx.x;
        b = blockIdx.y;
        n_cblk = gridDim.z / a.n_splits;
        split = (int)blockIdx.z % a.n_splits;
        cblk_first = n_cblk - 1 - (int)blockIdx.z / a.n_splits;
    }
    const int group = st.Hq / st.Hkv;
    const int ncols = a.T_new * group;
    const int cap = st.max_blocks_per_seq * kPageTokens;
    const int slot = resolve_slot(st);

    int n0 = a.lens[b] + a.lens_bias;                              // keys visible to query row 0
    n0 = n0 < 0 ? 0 : n0;
    if (n0 > cap - (a.T_new - 1)) n0 = cap - (a.T_new - 1);

    for (int turn = 0; turn < turns; ++turn) {
    const int cblk = turn == 0 ? cblk_first : cblk_second;
    // this lane's columns and their query fragments
    const int c_lo = cblk * kWideCols + wave * (NT * 16);
    size_t q_off[NT];
    bool col_ok[NT];
    int n_col[NT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const int cidx = c_lo + ct * 16 + col;
        col_ok[ct] = cidx < ncols;
        const int row = col_ok[ct] ? cidx / group : 0;
        const int hc = col_ok[ct] ? cidx % group : 0;
        q_off[ct] = (((size_t)b * a.T_new + row) * st.Hq + g * group + hc) * D;
        n_col[ct] = n0 + row;
    }
    bf16x8 qf[NT][KS];
    const unsigned short* qbase = static_cast<const unsigned short*>(a.q);
#pragma unroll
    for (int ct = 0; ct < NT; ++ct)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint4 w = make_uint4(0, 0, 0, 0);
            if (col_ok[ct]) w = *reinterpret_cast<const uint4*>(qbase + q_off[ct] + s * 32 + quad * 8);
            qf[ct][s] = __builtin_bit_cast(bf16x8, w);
        }
    const bool wave_has = c_lo < ncols;
    int c_hi = c_lo + NT * 16 - 1;
    if (c_hi > ncols - 1) c_hi = ncols - 1;
    const int n_min = wave_has ? n0 + c_lo / group : 0;            // fewest keys any of the wavefront's rows sees
    const int n_max = wave_has ? n0 + c_hi / group : 0;            // most
    const int my_pages = (n_max + kPageTokens - 1) / kPageTokens;
    int wg_hi = cblk * kWideCols + kWideCols - 1;
    if (wg_hi > ncols - 1) wg_hi = ncols - 1;
    const int wg_pages = (n0 + wg_hi / group + kPageTokens - 1) / kPageTokens;
    // With few (sequence, kv head) pairs and a long context the pairs of pages are also split
    // over workgroups (a.pages_per_split is a multiple of four): this one takes pairs pair_lo ..
    // pair_lo + wg_pairs, and where more than one split has work the states are published and merged
    // by the last to arrive, as in the kernel above.
    const int all_pairs = (wg_pages + 1) / 2;
    const int pairs_per_split = a.pages_per_split / 2;
    const int live_splits = (all_pairs + pairs_per_split - 1) / pairs_per_split;
    if (split > 0 && split >= live_splits) return;
    const int pair_lo = split * pairs_per_split;
    const int wg_pairs = all_pairs - pair_lo < pairs_per_split ? (all_pairs > pair_lo ? all_pairs - pair_lo : 0) : pairs_per_split;

    // The small bf16 variant takes its pages from global memory straight into LDS (the plain page
    // image is exactly what a wavefront-wide 16-byte-per-lane load lays down): no staging registers,
    // no LDS store instructions.
    constexpr bool kDma = NT == 1 && !kFp8 && kPageVecs % kWideThreads == 0;
    __shared__ u32x4 tile[2][2 * kPageVecs];
    using Elem = std::conditional_t<kFp8, unsigned char, unsigned short>;   // page_offset counts elements
    const Elem* pool = static_cast<const Elem*>(st.pool);
    // kDepth page pairs are in flight from global memory to registers at any time (a workgroup
    // walks its pairs one after another, so the bytes it keeps in flight are all that hides the
    // memory latency); slot k of `stage` holds the pairs with index = k mod kDepth.
    constexpr int kDepth = NT == 1 ? 2 : 4;                        // fewer registers where occupancy matters more
    constexpr int kPasses = (kRawVecs + kWideThreads - 1) / kWideThreads;    // passes of the workgroup over one page
    u32x4 stage[kDepth][2 * kPasses];
    // Each page of the pair is copied by whole passes of the workgroup, so that the page index --
    // and with it the page-table entry -- is the same for every thread of a pass: a scalar load,
    // which does not queue behind the vector loads already in flight.
#define KVS_FETCH_PAIR(pair, slot_)                                                                   \
    _Pragma("unroll") for (int pg = 0; pg < 2; ++pg) {                                                \
        int page = 2 * (pair_lo + (pair)) + pg;                                                       \
        page = page < wg_pages ? page : (wg_pages > 0 ? wg_pages - 1 : 0);   /* past the end: a page nobody reads */ \
        const u32x4* src = reinterpret_cast<const u32x4*>(pool + page_offset(st, slot, safe_block_of_uniform(st, b, page), g)); \
        _Pragma("unroll") for (int i = 0; i < kPasses; ++i) {                                         \
            const int v = i * kWideThreads + (int)threadIdx.x;                                        \
            if (kRawVecs % kWideThreads == 0 || v < kRawVecs)                                         \
                stage[slot_][pg * kPasses + i] = kReadOnce ? __builtin_nontemporal_load(src + v) : src[v];  \
        }                                                                                             \
    }
    // bf16 piece `v_` of page pg (0 / 1) of a pair into its place in tile[buf]
#define KVS_STORE_PIECE(buf, pg, v_, piece_)                                                          \
    {                                                                                                 \
        const int vv = (v_);                                                                          \
        const u32x4 pc = (piece_);                                                                    \
        if (!kCatV) {                                            /* the page as it is */              \
            tile[buf][(pg) * kPageVecs + vv] = pc;                                                    \
        } else if (vv < KS * 64) {                               /* a key piece: the page's own order */ \
            tile[buf][(pg) * KS * 64 + vv] = pc;                                                      \
        } else {                                                 /* a value piece: halves to two pair operands */ \
            const int vs = (vv - KS * 64) >> 6, vl = vv & 63;                                         \
            u32x2* dst = reinterpret_cast<u32x2*>(&tile[buf][2 * KS * 64 + (2 * vs) * 64 + vl]) + (pg); \
            dst[0] = u32x2{pc.x, pc.y};                                                               \
            dst[2 * 64] = u32x2{pc.z, pc.w};                                                          \
        }                                                                                             \
    }
#define KVS_PUT_PAIR(buf, slot_)                                                                      \
    _Pragma("unroll") for (int pg = 0; pg < 2; ++pg)                                                  \
        _Pragma("unroll") for (int i = 0; i < kPasses; ++i) {                                         \
            const int v = i * kWideThreads + (int)threadIdx.x;                                        \
            if (kRawVecs % kWideThreads == 0 || v < kRawVecs) {                                       \
                const u32x4 raw = stage[slot_][pg * kPasses + i];                                     \
                if constexpr (kFp8) {                            /* raw block r -> bf16 blocks 2r, 2r + 1 */ \
                    u32x4 w0, w1;                                                                     \
                    widen_piece(raw, w0, w1);                                                         \
                    const int at0 = (v >> 6) * 128 + (v & 63);                                        \
                    KVS_STORE_PIECE(buf, pg, at0, w0)                                                 \
                    KVS_STORE_PIECE(buf, pg, at0 + 64, w1)                                            \
                } else {                                                                              \
                    KVS_STORE_PIECE(buf, pg, v, raw)                                                  \
                }                                                                                     \
            }                                                                                         \
        }

    const float scale_log2 = 1.44269504088896340736f * (D == 128 ? 0.08838834764831845f : 0.125f);
    float m[NT], l[NT];
    floatx4 o[NT][DT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        m[ct] = kNoReference;                                      // finite, far below any score: pair_softmax_by_sum
        l[ct] = 0.f;
#pragma unroll
        for (int c = 0; c < DT; ++c) o[ct][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // One step of the workgroup: the wavefront's softmax / accumulation over pair `pair` (buffer
    // j & 1), then pair + 1 goes from its register slot into the other buffer and pair + 1 + kDepth
    // is fetched into that slot.  kAll: every fetch, LDS write and barrier is known to be due, and
    // the step is straight-line code.
#define KVS_WIDE_COMPUTE(pair, buf)                                                                   \
    {                                                                                                 \
        const int tok_a = 2 * (pair_lo + (pair)) * kPageTokens, tok_b = tok_a + kPageTokens;          \
        if (tok_a < n_max) {                                                                          \
            const bool have_b = 2 * (pair_lo + (pair)) + 1 < my_pages;                                \
            /* keys first; the value operands are fetched from LDS once the score products are */     \
            /* issued, into the registers the keys no longer need */                                  \
            constexpr int kSecond = kCatV ? KS * 64 : kPageVecs;   /* where the second page's keys start */ \
            u32x4 ka[KS], kb[KS];                                                                     \
            _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                          \
                ka[s] = tile[buf][s * 64 + lane];                                                     \
                kb[s] = tile[buf][kSecond + s * 64 + lane];        /* an absent second page is zeroed below */ \
            }                                                                                         \
            floatx4 sa[NT], sb[NT];                                                                   \
            bf16x8 pf[NT];                                                                            \
            pair_qk<D, NT>(ka, kb, have_b, qf, sa, sb);                                               \
            if constexpr (kCatV) {                                                                    \
                u32x4 vcat[DT];                                                                       \
                _Pragma("unroll") for (int c = 0; c < DT; ++c) vcat[c] = tile[buf][2 * KS * 64 + c * 64 + lane]; \
                pair_softmax_by_sum<D, NT>(sa, sb, have_b, tok_a, tok_b, n_min, n_col, m, l, o, quad, scale_log2, pf); \
                pair_values_cat<D, NT>(vcat, have_b, tok_a, tok_b, n_max, quad, pf, o);               \
            } else {                                                                                  \
                u32x4 va[KS], vb[KS];                                                                 \
                _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                      \
                    va[s] = tile[buf][(KS + s) * 64 + lane];                                          \
                    vb[s] = tile[buf][kPageVecs + (KS + s) * 64 + lane];                              \
                }                                                                                     \
                pair_softmax_by_sum<D, NT>(sa, sb, have_b, tok_a, tok_b, n_min, n_col, m, l, o, quad, scale_log2, pf); \
                pair_values<D, NT>(va, vb, have_b, tok_a, tok_b, n_max, quad, pf, o);                 \
            }                                                                                         \
        }                                                                                             \
    }
#define KVS_WIDE_STEP(pair, j, kAll)                                                                  \
    if (kAll || (pair) < wg_pairs) {                                                                  \
        const int buf = (j) & 1;                                   /* kDepth is even */               \
        KVS_WIDE_COMPUTE(pair, buf)                                                                   \
        if (kAll || (pair) + 1 < wg_pairs) {                                                          \
            KVS_PUT_PAIR(buf ^ 1, ((j) + 1) % kDepth)              /* that buffer was last read before the previous barrier */ \
            if (kAll || (pair) + 1 + kDepth < wg_pairs) { KVS_FETCH_PAIR((pair) + 1 + kDepth, ((j) + 1) % kDepth) } \
        }                                                                                             \
        __syncthreads();                                                                              \
    }
    // The pairs whose every fetch is due (all but the last kDepth + 1, in whole rounds) run as
    // straight-line code with a fixed number of loads per step, so that the compiler's waits name
    // exactly the loads they need.  With a branch around any load it must assume the fewest loads in
    // flight, and every wait then drains all of them, which undoes the prefetch.  The query
    // fragments are waited for once, before the loop, for the same reason (the compiler cannot see
    // that a wavefront without keys never uses them and would wait for them inside it).  The last
    // pairs take the same step with its branches.
    // (Only in the 8-wavefront variant: the small one, bound by HBM and not by its own latencies,
    // measured 128 us with exact waits against 122 us with the draining ones on the 64-row chunk.)
    if constexpr (kDma) {
        static_assert(!kDma || kPageVecs % kWideThreads == 0, "whole passes of the workgroup over a page");
        // Direct loads: pair p lives in buffer p % 2.  At step i the loads of pair i + 1 are issued
        // into the buffer pair i - 1 was read from (all wavefronts have passed the barrier behind it),
        // pair i is consumed, and before the barrier every wavefront waits until its loads have
        // landed.  One pair of look-ahead is the measured optimum on the 64-row chunk of the
        // Llama-2-13B shape: two pairs ahead with exact waits took 128 us against 115 us (640
        // workgroups already keep 10 MB in flight; more only lengthens the queues of the memory).
        // The loads are assembly (the compiler would otherwise hold every LDS read behind them) and
        // so are the waits.
#define KVS_DMA_PAIR(pair, buf)                                                                       \
        _Pragma("unroll") for (int pg = 0; pg < 2; ++pg) {                                            \
            int page = 2 * (pair_lo + (pair)) + pg;                                                   \
            page = page < wg_pages ? page : (wg_pages > 0 ? wg_pages - 1 : 0);                        \
            const u32x4* src = reinterpret_cast<const u32x4*>(pool + page_offset(st, slot, safe_block_of_uniform(st, b, page), g)); \
            _Pragma("unroll") for (int i = 0; i < kPasses; ++i) {                                     \
                const unsigned to = (unsigned)(size_t)&tile[buf][pg * kPageVecs + i * kWideThreads + wave * 64]; \
                if constexpr (kReadOnce)                                                              \
                    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" \
                                 :: "v"(src + i * kWideThreads + (int)threadIdx.x), "s"(to) : "memory"); \
                else                                                                                  \
                    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"  \
                                 :: "v"(src + i * kWideThreads + (int)threadIdx.x), "s"(to) : "memory"); \
            }                                                                                         \
        }
#define KVS_WAIT_LANDED asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[ct][ks]));   // the queries have arrived
        if (wg_pairs > 0) { KVS_DMA_PAIR(0, 0) }
        KVS_WAIT_LANDED
        __builtin_amdgcn_s_barrier();
        for (int p0 = 0; p0 < wg_pairs; p0 += 2) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int pair = p0 + j;
                if (pair < wg_pairs) {                                 // uniform over the workgroup
                    if (pair + 1 < wg_pairs) { KVS_DMA_PAIR(pair + 1, j ^ 1) }
                    KVS_WIDE_COMPUTE(pair, j)
                    KVS_WAIT_LANDED
                    __builtin_amdgcn_s_barrier();
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#undef KVS_WAIT_LANDED
#undef KVS_DMA_PAIR
    } else {
    const int n_straight = NT > 1 && wg_pairs > kDepth + 1 ? (wg_pairs - kDepth - 1) / kDepth * kDepth : 0;
    if (n_straight > 0) {
#pragma unroll
        for (int j = 0; j < kDepth; ++j) { KVS_FETCH_PAIR(j, j) }
        KVS_PUT_PAIR(0, 0)
        KVS_FETCH_PAIR(kDepth, 0)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[ct][ks]));
        __syncthreads();
        for (int p0 = 0; p0 < n_straight; p0 += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) { KVS_WIDE_STEP(p0 + j, j, true) }
        }
    } else {
#pragma unroll
        for (int j = 0; j < kDepth; ++j)
            if (j < wg_pairs) { KVS_FETCH_PAIR(j, j) }
        if (wg_pairs > 0) {
            KVS_PUT_PAIR(0, 0)
            if (kDepth < wg_pairs) { KVS_FETCH_PAIR(kDepth, 0) }
        }
        __syncthreads();
    }
    for (int p0 = n_straight; p0 < wg_pairs; p0 += kDepth) {
#pragma unroll
        for (int j = 0; j < kDepth; ++j) { KVS_WIDE_STEP(p0 + j, j, false) }
    }
    }
#undef KVS_WIDE_STEP
#undef KVS_WIDE_COMPUTE
#undef KVS_FETCH_PAIR
#undef KVS_PUT_PAIR
#undef KVS_STORE_PIECE

    // lane holds channels c*16 + 4*quad .. +3 of its column in o[ct][c]
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const float lsum = column_sum(l[ct]);
        if (!col_ok[ct]) continue;
        const int cidx = c_lo + ct * 16 + col;
        const size_t row = ((size_t)b * a.T_new + cidx / group) * st.Hq + g * group + cidx % group;
        if (live_splits <= 1) {                                    // the only split with keys: the finished rows
            const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
            float* dst = a.out + row * D + quad * 4;
#pragma unroll
            for (int c = 0; c < DT; ++c) *reinterpret_cast<floatx4*>(dst + c * 16) = o[ct][c] * inv;
        } else {                                                   // this split's state of the column
            float* part = a.partials + (row * a.n_splits + split) * (size_t)(D + 2);
#pragma unroll
            for (int c = 0; c < DT; ++c) {
                publish_pair(part + c * 16 + quad * 4, o[ct][c][0], o[ct][c][1]);
                publish_pair(part + c * 16 + quad * 4 + 2, o[ct][c][2], o[ct][c][3]);
            }
            if (quad == 0) publish_pair(part + D, lsum > 0.f ? m[ct] : -INFINITY, lsum)   /* saw nothing: as the merge expects it */;
        }
    }
    if constexpr (NT == 2 && !kReadOnce) {                         // the variant that may take a second turn
        if (live_splits > 1 && arrived_last(a.counters + ((size_t)b * st.Hkv + g) * n_cblk + cblk, live_splits))
            merge_splits<D>(a, b, g, cblk * kWideCols, kWideCols, ncols, group, live_splits, kWideThreads, a.n_splits, 1, 0);
    } else {
        if (live_splits <= 1) return;
        if (!arrived_last(a.counters + ((size_t)b * st.Hkv + g) * n_cblk + cblk, live_splits)) return;
        merge_splits<D>(a, b, g, cblk * kWideCols, kWideCols, ncols, group, live_splits, kWideThreads, a.n_splits, 1, 0);
    }
    }   // turns
}

template <int D, bool kFp8>
int launch_bf16(const AttnArgs& args, hipStream_t s)
{
    AttnArgs a = args;
    a.col_blocks = a.col_paired = 0;
    const int group = a.st.Hq / a.st.Hkv;
    if (a.T_new == 1) {
        dim3 grid(a.st.Hkv, a.B, a.n_splits);
        hipLaunchKernelGGL((attn_bf16_kernel<D, 1, 4, kFp8>), grid, dim3(kThreads), 0, s, a);
    } else if (a.wide_cols == 256) {
        // Shared-page kernels (the host chose the shape by the number of columns per (sequence, kv
        // head) and, where those workgroups alone would not fill the chip, a split of the context).
        // Enough columns to share every page among eight wavefronts of 32 columns:
        const int ncols = a.T_new * group;
        const unsigned blocks = (ncols + 255) / 256;
        dim3 grid(a.st.Hkv, a.B, blocks * a.n_splits);
        if (blocks == 1) {
            hipLaunchKernelGGL((attn_bf16_wide_kernel<D, 2, 8, true, kFp8>), grid, dim3(512), 0, s, a);
        } else if (a.n_splits == 1 && blocks >= 4) {
            // four or more column blocks: workgroups of two blocks each, a long one and a short one, all
            // about the same length, the workgroups of a (sequence, kv head) side by side on one XCD (see
            // the kernel).  Llama-2-13B shape, the last rows of a 2048-token context: 1024 rows 800 -> 740 us,
            // 1280 rows 938 -> 878 us, 1792 rows 1088 -> 1014 us, all 2048 rows 1124 -> 1030 us; three blocks
            // lose (768 rows 679 -> 705 us) and keep the grid below.
            a.col_blocks = (int)blocks;
            a.col_paired = 1;
            const unsigned rounds = ((unsigned)a.B * a.st.Hkv + 7) / 8;
            hipLaunchKernelGGL((attn_bf16_wide_kernel<D, 2, 8, false, kFp8>), dim3(8 * rounds * ((blocks + 1) / 2)), dim3(512), 0, s, a);
        } else if (a.n_splits == 1 && blocks == 2) {
            // two column blocks walk the same pages: side by side on one XCD (see the kernel).  Measured on the
            // Llama-2-13B shape: 512 rows 496 -> 476 us.  With more blocks the side-by-side order costs more at the
            // launch's end, where long blocks start late, than the shared pages save (1024 rows 822 -> 854 us,
            // 2048 rows 1144 -> 1295 us), so those keep the grid that starts the longest blocks first.
            a.col_blocks = (int)blocks;
            const unsigned rounds = ((unsigned)a.B * a.st.Hkv + 7) / 8;
            hipLaunchKernelGGL((attn_bf16_wide_kernel<D, 2, 8, false, kFp8>), dim3(8 * rounds * blocks), dim3(512), 0, s, a);
        } else {
            hipLaunchKernelGGL((attn_bf16_wide_kernel<D, 2, 8, false, kFp8>), grid, dim3(512), 0, s, a);
        }
    } else if (a.wide_cols == 128) {
        // 65 to 128 columns: eight wavefronts of 16 columns, so that 128 columns share one pass over the pages.
        dim3 grid(a.st.Hkv, a.B, a.n_splits);
        hipLaunchKernelGGL((attn_bf16_wide_kernel<D, 1, 8, true, kFp8>), grid, dim3(512), 0, s, a);
    } else if (a.wide_cols == 64) {
        // 64 columns: 16 per wavefront, four wavefronts; small enough in registers for several
        // workgroups per compute unit to hide each other's softmax arithmetic.
        dim3 grid(a.st.Hkv, a.B, a.n_splits);
        hipLaunchKernelGGL((attn_bf16_wide_kernel<D, 1, 4, true, kFp8>), grid, dim3(256), 0, s, a);
    } else {
        const int cgroups = (a.T_new * group + 63) / 64;
        dim3 grid(a.st.Hkv, a.B, a.n_splits * cgroups);
        hipLaunchKernelGGL((attn_bf16_kernel<D, 4, 2, kFp8>), grid, dim3(kThreads), 0, s, a);
    }
    if (hipError_t e = hipGetLastError()) return (int)e;
    return 0;
}

}  // namespace

int launch_attention(const AttnArgs& a, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (a.st.dtype == 0) {
        dim3 grid(a.st.Hq, a.T_new, a.B);
        hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(64), 0, s, a);
        return (int)hipGetLastError();
    }
    if (a.st.dtype == 2) return a.st.head_dim == 128 ? launch_bf16<128, true>(a, s) : launch_bf16<64, true>(a, s);
    return a.st.head_dim == 128 ? launch_bf16<128, false>(a, s) : launch_bf16<64, false>(a, s);
}

const char* hip_error_string(int err) { return hipGetErrorString(static_cast<hipError_t>(err)); }

}  // namespace kvs
