// Decode attention over the slot-indexed, paged KV store with the context shared out by tokens
// (gfx950, bf16 and fp8 stores, one length per sequence).
//
// The operation is the ordinary decode-step attention of the host model after the sharing
// strategy has redirected a layer to its donor's cache (paper Sec. 3.2); the slot is resolved on
// the device as slot_of_layer[share_map[layer]].  What is particular to this kernel is how the
// keys and values of a launch are shared out among its workgroups: not by (sequence, kv head) or
// by a fixed number of splits per sequence, but by tokens.  The pages of all (kv head, sequence)
// segments form one line (kvs_flat_plan.h), the grid's workgroups take equal shares of it whatever
// the lengths are, and a share may begin in the middle of one sequence, hold several whole ones and
// end in the middle of another.  A batch of very unequal lengths, one long sequence among short
// ones, or a store far below its capacity therefore keeps every compute unit streaming the same
// number of bytes.
//
// A workgroup walks its share octet by octet (eight pages, a pair per wavefront; 16 KiB are in
// flight per wavefront, one to four octets by page size) and keeps one online-softmax state per wavefront, as the split kernel in
// kvs_attention.hip does.  Where the line passes from one segment to the next, the four states are
// merged through LDS and the segment is finished: written out normalised when the whole segment
// lay inside this share, else published as a partial state.  A workgroup publishes at most two
// partial states (its first and its last segment); at its end it bumps the arrival counters of
// those segments, and whoever arrives last at a segment merges its parts in a fixed order.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kvs_attn_tiles.h"
#include "kvs_device.h"
#include "kvs_flat_plan.h"
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kLargeLaunchOctets = 24;     // octets per launched workgroup from which a launch counts as large
static_assert(kOctetPages == 2 * kWaves, "an octet is one pair of pages per wavefront");

// A page through a buffer descriptor of `bytes` bytes (the page's size, or 0 for a page that does
// not exist: every load is then out of range, returns zeros and sends nothing to memory).  The load
// instructions are issued either way, which keeps the number of loads per step fixed.  Streamed
// past the caches like load_page.
template <typename Regs>
__device__ __forceinline__ void load_page_checked(Regs& r, const void* page, unsigned bytes, int lane)
{
    constexpr int n = sizeof(r.k) / sizeof(r.k[0]);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(page), 0, (int)bytes, 0x00020000);
#pragma unroll
    for (int s = 0; s < n; ++s) r.k[s] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16 + s * 1024, 0, 2);
#pragma unroll
    for (int s = 0; s < n; ++s) r.v[s] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16 + (n + s) * 1024, 0, 2);
}

// A place on the line of octets: kv head, sequence, octet inside the sequence (of `octs`).
struct Cursor {
    int g, b, oi, octs;
};

// A partial state this workgroup published: segment index (kv head * B + sequence), how many
// workgroups hold a part of the segment and which is the first of them.
struct Published {
    int seg, parts, first_wg, b, g;
};

// kDepth: octets each wavefront keeps in flight.  Every step issues the same number of load
// instructions whether its pages exist or not (a page nobody consumes is fetched from the pool's
// first page, which stays in the caches), and no load sits inside a branch: only then does the
// compiler know how many loads are younger than the ones a step waits for, and waits for exactly
// those instead of draining everything in flight.
template <int D, bool kFp8, int kDepth>
__global__ __launch_bounds__(kThreads) void attn_decode_flat_kernel(AttnArgs a)
{
    constexpr int KS = D / 32;   // k-steps of the score MFMA = 1-KiB chunks per bf16 page
    constexpr int DT = D / 16;   // 16-channel tiles of the output
    using Raw = std::conditional_t<kFp8, PageRegs8<D>, PageRegs<D>>;    // a page as it sits in the store
    const StoreView& st = a.st;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int quad = lane >> 4, col = lane & 15;
    const int wg = blockIdx.x, n_launched = gridDim.x;
    const int B = a.B, Hkv = st.Hkv, group = st.Hq / st.Hkv;
    const int max_pages = st.max_blocks_per_seq;
    const int cap = max_pages * kPageTokens;
    const bool carries_new = a.k_new != nullptr;
    const void* pool = st.pool;

    // Until the lengths are known the share is taken for what it would be if every sequence were
    // full, and the page-table entries of this wavefront's first two pairs are fetched on that
    // guess in the same round trip as the lengths (right exactly when the store is full).
    const int full_octs = (max_pages + kOctetPages - 1) / kOctetPages;
    // How many of the launched workgroups stream.  A large launch over bf16 pages of 128 channels
    // takes three quarters of them: one workgroup per compute unit asks for more than the memory
    // delivers, the XCDs are then served unequally (their workgroups finish up to 10 us apart on
    // 4 x 32k tokens) and the launch waits for the slowest; with 24 instead of 32 workgroups per XCD
    // all of them stream at the same rate (4 x 32k tokens 84.5 -> 83.1 us, 32 ragged sequences 98.0 ->
    // 95.6 us).  Not where the shares are whole segments (nothing is published or merged then, which
    // is worth more: 8 x 4096 tokens, 32 kv heads 82.7 against 83.5 us), not for small launches
    // (4 x 16k tokens 45.3 against 45.8 us) and not for fp8 pages, whose widening needs every compute unit.
    auto streaming_workgroups = [&](int total_octs, int seg_octs) {    // seg_octs: every segment's length, 0 if they differ
        if (kFp8 || D != 128 || n_launched < 64 || total_octs < kLargeLaunchOctets * n_launched) return n_launched;
        if (seg_octs > 0 && total_octs % n_launched == 0 && (total_octs / n_launched) % seg_octs == 0) return n_launched;
        const int n = (n_launched - n_launched / 4) & ~7;
        return n >= Hkv ? n : n_launched;
    };
    const int n_guess = streaming_workgroups(Hkv * B * full_octs, full_octs);
    const FlatShare guess = wg < n_guess ? flat_share(wg, n_guess, Hkv * B * full_octs) : FlatShare{0, 0};
    int guess_b[2], guess_page[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int in_head = (guess.lo + j) % (B * full_octs);
        guess_b[j] = in_head / full_octs;
        guess_page[j] = (in_head % full_octs) * kOctetPages + 2 * wave;
    }

    // Start-up look-ups in one round trip: the lengths (lane = sequence), and a gathered load in
    // which lane 1 fetches the layer's donor, lanes 2..5 the guessed page-table entries and lanes
    // 8..63 the slots of layers 0..55.  Only a donor beyond layer 55 costs a dependent look-up.
    const int32_t* look = nullptr;
    if (lane == 1) {
        look = st.share_map + st.layer;
    } else if (lane >= 2 && lane < 6) {
        const int j = (lane - 2) >> 1;
        int pg = (j ? guess_page[1] : guess_page[0]) + ((lane - 2) & 1);
        pg = pg < max_pages ? pg : max_pages - 1;
        if (st.block_table) look = st.block_table + (size_t)(j ? guess_b[1] : guess_b[0]) * max_pages + pg;
    } else if (lane >= 8 && lane - 8 < st.L) {
        look = st.slot_of_layer + (lane - 8);
    }
    const int len_raw_lane = lane < B ? a.lens[lane] : 0;
    const int looked = look ? *look : 0;

    // the strategy's substitution: this layer reads the slot of its donor (itself if none)
    const int donor_raw = __builtin_amdgcn_readlane(looked, 1);
    const int donor = donor_raw < 0 ? 0 : (donor_raw >= st.L ? st.L - 1 : donor_raw);
    const int slot_raw = donor < 56 ? __builtin_amdgcn_readlane(looked, 8 + donor) : st.slot_of_layer[donor];
    const int slot = slot_raw < 0 ? 0 : (slot_raw >= st.n_slots ? st.n_slots - 1 : slot_raw);

    // Keys each sequence holds in its pages (a step that carries its own new token: the tokens
    // before it), in pages and in octets, and the running sum of the octets over the sequences.
    int n0_lane = len_raw_lane + a.lens_bias - (carries_new ? 1 : 0);
    n0_lane = n0_lane < 0 ? 0 : (n0_lane > cap ? cap : n0_lane);
    if (lane >= B) n0_lane = 0;
    const int pages_lane = (n0_lane + kPageTokens - 1) / kPageTokens;
    const int octs_lane = (pages_lane + kOctetPages - 1) / kOctetPages;
    int incl = octs_lane;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    const int head_octs = __builtin_amdgcn_readlane(incl, 63);       // octets of one kv head
    const int total = head_octs * Hkv;
    const int octs_first = __builtin_amdgcn_readfirstlane(octs_lane);
    const int n_wg = streaming_workgroups(total, __all(lane >= B || octs_lane == octs_first) ? octs_first : 0);
    const FlatPlan plan(n_wg, total);
    const FlatShare mine = wg < n_wg ? plan.share(wg) : FlatShare{0, 0};

    auto advance = [&](Cursor& c) {                                  // only called while an octet follows on the line
        if (++c.oi < c.octs) return;
        c.oi = 0;
        do {
            if (++c.b == B) {
                c.b = 0;
                ++c.g;
            }
            c.octs = __builtin_amdgcn_readlane(octs_lane, c.b);
        } while (c.octs == 0);
    };
    // The pair of pages this wavefront takes of the octet at c (live: the octet belongs to this
    // workgroup's share).  Page-table look-ups are scalar loads and may sit in branches; the page
    // loads themselves are unconditional: a page that does not exist is read through an empty
    // buffer descriptor, whose loads return zeros without touching memory.
    constexpr unsigned kPageBytes = 2u * kPageTokens * D * (kFp8 ? 1u : 2u);       // keys and values of one page
    const size_t elem_bytes = kFp8 ? 1 : 2;
    auto fetch = [&](const Cursor& c, bool live, Raw& ra, Raw& rb, bool guessed, int j) {
        const int pa = c.oi * kOctetPages + 2 * wave;
        const int pages = live ? __builtin_amdgcn_readlane(pages_lane, c.b) : 0;
        const bool known = guessed && st.block_table;            // the entry came with the start-up look-ups
        size_t off_a = 0, off_b = 0;
        if (pa < pages) {
            int blk = known ? __builtin_amdgcn_readlane(looked, 2 + 2 * j) : safe_block_of_uniform(st, c.b, pa);
            blk = blk < 0 ? 0 : (blk >= st.num_blocks ? st.num_blocks - 1 : blk);
            off_a = page_offset(st, slot, blk, c.g);
        }
        if (pa + 1 < pages) {
            int blk = known ? __builtin_amdgcn_readlane(looked, 3 + 2 * j) : safe_block_of_uniform(st, c.b, pa + 1);
            blk = blk < 0 ? 0 : (blk >= st.num_blocks ? st.num_blocks - 1 : blk);
            off_b = page_offset(st, slot, blk, c.g);
        }
        load_page_checked(ra, static_cast<const char*>(pool) + off_a * elem_bytes, pa < pages ? kPageBytes : 0u, lane);
        load_page_checked(rb, static_cast<const char*>(pool) + off_b * elem_bytes, pa + 1 < pages ? kPageBytes : 0u, lane);
    };

    const unsigned short* qbase = static_cast<const unsigned short*>(a.q);
    const float scale_log2 = 1.44269504088896340736f * (D == 128 ? 0.08838834764831845f : 0.125f);
    // the new row as the store will hold it: as given (bf16 store), rounded to E4M3 (fp8 store)
    auto as_stored = [](unsigned short h) -> float {
        const unsigned w = kFp8 ? e4m3_to_bf16(bf16_to_e4m3(h)) : h;
        return __uint_as_float(w << 16);
    };
    // This step's own token of (sequence b, kv head g) into its place in the store, for the steps
    // to come (this launch masks that position).
    auto store_new_row = [&](int b, int g, int new_pos) {
        const unsigned short* k_row = static_cast<const unsigned short*>(a.k_new) + ((size_t)b * Hkv + g) * D;
        const unsigned short* v_row = static_cast<const unsigned short*>(a.v_new) + ((size_t)b * Hkv + g) * D;
        const int blk = block_of(st, b, new_pos / kPageTokens);
        if (blk < 0 || blk >= st.num_blocks) return;
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
    };

    Published pub0 = {0, 0, 0, 0, 0}, pub1 = {0, 0, 0, 0, 0};
    if (mine.count > 0) {
        // where the share begins: kv head, the first sequence that ends behind that octet, the octet in it
        Cursor cur;
        cur.g = mine.lo / head_octs;
        const int within = mine.lo - cur.g * head_octs;
        cur.b = __builtin_popcountll(__ballot(incl <= within));
        cur.octs = __builtin_amdgcn_readlane(octs_lane, cur.b);
        cur.oi = within - (__builtin_amdgcn_readlane(incl, cur.b) - cur.octs);
        Cursor ahead = cur;                                          // the octet whose pages are fetched next

        // state of the segment being consumed
        int seg_n = 0, seg_len_raw = 0;
        bf16x8 qf[1][KS];
        float m[1], l[1];
        floatx4 o[1][DT];
        auto begin_segment = [&](const Cursor& c, bool settle) {
            seg_n = __builtin_amdgcn_readlane(n0_lane, c.b);
            seg_len_raw = __builtin_amdgcn_readlane(len_raw_lane, c.b);
            const bool col_ok = col < group;
            const size_t q_off = ((size_t)c.b * st.Hq + c.g * group + (col_ok ? col : 0)) * D;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                uint4 w = make_uint4(0, 0, 0, 0);
                if (col_ok) w = *reinterpret_cast<const uint4*>(qbase + q_off + s * 32 + quad * 8);
                qf[0][s] = __builtin_bit_cast(bf16x8, w);
            }
            m[0] = -INFINITY;
            l[0] = 0.f;
#pragma unroll
            for (int c2 = 0; c2 < DT; ++c2) o[0][c2] = floatx4{0.f, 0.f, 0.f, 0.f};
            // The queries are waited for here, inside the branch that loads them: left pending, they
            // would be the youngest loads on this path, and where it rejoins the loop the compiler
            // would make every step wait for "them", i.e. for everything in flight.  (The share's
            // first segment settles them itself, behind its first page loads.)
            if (settle) {
#pragma unroll
                for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qf[0][s]));
            }
        };

        __shared__ float lds_new_score[16];           // log2-domain score of the step's own token, per column
        __shared__ float lds_o[kWaves][16][D + 4];
        __shared__ float lds_m[kWaves][16];
        __shared__ float lds_l[kWaves][16];
        bool first_segment = true;
        // The segment (kv head g, sequence b) ends here for this workgroup: merge the four wavefront
        // states and either write the finished rows or publish the part.
        auto finish_segment = [&](int g, int b) {
            const int octs = __builtin_amdgcn_readlane(octs_lane, b);
            const int seg_lo = g * head_octs + __builtin_amdgcn_readlane(incl, b) - octs;
            const int first_wg = plan.owner(seg_lo);
            const int parts = plan.owner(seg_lo + octs - 1) - first_wg + 1;
            // A step that carries its own new token: the workgroup that holds the segment's first
            // octet adds it as one more state (score, weight 1, value row v_new) and stores the row.
            const int new_pos = seg_len_raw - 1;
            const bool adds_new = carries_new && new_pos >= 0 && new_pos < cap && first_wg == wg;
            const unsigned short* v_row = static_cast<const unsigned short*>(a.v_new) + ((size_t)b * Hkv + g) * D;
            __syncthreads();                          // the LDS arrays are free again (readers of the segment before)
            if (adds_new) {
                store_new_row(b, g, new_pos);
                const unsigned short* k_row = static_cast<const unsigned short*>(a.k_new) + ((size_t)b * Hkv + g) * D;
                // q . k_new for the 16 columns: a wavefront takes four columns, sixteen lanes each
                constexpr int CH = D / 16;
                const int cc = wave * 4 + quad, part = col;
                float dot = 0.f;
                if (cc < group) {
                    const unsigned short* qr = qbase + ((size_t)b * st.Hq + g * group + cc) * D + part * CH;
#pragma unroll
                    for (int e = 0; e < CH; ++e)
                        dot += __uint_as_float((unsigned)qr[e] << 16) * as_stored(k_row[part * CH + e]);
                }
#pragma unroll
                for (int o_ = 8; o_ > 0; o_ >>= 1) dot += __shfl_xor(dot, o_);
                if (part == 0) lds_new_score[cc] = cc < group ? dot * scale_log2 : -INFINITY;
            }
            const float lsum = column_sum(l[0]);
            if (quad == 0) {
                lds_m[wave][col] = m[0];
                lds_l[wave][col] = lsum;
            }
#pragma unroll
            for (int c2 = 0; c2 < DT; ++c2)
                *reinterpret_cast<floatx4*>(&lds_o[wave][col][c2 * 16 + quad * 4]) = o[0][c2];
            __syncthreads();
            for (int idx = threadIdx.x; idx < 16 * (D / 4); idx += kThreads) {
                const int cc = idx / (D / 4);
                const int d4 = (idx % (D / 4)) * 4;
                if (cc >= group) continue;
                float mw[kWaves], M = -INFINITY;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    mw[w] = lds_m[w][cc];
                    M = fmaxf(M, mw[w]);
                }
                const float m_new_tok = adds_new ? lds_new_score[cc] : -INFINITY;
                M = fmaxf(M, m_new_tok);
                const float M_use = M == -INFINITY ? 0.f : M;
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
                float lt = 0.f;
                if (adds_new) {                                   // weight 2^(score - M), value row v_new
                    const float wgt = __builtin_amdgcn_exp2f(m_new_tok - M_use);
                    acc = wgt * floatx4{as_stored(v_row[d4]), as_stored(v_row[d4 + 1]), as_stored(v_row[d4 + 2]),
                                        as_stored(v_row[d4 + 3])};
                    lt = wgt;
                }
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const float wgt = __builtin_amdgcn_exp2f(mw[w] - M_use);
                    acc += wgt * *reinterpret_cast<const floatx4*>(&lds_o[w][cc][d4]);
                    lt += wgt * lds_l[w][cc];
                }
                if (parts <= 1) {
                    const float inv = lt > 0.f ? 1.f / lt : 0.f;
                    const size_t row = (size_t)b * st.Hq + g * group + cc;
                    *reinterpret_cast<floatx4*>(a.out + row * D + d4) = acc * inv;
                } else {
                    // one record per (workgroup + segment index, head of the group): the records of a
                    // segment's parts are consecutive
                    const size_t rec = ((size_t)wg + (size_t)g * B + b) * group + cc;
                    float* part = a.partials + rec * (size_t)(D + 2);
                    publish_pair(part + d4, acc[0], acc[1]);
                    publish_pair(part + d4 + 2, acc[2], acc[3]);
                    if (d4 == 0) publish_pair(part + D, M, lt);
                }
            }
            if (parts > 1) {
                const Published p = {g * B + b, parts, first_wg, b, g};
                if (first_segment) pub0 = p; else pub1 = p;
            }
            first_segment = false;
        };

        // kDepth octets in flight per wavefront; the steps are rounded up to whole turns of the ring,
        // the ones past the share fetch and consume nothing real
        // The first segment's queries are requested first and waited for behind the first page loads:
        // waited for where they are requested, their round trip stood before the first page load.
        Raw ring[kDepth][2];
        begin_segment(cur, false);
#pragma unroll
        for (int j = 0; j < kDepth; ++j) {
            const bool live = j < mine.count;
            if (j > 0 && live) advance(ahead);
            const bool hit = j < 2 && live && ahead.b == guess_b[j < 2 ? j : 0] &&
                             ahead.oi * kOctetPages + 2 * wave == guess_page[j < 2 ? j : 0];
            fetch(ahead, live, ring[j][0], ring[j][1], hit, j < 2 ? j : 0);
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qf[0][s]));
        int seg_g = cur.g, seg_b = cur.b;
        for (int o0 = 0; o0 < mine.count; o0 += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) {
                const int oo = o0 + j;
                const bool live = oo < mine.count;
                if (live && oo > 0 && cur.oi == 0) {         // the line has passed into the next segment
                    finish_segment(seg_g, seg_b);
                    begin_segment(cur, true);
                    seg_g = cur.g;
                    seg_b = cur.b;
                }
                const int pa = cur.oi * kOctetPages + 2 * wave;
                const int pages = live ? __builtin_amdgcn_readlane(pages_lane, cur.b) : 0;
                if (pa < pages) {
                    const bool have_b = pa + 1 < pages;
                    const int n_col[1] = {seg_n};
                    if constexpr (kFp8) {
                        PageRegs<D> wa, wb;                      // widened to bf16 operands
                        widen<D>(ring[j][0], wa);
                        widen<D>(ring[j][1], wb);                // an absent page is zeroed by consume_pair
                        consume_pair<D, 1>(wa, wb, have_b, pa * kPageTokens, (pa + 1) * kPageTokens, seg_n, seg_n, n_col, qf,
                                           m, l, o, quad, scale_log2);
                    } else {
                        consume_pair<D, 1>(ring[j][0], ring[j][1], have_b, pa * kPageTokens, (pa + 1) * kPageTokens, seg_n,
                                           seg_n, n_col, qf, m, l, o, quad, scale_log2);
                    }
                }
                const bool more = oo + kDepth < mine.count;
                if (more) advance(ahead);
                fetch(ahead, more, ring[j][0], ring[j][1], false, 0);
                if (oo + 1 < mine.count) advance(cur);
            }
        }
        finish_segment(seg_g, seg_b);
    }

    // Sequences without any key in their pages take no octet of the line: workgroup g writes their
    // rows for kv head g (the step's own token alone, or zeros).
    if (wg < Hkv) {
        const int g = wg;
        for (int b = 0; b < B; ++b) {
            if (__builtin_amdgcn_readlane(octs_lane, b) != 0) continue;
            const int new_pos = __builtin_amdgcn_readlane(len_raw_lane, b) - 1;
            const bool has_new = carries_new && new_pos >= 0 && new_pos < cap;
            const unsigned short* v_row = static_cast<const unsigned short*>(a.v_new) + ((size_t)b * Hkv + g) * D;
            for (int idx = threadIdx.x; idx < group * D; idx += kThreads) {
                const size_t row = (size_t)b * st.Hq + g * group + idx / D;
                a.out[row * D + idx % D] = has_new ? as_stored(v_row[idx % D]) : 0.f;
            }
            if (has_new) store_new_row(b, g, new_pos);
        }
    }

    // Arrival at the segments this workgroup holds a part of (at most its first and its last): the
    // workgroup that arrives last at a segment finds every other part published and merges them.
    // Nobody waits for anybody.
    if (pub0.parts <= 1 && pub1.parts <= 1) return;
    __shared__ int s_is_last[2];
    // vmcnt(0): every device-scope store this wavefront issued has been acknowledged
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (threadIdx.x < 2) {
        const Published& p = threadIdx.x ? pub1 : pub0;
        int last = 0;
        if (p.parts > 1) {
            int* counter = a.counters + p.seg;
            last = atomicAdd(counter, 1) == p.parts - 1;
            if (last) atomicExch(counter, 0);                    // leave the counter ready for the next call
        }
        s_is_last[threadIdx.x] = last;
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (!s_is_last[k]) continue;
        const Published& p = k ? pub1 : pub0;
        // records (first_wg + seg + part) * group + head, one workgroup apart per part
        const size_t rec_first = ((size_t)p.first_wg + p.seg) * group - ((size_t)p.b * st.Hq + (size_t)p.g * group);
        merge_splits<D>(a, p.b, p.g, 0, 16, group, group, p.parts, kThreads, 1, group, rec_first);
    }
}

}  // namespace

size_t decode_flat_partial_floats(int n_wg, int B, int Hq, int Hkv, int head_dim)
{
    return ((size_t)n_wg + (size_t)B * Hkv) * (size_t)(Hq / Hkv) * (size_t)(head_dim + 2);
}

int launch_decode_flat(const AttnArgs& a, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(a.n_items), block(kThreads);
    // 16 KiB in flight per wavefront (64 KiB per compute unit) in every variant: one pair of bf16
    // pages at head_dim 128, two pairs of fp8 pages or of bf16 pages at head_dim 64, four of fp8 pages
    // at head_dim 64.  Measured on 4 x 32k tokens, 8 kv heads: twice that changes nothing for bf16
    // (85.4 against 85.6 us) and costs fp8 slots 1.7 us (47.4 against 49.1 us: more in flight only
    // lengthens the queues of the memory system), half of it costs fp8 slots 9 us.
    if (a.st.dtype == 2) {
        if (a.st.head_dim == 128) hipLaunchKernelGGL((attn_decode_flat_kernel<128, true, 2>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((attn_decode_flat_kernel<64, true, 4>), grid, block, 0, s, a);
    } else {
        if (a.st.head_dim == 128) hipLaunchKernelGGL((attn_decode_flat_kernel<128, false, 1>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((attn_decode_flat_kernel<64, false, 2>), grid, block, 0, s, a);
    }
    return (int)hipGetLastError();
}

}  // namespace kvs
