// Host side of libkvs: argument checks, the strategy-search walk, launch geometry.
// Everything that can be decided without the GPU is decided here, before any HIP call.
#include "../../include/kvs.h"
#include "../../include/kvs_testing.h"
#include "kvs_flat_plan.h"
#include "kvs_internal.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <numeric>
#include <string>
#include <vector>

namespace {

thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

std::atomic<int> g_split_tokens{0};
std::atomic<int> g_decode_workgroups{0};

// Workgroups the decode grid should at least reach: one per compute unit.  Measured on
// MI355X, four wavefronts per compute unit with three pages in flight each already saturate
// HBM, and every further workgroup pays its own start-up (map and page-table look-ups, query
// load) and merge, so the context is split no finer than needed to cover the 256 units.
constexpr int kTargetWorkgroups = 256;
constexpr int kMinPagesPerSplit = 4;   // one page per wavefront of the workgroup

int check_desc(const kvs_desc* d)
{
    if (!d) return fail(KVS_ERR_INVALID_ARG, "descriptor is NULL");
    if (d->L <= 0 || d->n_slots <= 0 || d->n_slots > d->L)
        return fail(KVS_ERR_INVALID_ARG, "need 0 < n_slots <= L (L=%d, n_slots=%d)", d->L, d->n_slots);
    if (d->Hq <= 0 || d->Hkv <= 0 || d->Hq % d->Hkv != 0)
        return fail(KVS_ERR_INVALID_ARG, "Hq=%d must be a positive multiple of Hkv=%d", d->Hq, d->Hkv);
    if (d->block_tokens != KVS_BLOCK_TOKENS)
        return fail(KVS_ERR_UNSUPPORTED, "block_tokens must be %d (got %d)", KVS_BLOCK_TOKENS, d->block_tokens);
    if (d->num_blocks <= 0 || d->max_blocks_per_seq <= 0)
        return fail(KVS_ERR_INVALID_ARG, "num_blocks and max_blocks_per_seq must be positive");
    if (d->max_blocks_per_seq > (1 << 26))
        return fail(KVS_ERR_CAPACITY, "max_blocks_per_seq too large");
    if (d->dtype == KVS_BF16 || d->dtype == KVS_FP8) {
        if (d->head_dim != 128 && d->head_dim != 64)
            return fail(KVS_ERR_UNSUPPORTED, "bf16 and fp8 stores support head_dim 64 or 128 (got %d)", d->head_dim);
        if (d->Hq / d->Hkv > 16)
            return fail(KVS_ERR_UNSUPPORTED, "bf16 and fp8 stores support at most 16 query heads per kv head");
    } else if (d->dtype == KVS_F32) {
        if (d->head_dim <= 0 || d->head_dim % 64 != 0 || d->head_dim > 256)
            return fail(KVS_ERR_UNSUPPORTED, "fp32 store supports head_dim 64, 128, 192 or 256 (got %d)", d->head_dim);
    } else {
        return fail(KVS_ERR_UNSUPPORTED, "unknown dtype %d", d->dtype);
    }
    return KVS_OK;
}

size_t elem_bytes(int dtype) { return dtype == KVS_BF16 ? 2 : (dtype == KVS_FP8 ? 1 : 4); }

int check_map(const int32_t* m, int L)
{
    if (!m || L <= 0) return fail(KVS_ERR_INVALID_ARG, "share map is NULL or L <= 0");
    for (int l = 0; l < L; ++l) {
        if (m[l] < 0 || m[l] > l)
            return fail(KVS_ERR_BAD_MAP, "share_map[%d]=%d: a donor must be the layer itself or one nearer the input", l, m[l]);
        if (m[m[l]] != m[l])
            return fail(KVS_ERR_BAD_MAP, "share_map[%d]=%d is itself a recipient (chains are not allowed)", l, m[l]);
    }
    return KVS_OK;
}

void number_slots(const int32_t* m, int L, int32_t* slot, int32_t* n_slots)
{
    int32_t next = 0;
    for (int l = 0; l < L; ++l)
        if (m[l] == l) slot[l] = next++;
    for (int l = 0; l < L; ++l)
        if (m[l] != l) slot[l] = slot[m[l]];
    *n_slots = next;
}

int check_store(const kvs_store* s, int layer)
{
    if (!s) return fail(KVS_ERR_INVALID_ARG, "store is NULL");
    if (int rc = check_desc(&s->desc)) return rc;
    if (!s->pool || !s->share_map || !s->slot_of_layer || !s->host_share_map || !s->host_slot_of_layer)
        return fail(KVS_ERR_INVALID_ARG, "store has a NULL pool, map or host mirror");
    if (layer < 0 || layer >= s->desc.L)
        return fail(KVS_ERR_INVALID_ARG, "layer %d out of range [0, %d)", layer, s->desc.L);
    if (int rc = check_map(s->host_share_map, s->desc.L)) return rc;
    for (int l = 0; l < s->desc.L; ++l) {
        const int32_t sl = s->host_slot_of_layer[l];
        if (sl < 0 || sl >= s->desc.n_slots)
            return fail(KVS_ERR_BAD_MAP, "slot_of_layer[%d]=%d outside [0, %d)", l, sl, s->desc.n_slots);
        if (sl != s->host_slot_of_layer[s->host_share_map[l]])
            return fail(KVS_ERR_BAD_MAP, "layer %d and its donor %d disagree on the slot", l, s->host_share_map[l]);
    }
    return KVS_OK;
}

kvs::StoreView view_of(const kvs_store* s, int layer)
{
    kvs::StoreView v;
    v.pool = s->pool;
    v.share_map = s->share_map;
    v.slot_of_layer = s->slot_of_layer;
    v.block_table = s->block_table;
    v.layer = layer;
    v.L = s->desc.L;
    v.n_slots = s->desc.n_slots;
    v.Hq = s->desc.Hq;
    v.Hkv = s->desc.Hkv;
    v.head_dim = s->desc.head_dim;
    v.dtype = s->desc.dtype;
    v.num_blocks = s->desc.num_blocks;
    v.max_blocks_per_seq = s->desc.max_blocks_per_seq;
    return v;
}

// Query columns (row, head-in-group pairs) one workgroup of the bf16 kernel covers.
int columns_per_workgroup(int T_new) { return T_new > 1 ? 64 : 16; }

struct Split { int pages_per_split, n_splits, n_col_groups, wide_cols, adaptive, want_splits, n_items; };

// A decode launch sizes the page range of a split on the device, by the lengths it finds there
// (the host never sees them).  Where the grid keeps one split index per (sequence, split) -- per-
// head lengths -- it carries this many times the indices a batch of full sequences needs.  More
// than 1 would let a sequence longer than the batch's mean take more workgroups than a shorter
// one; measured, the workgroups that only leave cost more than that gains.
constexpr int kSplitHeadroom = 1;

Split choose_split(const kvs_desc* d, int B, int T_new, bool per_head_lens = false)
{
    Split s;
    const int max_pages = d->max_blocks_per_seq;
    s.wide_cols = 0;
    s.adaptive = 0;
    s.want_splits = 1;
    s.n_items = 0;
    if (d->dtype == KVS_F32) {           // the fp32 kernel walks the whole context in one wave
        s.pages_per_split = max_pages;
        s.n_splits = 1;
        s.n_col_groups = 1;
        return s;
    }
    const int group = d->Hq / d->Hkv;
    const int ncols = T_new * group;
    s.n_col_groups = (ncols + columns_per_workgroup(T_new) - 1) / columns_per_workgroup(T_new);
    // Prefill with at least 64 query columns per (sequence, kv head) takes a shared-page kernel: 256
    // columns per workgroup (8 wavefronts x 32), 128 (8 x 16) or 64 (4 x 16).  The smaller two run
    // several workgroups per compute unit, hence the larger target.
    long items = (long)B * d->Hkv * s.n_col_groups, target = kTargetWorkgroups;
    if (T_new > 1 && ncols >= 64) {
        s.wide_cols = ncols > 128 ? 256 : (ncols > 64 ? 128 : 64);
        items = (long)B * d->Hkv * ((ncols + s.wide_cols - 1) / s.wide_cols);
        target = s.wide_cols == 256 ? kTargetWorkgroups : 2 * kTargetWorkgroups;
    }
    int pps;
    const int forced = g_split_tokens.load();
    const long most = max_pages / 16 > 0 ? max_pages / 16 : 1;               // no split below 16 pages
    long want = 1;
    if (forced > 0) {
        pps = forced / KVS_BLOCK_TOKENS;
    } else {
        want = (target + items - 1) / items;                                 // splits wanted
        want = std::max(1L, std::min(want, most));
        pps = (int)((max_pages + want - 1) / want);
        pps = (pps + 3) / 4 * 4;
    }
    pps = std::max(kMinPagesPerSplit, std::min(pps, (max_pages + 3) / 4 * 4));
    s.pages_per_split = pps;
    s.n_splits = (max_pages + pps - 1) / pps;
    // (the kernels add up all lengths in pages, or in groups of eight pages, as 32-bit integers)
    if (T_new == 1 && forced == 0 && !per_head_lens && B <= 64 && (size_t)B * d->Hkv <= kvs::kMaxCounters &&
        items * max_pages < (1L << 28)) {
        // One length per sequence, at most 64 sequences: the launch's pages are shared out by tokens
        // among a fixed number of workgroups, whatever the lengths turn out to be on the device (one
        // workgroup per compute unit; at least one per kv head, which the rows of empty sequences need).
        const long octets = (long)B * d->Hkv * ((max_pages + 7) / 8);
        s.adaptive = 3;
        const int forced_grid = g_decode_workgroups.load();
        s.n_items = (int)std::max<long>(std::min<long>(forced_grid > 0 ? forced_grid : kTargetWorkgroups, octets), d->Hkv);
        return s;
    }
    // Per-head lengths, or more than 64 sequences: the split kernel, which sizes its splits on the
    // device while the (sequence, kv head) pairs are few.  (With more than two workgroups per compute
    // unit the order in which they are handed out evens out unequal lengths by itself, and every
    // workgroup would scan that many more lengths.)
    if (T_new == 1 && forced == 0 && items <= 2 * kTargetWorkgroups && items * max_pages < (1L << 30)) {
        const int spare = (int)std::min(most, kSplitHeadroom * want);
        if (spare > 1) {
            s.adaptive = 1;
            s.want_splits = (int)want;
            s.n_splits = std::max(s.n_splits, spare);
        }
    }
    return s;
}

// Workspace layout: the counter region (fixed size, so that calls of any shape agree on where it
// ends), then the per-split partial states.  Counters are indexed by (sequence, kv head, column
// group) and are touched only by calls that split the context; the built-in policy splits only
// while those items are fewer than the workgroups it aims for, far below the region's capacity.
size_t counters_used(const kvs_desc* d, int B, const Split& s)
{
    if (s.n_splits <= 1 && !s.adaptive) return 0;
    return (size_t)B * d->Hkv * s.n_col_groups;
}

size_t partial_floats(const kvs_desc* d, int B, int T_new, const Split& s)
{
    if (s.adaptive == 3) return kvs::decode_flat_partial_floats(s.n_items, B, d->Hq, d->Hkv, d->head_dim);
    if (s.n_splits <= 1) return 0;
    return (size_t)B * T_new * d->Hq * s.n_splits * (size_t)(d->head_dim + 2);
}

}  // namespace

namespace kvs {
int report_error(int code, const char* message) { return fail(code, "%s", message); }
}  // namespace kvs

extern "C" {

const char* kvs_last_error(void) { return g_last_error.c_str(); }

int kvs_validate_share_map(const int32_t* share_map, int L) { return check_map(share_map, L); }

int kvs_slots_from_share_map(const int32_t* share_map, int L, int32_t* slot_of_layer, int32_t* n_slots)
{
    if (!slot_of_layer || !n_slots) return fail(KVS_ERR_INVALID_ARG, "output pointer is NULL");
    if (int rc = check_map(share_map, L)) return rc;
    number_slots(share_map, L, slot_of_layer, n_slots);
    return KVS_OK;
}

int kvs_build_share_map(const float* dist, int L, int target_shared, int order,
                        kvs_accept_fn accept, void* user,
                        int32_t* share_map, int32_t* slot_of_layer,
                        int32_t* n_slots, int32_t* n_shared)
{
    if (!dist || !share_map || !slot_of_layer || !n_slots || !n_shared)
        return fail(KVS_ERR_INVALID_ARG, "NULL argument");
    if (L <= 0 || target_shared < 0 || target_shared >= L)
        return fail(KVS_ERR_INVALID_ARG, "need L > 0 and 0 <= target_shared < L (L=%d, C=%d)", L, target_shared);
    if (order != 0 && order != 1) return fail(KVS_ERR_INVALID_ARG, "order must be 0 or 1");

    struct Pair { float d; int32_t i, j; };
    std::vector<Pair> ranking;
    ranking.reserve((size_t)L * (L - 1) / 2);
    for (int i = 0; i < L; ++i)
        for (int j = i + 1; j < L; ++j) {
            const float v = dist[(size_t)i * L + j];
            if (std::isnan(v)) return fail(KVS_ERR_INVALID_ARG, "dist[%d][%d] is NaN", i, j);
            ranking.push_back({v, i, j});
        }
    // Pairs were generated in (i, j) order, so a stable sort keeps that order among ties.
    if (order == 0)
        std::stable_sort(ranking.begin(), ranking.end(), [](const Pair& a, const Pair& b) { return a.d > b.d; });
    else
        std::stable_sort(ranking.begin(), ranking.end(), [](const Pair& a, const Pair& b) { return a.d < b.d; });

    std::vector<int32_t> map(L), candidate(L);
    std::iota(map.begin(), map.end(), 0);
    std::vector<char> donates(L, 0);
    int shared = 0;
    for (const Pair& r : ranking) {
        if (shared == target_shared) break;
        const bool receiver_free = map[r.j] == r.j && !donates[r.j];
        const bool donor_free = map[r.i] == r.i;
        if (!receiver_free || !donor_free) continue;
        candidate = map;
        candidate[r.j] = r.i;
        if (accept && !accept(candidate.data(), L, user)) continue;   // similarity at or below threshold
        map.swap(candidate);
        donates[r.i] = 1;
        ++shared;
    }
    std::copy(map.begin(), map.end(), share_map);
    number_slots(share_map, L, slot_of_layer, n_slots);
    *n_shared = shared;
    if (shared != target_shared)
        return fail(KVS_ERR_TARGET_UNREACHED, "ranking exhausted with %d of %d layers shared", shared, target_shared);
    return KVS_OK;
}

size_t kvs_store_bytes(const kvs_desc* d)
{
    if (check_desc(d) != KVS_OK) return 0;
    return (size_t)d->n_slots * d->num_blocks * d->Hkv * 2 * KVS_BLOCK_TOKENS * (size_t)d->head_dim *
           elem_bytes(d->dtype);
}

int kvs_testing_force_split_tokens(int tokens)
{
    if (tokens < 0 || tokens % 64 != 0) return fail(KVS_ERR_INVALID_ARG, "split tokens must be 0 or a multiple of 64");
    g_split_tokens.store(tokens);
    return KVS_OK;
}

int kvs_testing_set_decode_workgroups(int n)
{
    if (n < 0 || n > 65535) return fail(KVS_ERR_INVALID_ARG, "need 0 <= n <= 65535");
    g_decode_workgroups.store(n);
    return KVS_OK;
}

int kvs_testing_flat_share(int i, int n, int total, int* first, int* count)
{
    if (n <= 0 || n > 65535 || i < 0 || i >= n || total < 0 || !first || !count)
        return fail(KVS_ERR_INVALID_ARG, "need 0 <= i < n <= 65535, total >= 0");
    const kvs::FlatShare s = kvs::flat_share(i, n, total);
    *first = s.lo;
    *count = s.count;
    return KVS_OK;
}

int kvs_testing_flat_owner(int o, int n, int total)
{
    if (n <= 0 || n > 65535 || o < 0 || o >= total) return -1;
    return kvs::flat_owner(o, n, total);
}

size_t kvs_workspace_bytes(const kvs_desc* d, int B, int max_q_rows)
{
    if (check_desc(d) != KVS_OK) return 0;
    if (B <= 0 || max_q_rows <= 0) { fail(KVS_ERR_INVALID_ARG, "B and max_q_rows must be positive"); return 0; }
    // The largest need over every row count a call may bring: fewer rows can mean more context
    // splits, so the need does not grow monotonically with the rows.  Once the rows alone give
    // enough workgroups nothing is split any more (and a forced split is the same for all row
    // counts), and the need only grows with the rows from there on: the walk stops there.
    const long capacity = (long)d->max_blocks_per_seq * KVS_BLOCK_TOKENS;
    const int last = (int)std::min<long>(max_q_rows, capacity);
    const int group = d->Hq / d->Hkv;
    auto need_for = [&](int r) {
        size_t n = 0;
        for (bool per_head : {false, true}) {          // a decode call may bring either kind of lengths
            const Split s = choose_split(d, B, r, per_head);
            n = std::max(n, kvs::kCounterRegionBytes + partial_floats(d, B, r, s) * sizeof(float));
        }
        return n;
    };
    size_t need = need_for(last);
    if (g_split_tokens.load() > 0 || d->dtype == KVS_F32) return std::max(need, need_for(1));
    for (int r = 1; r < last; ++r) {
        need = std::max(need, need_for(r));
        if ((long)r * group > 128 && choose_split(d, B, r).n_splits == 1) break;
    }
    return need;
}

static int append_common(const kvs_store* store, int layer, const void* k_new, const void* v_new,
                         const int32_t* start_pos, int pos_per_head, int B, int T_new, void* stream,
                         int pos_bias = 0)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!k_new || !v_new || !start_pos) return fail(KVS_ERR_INVALID_ARG, "k_new, v_new or start_pos is NULL");
    if (B <= 0 || T_new <= 0) return fail(KVS_ERR_INVALID_ARG, "B and T_new must be positive (B=%d, T_new=%d)", B, T_new);
    if (T_new > store->desc.max_blocks_per_seq * KVS_BLOCK_TOKENS)
        return fail(KVS_ERR_CAPACITY, "T_new=%d exceeds the per-sequence capacity %d", T_new,
                    store->desc.max_blocks_per_seq * KVS_BLOCK_TOKENS);
    if (!store->block_table && (long)B * store->desc.max_blocks_per_seq > store->desc.num_blocks)
        return fail(KVS_ERR_CAPACITY, "contiguous store: B * max_blocks_per_seq exceeds num_blocks");
    if (B > 65535 || store->desc.Hkv > 65535) return fail(KVS_ERR_CAPACITY, "B and Hkv are limited to 65535");
    if (store->host_share_map[layer] != layer) return KVS_NOOP;   // the layer reads its donor's cache
    kvs::CopyArgs a;
    a.st = view_of(store, layer);
    a.k = const_cast<void*>(k_new);
    a.v = const_cast<void*>(v_new);
    a.start_pos = start_pos;
    a.pos_per_head = pos_per_head;
    a.pos_bias = pos_bias;
    a.t0 = 0;
    a.B = B;
    a.T = T_new;
    if (int e = kvs::launch_append(a, stream)) return fail(KVS_ERR_HIP, "append launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

int kvs_append_kv(const kvs_store* store, int layer, const void* k_new, const void* v_new,
                  const int32_t* start_pos, int B, int T_new, void* stream)
{
    return append_common(store, layer, k_new, v_new, start_pos, 0, B, T_new, stream);
}

int kvs_append_kv_per_head(const kvs_store* store, int layer, const void* k_new, const void* v_new,
                           const int32_t* pos, int B, int T_new, void* stream)
{
    return append_common(store, layer, k_new, v_new, pos, 1, B, T_new, stream);
}

int kvs_compact_kv(const kvs_store* store, int layer, const int32_t* keep_idx, const int32_t* keep_count,
                   int max_keep, int B, void* stream)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!keep_idx || !keep_count) return fail(KVS_ERR_INVALID_ARG, "keep_idx or keep_count is NULL");
    if (B <= 0 || max_keep <= 0) return fail(KVS_ERR_INVALID_ARG, "B and max_keep must be positive (B=%d, max_keep=%d)", B, max_keep);
    if (max_keep > store->desc.max_blocks_per_seq * KVS_BLOCK_TOKENS)
        return fail(KVS_ERR_CAPACITY, "max_keep=%d exceeds the per-sequence capacity %d", max_keep,
                    store->desc.max_blocks_per_seq * KVS_BLOCK_TOKENS);
    if (!store->block_table && (long)B * store->desc.max_blocks_per_seq > store->desc.num_blocks)
        return fail(KVS_ERR_CAPACITY, "contiguous store: B * max_blocks_per_seq exceeds num_blocks");
    if (B > 65535) return fail(KVS_ERR_CAPACITY, "B is limited to 65535");
    if (store->host_share_map[layer] != layer) return KVS_NOOP;   // its donor's compaction is the one it reads
    kvs::CompactArgs a;
    a.st = view_of(store, layer);
    a.keep_idx = keep_idx;
    a.keep_count = keep_count;
    a.max_keep = max_keep;
    a.B = B;
    if (int e = kvs::launch_compact(a, stream)) return fail(KVS_ERR_HIP, "compaction launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

int kvs_project_append_kv(const kvs_store* store, int layer, const void* x, int hidden, const void* w_k,
                          const void* w_v, const float* rope_cos, const float* rope_sin, int rope_positions,
                          const int32_t* start_pos, int B, int T_new, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!x || !w_k || !w_v || !start_pos) return fail(KVS_ERR_INVALID_ARG, "x, w_k, w_v or start_pos is NULL");
    if ((rope_cos == nullptr) != (rope_sin == nullptr))
        return fail(KVS_ERR_INVALID_ARG, "rope_cos and rope_sin must be given together");
    if (store->desc.dtype == KVS_F32) return fail(KVS_ERR_UNSUPPORTED, "the fused projection needs a bf16 or fp8 store");
    if (hidden <= 0 || hidden % 128 != 0) return fail(KVS_ERR_UNSUPPORTED, "hidden must be a positive multiple of 128 (got %d)", hidden);
    if (B <= 0 || T_new <= 0) return fail(KVS_ERR_INVALID_ARG, "B and T_new must be positive (B=%d, T_new=%d)", B, T_new);
    const long capacity = (long)store->desc.max_blocks_per_seq * KVS_BLOCK_TOKENS;
    if (T_new > capacity) return fail(KVS_ERR_CAPACITY, "T_new=%d exceeds the per-sequence capacity %ld", T_new, capacity);
    if (rope_cos && rope_positions < capacity)
        return fail(KVS_ERR_CAPACITY, "rotary tables cover %d positions, the store holds %ld per sequence", rope_positions, capacity);
    if ((long)B * T_new > (1L << 30) || ((long)B * T_new + 15) / 16 > 65535)
        return fail(KVS_ERR_CAPACITY, "B * T_new is limited to 16 * 65535 rows per call");
    if (!store->block_table && (long)B * store->desc.max_blocks_per_seq > store->desc.num_blocks)
        return fail(KVS_ERR_CAPACITY, "contiguous store: B * max_blocks_per_seq exceeds num_blocks");
    if (store->host_share_map[layer] != layer) return KVS_NOOP;   // the work sharing saves
    const size_t need = kvs::project_workspace_bytes(store->desc.Hkv, store->desc.head_dim, hidden, B * T_new);
    if (!workspace || workspace_bytes < need)
        return fail(KVS_ERR_INVALID_ARG, "workspace too small: need %zu bytes, got %zu", need, workspace_bytes);
    kvs::ProjectArgs a;
    a.st = view_of(store, layer);
    a.x = x;
    a.w_k = w_k;
    a.w_v = w_v;
    a.rope_cos = rope_cos;
    a.rope_sin = rope_sin;
    a.start_pos = start_pos;
    a.hidden = hidden;
    a.B = B;
    a.T = T_new;
    if (int e = kvs::launch_project_append(a, workspace, stream)) return fail(KVS_ERR_HIP, "projection launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

size_t kvs_project_workspace_bytes(const kvs_desc* d, int hidden, int B, int T_new)
{
    if (check_desc(d) != KVS_OK) return 0;
    if (d->dtype == KVS_F32 || hidden <= 0 || hidden % 128 != 0 || B <= 0 || T_new <= 0 || (long)B * T_new > (1L << 30)) {
        fail(KVS_ERR_INVALID_ARG, "bf16 or fp8 store, hidden a positive multiple of 128, B and T_new positive");
        return 0;
    }
    return kvs::project_workspace_bytes(d->Hkv, d->head_dim, hidden, B * T_new);
}

int kvs_gather_kv(const kvs_store* store, int layer, int t0, int T, int B,
                  void* k_out, void* v_out, void* stream)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!k_out || !v_out) return fail(KVS_ERR_INVALID_ARG, "k_out or v_out is NULL");
    if (B <= 0 || T <= 0 || t0 < 0) return fail(KVS_ERR_INVALID_ARG, "need B > 0, T > 0, t0 >= 0");
    if ((long)t0 + T > (long)store->desc.max_blocks_per_seq * KVS_BLOCK_TOKENS)
        return fail(KVS_ERR_CAPACITY, "tokens [%d, %d) exceed the per-sequence capacity", t0, t0 + T);
    if (!store->block_table && (long)B * store->desc.max_blocks_per_seq > store->desc.num_blocks)
        return fail(KVS_ERR_CAPACITY, "contiguous store: B * max_blocks_per_seq exceeds num_blocks");
    kvs::CopyArgs a;
    a.st = view_of(store, layer);
    a.k = k_out;
    a.v = v_out;
    a.start_pos = nullptr;
    a.pos_per_head = 0;
    a.pos_bias = 0;
    a.t0 = t0;
    a.B = B;
    a.T = T;
    if (int e = kvs::launch_gather(a, stream)) return fail(KVS_ERR_HIP, "gather launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

int kvs_check_store(const kvs_store* store, int B, int32_t* report, void* stream)
{
    if (int rc = check_store(store, 0)) return rc;
    if (!report) return fail(KVS_ERR_INVALID_ARG, "report is NULL");
    if (B < 0) return fail(KVS_ERR_INVALID_ARG, "B must not be negative (B=%d)", B);
    if (store->desc.L > kvs::kMaxCheckedLayers)
        return fail(KVS_ERR_UNSUPPORTED, "the check covers at most %d layers (L=%d)", kvs::kMaxCheckedLayers, store->desc.L);
    if (!store->block_table && (long)B * store->desc.max_blocks_per_seq > store->desc.num_blocks)
        return fail(KVS_ERR_CAPACITY, "contiguous store: B * max_blocks_per_seq exceeds num_blocks");
    kvs::CheckArgs a = {};
    a.st = view_of(store, 0);
    a.B = B;
    a.report = report;
    std::copy(store->host_share_map, store->host_share_map + store->desc.L, a.host_share_map);
    std::copy(store->host_slot_of_layer, store->host_slot_of_layer + store->desc.L, a.host_slot_of_layer);
    if (int e = kvs::launch_check_store(a, stream)) return fail(KVS_ERR_HIP, "store check launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

static int attention_common(const kvs_store* store, int layer, const void* q, const int32_t* lens,
                            int lens_per_head, int lens_bias, int B, int T_new, float* out, void* workspace,
                            size_t workspace_bytes, void* stream, const void* k_new = nullptr,
                            const void* v_new = nullptr)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!q || !lens || !out) return fail(KVS_ERR_INVALID_ARG, "q, lengths or out is NULL");
    if (B <= 0 || T_new <= 0) return fail(KVS_ERR_INVALID_ARG, "B and T_new must be positive (B=%d, T_new=%d)", B, T_new);
    const kvs_desc* d = &store->desc;
    if (T_new > d->max_blocks_per_seq * KVS_BLOCK_TOKENS)
        return fail(KVS_ERR_CAPACITY, "T_new=%d exceeds the per-sequence capacity", T_new);
    if (!store->block_table && (long)B * d->max_blocks_per_seq > d->num_blocks)
        return fail(KVS_ERR_CAPACITY, "contiguous store: B * max_blocks_per_seq exceeds num_blocks");
    const Split s = choose_split(d, B, T_new, lens_per_head != 0);
    if (B > 65535 || (long)s.n_splits * s.n_col_groups > 65535)
        return fail(KVS_ERR_CAPACITY, "launch too large: B and splits x column groups are limited to 65535");
    if (counters_used(d, B, s) > kvs::kMaxCounters)        // only a forced split of a very large batch gets here
        return fail(KVS_ERR_CAPACITY, "a split context is limited to %zu (sequence, kv head, column group) items", kvs::kMaxCounters);
    const size_t need = kvs::kCounterRegionBytes + partial_floats(d, B, T_new, s) * sizeof(float);
    if (!workspace || workspace_bytes < need)
        return fail(KVS_ERR_INVALID_ARG, "workspace too small: need %zu bytes, got %zu", need, workspace_bytes);
    kvs::AttnArgs a;
    a.st = view_of(store, layer);
    a.q = q;
    a.lens = lens;
    a.lens_per_head = lens_per_head;
    a.k_new = k_new;
    a.v_new = v_new;
    a.lens_bias = lens_bias;
    a.B = B;
    a.T_new = T_new;
    a.out = out;
    a.counters = static_cast<int32_t*>(workspace);
    a.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kvs::kCounterRegionBytes);
    a.pages_per_split = s.pages_per_split;
    a.n_splits = s.n_splits;
    a.wide_cols = s.wide_cols;
    a.col_blocks = 0;
    a.col_paired = 0;
    a.adaptive = s.adaptive;
    a.want_splits = s.want_splits;
    a.n_items = s.n_items;
    if (int e = s.adaptive == 3 ? kvs::launch_decode_flat(a, stream) : kvs::launch_attention(a, stream))
        return fail(KVS_ERR_HIP, "attention launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

int kvs_decode_attention(const kvs_store* store, int layer, const void* q, const int32_t* seq_lens,
                         int B, float* out, void* workspace, size_t workspace_bytes, void* stream)
{
    return attention_common(store, layer, q, seq_lens, 0, 0, B, 1, out, workspace, workspace_bytes, stream);
}

int kvs_decode_step(const kvs_store* store, int layer, const void* q, const void* k_new, const void* v_new,
                    const int32_t* seq_lens, int B, float* out, void* workspace, size_t workspace_bytes,
                    void* stream)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!k_new || !v_new || !seq_lens) return fail(KVS_ERR_INVALID_ARG, "k_new, v_new or seq_lens is NULL");
    const bool own = store->host_share_map[layer] == layer;
    if (own && store->desc.dtype == KVS_F32) {
        // the fp32 store: the two launches the fused kernel replaces
        if (int rc = append_common(store, layer, k_new, v_new, seq_lens, 0, B, 1, stream, -1)) return rc;
        return attention_common(store, layer, q, seq_lens, 0, 0, B, 1, out, workspace, workspace_bytes, stream);
    }
    return attention_common(store, layer, q, seq_lens, 0, 0, B, 1, out, workspace, workspace_bytes, stream,
                            own ? k_new : nullptr, own ? v_new : nullptr);
}

int kvs_decode_attention_per_head(const kvs_store* store, int layer, const void* q, const int32_t* kv_lens,
                                  int B, float* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (int rc = check_store(store, layer)) return rc;
    if (!kv_lens) return fail(KVS_ERR_INVALID_ARG, "kv_lens is NULL");
    if (B <= 0) return fail(KVS_ERR_INVALID_ARG, "B must be positive (B=%d)", B);
    // the lengths of the slot this layer reads: its donor's (the host copies of the two maps
    // mirror the device ones the kernel resolves the pages with)
    const int slot = store->host_slot_of_layer[store->host_share_map[layer]];
    const int32_t* lens = kv_lens + (size_t)slot * B * store->desc.Hkv;
    return attention_common(store, layer, q, lens, 1, 0, B, 1, out, workspace, workspace_bytes, stream);
}

int kvs_prefill_attention(const kvs_store* store, int layer, const void* q, const int32_t* start_pos,
                          int B, int T_new, float* out, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    return attention_common(store, layer, q, start_pos, 0, 1, B, T_new, out, workspace, workspace_bytes, stream);
}

size_t kvs_distance_workspace_bytes(int L)
{
    if (L <= 0 || L > 128) { fail(KVS_ERR_UNSUPPORTED, "L must be in [1, 128]"); return 0; }
    return kvs::distance_workspace_bytes(L);
}

int kvs_layer_distance(const void* kv_samples, int S, int L, size_t N, int dtype,
                       float* dK2, float* dV2, float* D, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    if (!kv_samples || !dK2 || !dV2 || !D) return fail(KVS_ERR_INVALID_ARG, "NULL argument");
    if (S <= 0 || L <= 0 || N == 0) return fail(KVS_ERR_INVALID_ARG, "S, L and N must be positive");
    if (L > 128) return fail(KVS_ERR_UNSUPPORTED, "L=%d: at most 128 layers are supported", L);
    if (dtype != KVS_F32 && dtype != KVS_BF16) return fail(KVS_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (N % 8 != 0) return fail(KVS_ERR_UNSUPPORTED, "N must be a multiple of 8 (got %zu)", N);
    if ((size_t)S * L * 2 > ((size_t)1 << 62) / N) return fail(KVS_ERR_CAPACITY, "input too large");
    const size_t need = kvs::distance_workspace_bytes(L);
    if (!workspace || workspace_bytes < need)
        return fail(KVS_ERR_INVALID_ARG, "workspace too small: need %zu bytes, got %zu", need, workspace_bytes);
    if (int e = kvs::launch_layer_distance(kv_samples, S, L, N, dtype, dK2, dV2, D, workspace, stream))
        return fail(KVS_ERR_HIP, "distance launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

size_t kvs_cos_sim_workspace_bytes(int S)
{
    if (S <= 0 || S > 65535) { fail(KVS_ERR_INVALID_ARG, "S must be in [1, 65535]"); return 0; }
    return kvs::cos_sim_workspace_bytes(S);
}

int kvs_avg_cos_sim(const void* hidden_shared, const void* hidden_original, int S, size_t N, int dtype, int mode,
                    float* similarity, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!hidden_shared || !hidden_original || !similarity) return fail(KVS_ERR_INVALID_ARG, "NULL argument");
    if (S <= 0 || S > 65535 || N == 0) return fail(KVS_ERR_INVALID_ARG, "need 0 < S <= 65535 and N > 0");
    if (dtype != KVS_F32 && dtype != KVS_BF16) return fail(KVS_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (mode != 0 && mode != 1) return fail(KVS_ERR_INVALID_ARG, "mode must be 0 (mean first) or 1 (per sentence)");
    const size_t need = kvs::cos_sim_workspace_bytes(S);
    if (!workspace || workspace_bytes < need)
        return fail(KVS_ERR_INVALID_ARG, "workspace too small: need %zu bytes, got %zu", need, workspace_bytes);
    if (int e = kvs::launch_cos_sim(hidden_shared, hidden_original, S, N, dtype, mode, similarity, workspace, stream))
        return fail(KVS_ERR_HIP, "similarity launch: %s", kvs::hip_error_string(e));
    return KVS_OK;
}

}  // extern "C"
