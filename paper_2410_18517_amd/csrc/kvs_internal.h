// Internal interface between the host-side C ABI (kvs_host.cpp) and the kernel launchers
// (*.hip).  Plain structs only; nothing here is visible to callers of the library.
#pragma once
#include <cstddef>
#include <cstdint>

namespace kvs {

// Every workspace starts with a region of arrival counters of this fixed size (they must start,
// and every call leaves them, at zero); the partial results of a call follow it.  The size does
// not depend on the call's shape, so calls of different batch sizes, row counts and kinds can
// take turns on one workspace without one call's partial results landing where another call
// keeps its counters.  A call that splits work uses at most kMaxCounters of them.
constexpr size_t kCounterRegionBytes = 64 * 1024;
constexpr size_t kMaxCounters = kCounterRegionBytes / sizeof(int32_t);

struct StoreView {
    void* pool;
    const int32_t* share_map;      // device [L]
    const int32_t* slot_of_layer;  // device [L]
    const int32_t* block_table;    // device [B][max_blocks_per_seq] or nullptr (contiguous)
    int32_t layer, L, n_slots, Hq, Hkv, head_dim, dtype, num_blocks, max_blocks_per_seq;
};

struct AttnArgs {
    StoreView st;
    const void* q;          // device [B][T_new][Hq][D], store dtype
    const int32_t* lens;    // device [B]: decode: tokens in the cache; prefill: position of row 0
    int32_t lens_per_head;  // 1: lens is [B][Hkv], the tokens each kv head of the slot still holds (decode only)
    const void* k_new;      // decode step that also stores this step's token (bf16 store, own-cache layer):
    const void* v_new;      //   device [B][1][Hkv][D]; the token sits at position lens[b] - 1.  Else nullptr.
    int32_t lens_bias;      // 0 for decode (row r sees lens + r keys), 1 for prefill
    int32_t B, T_new;
    float* out;             // device fp32 [B][T_new][Hq][D]
    float* partials;        // device fp32 [B][T_new][Hq][n_splits][D + 2]
    int32_t* counters;      // device [B][Hkv][n_col_groups], zero between calls
    int32_t pages_per_split, n_splits;   // n_splits: split indices in the grid and records per row in partials
    int32_t adaptive;       // decode: 1 = the split kernel sizes the splits by the lengths it finds (pages_per_split is then
    int32_t want_splits;    //   what full sequences get); want_splits: workgroups a sequence of mean length is shared among.
    int32_t n_items;        //   3 = the kernel of kvs_decode.hip: n_items workgroups share the launch's pages out by
                            //   tokens; partials one record per (workgroup + segment, head of the group)
    int32_t wide_cols;      // prefill: 0 = the page-splitting kernel, else columns per workgroup of the shared-page kernel (64, 128, 256)
    int32_t col_blocks;     // set by the launch: > 0 = the shared-page kernel runs on a 1-D grid dealt to the XCDs, with this
                            //   many column blocks per (sequence, kv head); 0 = grid (kv head, sequence, blocks x splits)
    int32_t col_paired;     //   1 = a workgroup of that grid takes two column blocks in turn, the k-th longest and the k-th shortest
};

struct CopyArgs {
    StoreView st;
    void* k;                // device [B][T][Hkv][D]
    void* v;
    const int32_t* start_pos;  // device [B] (append) or nullptr (gather: t0 for all)
    int32_t pos_per_head;      // 1: start_pos is [B][Hkv]
    int32_t pos_bias;          // added to every start position (-1: the caller passed lengths that count the new row)
    int32_t t0, B, T;
};

struct CompactArgs {
    StoreView st;
    const int32_t* keep_idx;    // device [B][Hkv][max_keep], increasing token positions
    const int32_t* keep_count;  // device [B][Hkv]
    int32_t max_keep, B;
};

constexpr int kMaxCheckedLayers = 256;   // the host copies of the maps travel as kernel arguments

struct CheckArgs {
    StoreView st;
    int32_t B;                                       // rows of the block table to look at
    int32_t* report;                                 // device [2]
    int32_t host_share_map[kMaxCheckedLayers];
    int32_t host_slot_of_layer[kMaxCheckedLayers];
};

struct ProjectArgs {
    StoreView st;
    const void* x;          // device [B][T][hidden], bf16
    const void* w_k;        // device [Hkv*D][hidden], bf16
    const void* w_v;
    const float* rope_cos;  // device [positions][D/2] or nullptr
    const float* rope_sin;
    const int32_t* start_pos;  // device [B]
    int32_t hidden, B, T;
    int32_t k_splits;       // workgroups sharing one output tile's contraction (set by the launcher)
    int32_t* counters;      // device, one per output tile, zero between calls
    float* partials;        // device [k_splits][tiles][256][2]
};

// Each returns hipError_t as int (0 = success) after enqueueing on `stream`.
int launch_append(const CopyArgs& a, void* stream);
int launch_gather(const CopyArgs& a, void* stream);
int launch_compact(const CompactArgs& a, void* stream);
int launch_check_store(const CheckArgs& a, void* stream);
int launch_attention(const AttnArgs& a, void* stream);
int launch_decode_flat(const AttnArgs& a, void* stream);          // a.adaptive == 3: grid of a.n_items workgroups
size_t decode_flat_partial_floats(int n_wg, int B, int Hq, int Hkv, int head_dim);
int launch_project_append(ProjectArgs a, void* workspace, void* stream);
size_t project_workspace_bytes(int Hkv, int head_dim, int hidden, int rows);
int launch_layer_distance(const void* kv, int S, int L, size_t N, int dtype, float* dK2, float* dV2,
                          float* D, void* workspace, void* stream);
size_t distance_workspace_bytes(int L);
int launch_cos_sim(const void* a, const void* b, int S, size_t N, int dtype, int mode, float* out, void* workspace,
                   void* stream);
size_t cos_sim_workspace_bytes(int S);
const char* hip_error_string(int err);
int report_error(int code, const char* message);   // sets what kvs_last_error() returns on this thread; returns code

}  // namespace kvs
