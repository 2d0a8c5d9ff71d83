/*
 * kvs.h -- C ABI of libkvs: decode attention over a layer-shared KV cache on MI355X (gfx950).
 *
 * Method (KVSharer, arXiv 2410.18517): a sharing strategy names, for some layers, a donor
 * layer nearer the input whose KV cache the layer reads instead of computing and storing
 * its own (Sec. 3.2 and the prefill/generation figure); everything after the substitution
 * is the host model's ordinary attention.  The strategy is found by ranking all layer
 * pairs by the Euclidean distance between their calibration-averaged KV caches, most
 * dissimilar first, and walking the ranking (Sec. 3.1.2, Algorithm 1).
 *
 * Conventions
 *   - Every function returns a status: KVS_OK / KVS_NOOP are not errors; negatives are.
 *     kvs_last_error() returns a thread-local description of the last failure.
 *   - The caller owns all memory.  Pointers marked "device" are GPU allocations made by the
 *     caller; "host" pointers are ordinary memory.  The library never allocates or frees
 *     device memory and never synchronises: every kernel is enqueued on the hipStream_t the
 *     caller passes as `void* stream` (NULL = the default stream).
 *   - Every argument check that does not need the GPU runs before the first HIP call.
 *   - share_map[l] is the layer whose cache layer l reads (l itself if l keeps its own);
 *     valid maps have share_map[l] <= l and share_map[share_map[l]] == share_map[l].
 *     slot_of_layer[l] is the KV-store slot of that cache; layers that keep their own
 *     cache own slots 0..n_slots-1 in increasing layer order.
 *
 * KV store layout (device, one allocation of kvs_store_bytes()):
 *     pool[slot][block][kv_head][K=0|V=1][page]     page = 16 tokens x head_dim elements
 *   A page is contiguous (4 KiB for bf16, head_dim 128).  Token j of sequence b lives in
 *   row j % 16 of block block_table[b][j / 16]; with block_table == NULL the store is
 *   contiguous per sequence: that block is b * max_blocks_per_seq + j / 16.  One block table
 *   serves all slots.  Element order inside a page:
 *     KVS_F32 : [token][channel].
 *     KVS_BF16: operand order of the matrix-core tiles that consume it, so a wavefront
 *               reads 1 KiB contiguous per load and feeds it to MFMA untransposed:
 *       K page: element (token t, channel c) at (((c/32)*4 + (c%32)/8)*16 + t)*8 + c%8
 *       V page: element (t, c) at ((((c/32)*4 + t/4)*16 + c%16)*2 + (c/16)%2)*4 + t%4
 *     KVS_FP8 : one byte per element, the OCP 8-bit float E4M3 (bias 7, largest value 448, no
 *               infinities), unscaled; rows and queries cross the boundary as bf16.  An append
 *               rounds to nearest, ties to even, saturating at +-448 (NaN stays NaN); a gather
 *               returns the stored values exactly.  The attention kernels widen the bytes to
 *               bf16 in registers and then run the bf16 path, so a slot costs half the HBM
 *               bytes of a bf16 slot per decode step.  In-page order, again the operand order:
 *       K page: element (t, c) at (((c/64)*4 + (c%32)/8)*16 + t)*16 + ((c/32)%2)*8 + c%8
 *       V page: element (t, c) at (((c/64)*4 + t/4)*16 + c%16)*16 + ((c/16)%4)*4 + t%4
 *   Only kvs_append_kv writes pages and only the attention kernels / kvs_gather_kv read
 *   them, so callers never depend on the in-page order.
 */
#ifndef KVS_H
#define KVS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVS_OK                     0
#define KVS_NOOP                   1   /* nothing to do (e.g. append on a layer that reads a donor) */
#define KVS_ERR_INVALID_ARG       -1
#define KVS_ERR_BAD_MAP           -2
#define KVS_ERR_CAPACITY          -3
#define KVS_ERR_TARGET_UNREACHED  -4
#define KVS_ERR_UNSUPPORTED       -5
#define KVS_ERR_HIP               -6

#define KVS_F32   0
#define KVS_BF16  1
#define KVS_FP8   2   /* store only: q, k_new, v_new and gathered rows are bf16 */

#define KVS_BLOCK_TOKENS 16

const char* kvs_last_error(void);

/* ---------------------------------------------------------------- strategy (host only) */

/* Similarity test of Algorithm 1 ("Avg_Cos_Sim(...) > T"), supplied by the caller because
 * it needs the model: return 1 to keep the candidate strategy, 0 to discard the pair. */
typedef int (*kvs_accept_fn)(const int32_t* candidate_share_map, int L, void* user);

/*
 * Structural part of Algorithm 1 (ranking + greedy walk).  Pairs (i < j) are ranked by
 * dist[i*L + j], largest first (order = 0, the paper's choice) or smallest first (order = 1,
 * the "share similar layers" ablation of Sec. 5.1); ties keep (i, j) lexicographic order.
 * In a pair the layer nearer the output (j) receives the cache of the layer nearer the input
 * (i).  Strategies stay depth one: a pair is passed over -- no accept call, not counted --
 * when j already receives or donates a cache or i already receives one.  The walk stops
 * when target_shared layers receive a cache.
 *   dist            host, L*L row-major, only the upper triangle is read; NaN -> INVALID_ARG
 *   accept          NULL accepts every candidate
 *   share_map, slot_of_layer   host, out[L];  n_slots, n_shared   host, out
 * Returns KVS_OK, or KVS_ERR_TARGET_UNREACHED with the partial strategy in the outputs
 * when the ranking is exhausted first (the search then reports that it found no strategy).
 * The random-sharing baseline (Sec. 5.3, random pairs at a fixed compression rate) is the same
 * walk over a ranking drawn at random: pass a matrix of independent random values, accept = NULL.
 */
int kvs_build_share_map(const float* dist, int L, int target_shared, int order,
                        kvs_accept_fn accept, void* user,
                        int32_t* share_map, int32_t* slot_of_layer,
                        int32_t* n_slots, int32_t* n_shared);

/* KVS_OK iff the host array is a depth-one map with donor <= layer; else KVS_ERR_BAD_MAP. */
int kvs_validate_share_map(const int32_t* share_map, int L);

/* Slot numbering of a valid map (host in, host out[L]); *n_slots = layers keeping a cache. */
int kvs_slots_from_share_map(const int32_t* share_map, int L, int32_t* slot_of_layer,
                             int32_t* n_slots);

/* ---------------------------------------------------------------- KV store */

typedef struct kvs_desc {
    int32_t L;                   /* layers of the model */
    int32_t n_slots;             /* layer caches actually held: L - (shared layers) */
    int32_t Hq, Hkv, head_dim;   /* Hq % Hkv == 0; query head h reads kv head h / (Hq/Hkv) */
    int32_t dtype;               /* KVS_F32, KVS_BF16: element type of the store and of q, k_new, v_new; KVS_FP8: see above */
    int32_t block_tokens;        /* must be KVS_BLOCK_TOKENS */
    int32_t num_blocks;          /* blocks per slot */
    int32_t max_blocks_per_seq;  /* columns of the block table; capacity = 16 * this */
} kvs_desc;

typedef struct kvs_store {
    kvs_desc desc;
    void* pool;                       /* device, kvs_store_bytes(&desc) bytes */
    const int32_t* share_map;         /* device [L] */
    const int32_t* slot_of_layer;     /* device [L] */
    const int32_t* block_table;       /* device [B][max_blocks_per_seq], or NULL = contiguous */
    const int32_t* host_share_map;    /* host [L]: same values; used for checks and KVS_NOOP only */
    const int32_t* host_slot_of_layer;/* host [L] */
} kvs_store;

/* Bytes of the pool; 0 (with kvs_last_error set) if the descriptor is invalid/unsupported.
 * Supported: KVS_BF16 and KVS_FP8 with head_dim 128 or 64 and Hq/Hkv <= 16; KVS_F32 with
 * head_dim a multiple of 64 up to 256. */
size_t kvs_store_bytes(const kvs_desc* desc);

/* Bytes of scratch the attention calls need for B sequences of 1 to max_q_rows query rows
 * each (1 for decode): enough for every row count in that range.  The scratch starts with a
 * region of arrival counters whose size is the same for every call (64 KiB), followed by the
 * split-context partial results.  The caller zero-fills the workspace once after allocating it;
 * every call leaves the counters zero again and writes partial results only behind the counter
 * region, so calls of different batch sizes, row counts and kinds (decode, prefill, per-head) may
 * take turns on one workspace that is large enough for each of them.  Calls sharing one
 * workspace must not overlap in time. */
size_t kvs_workspace_bytes(const kvs_desc* desc, int B, int max_q_rows);

/*
 * Store this step's keys/values of `layer` (Sec. 3.2: only layers that keep their own cache
 * compute and store KV).  k_new, v_new: device [B][T_new][Hkv][head_dim] of desc.dtype,
 * copied bit for bit.  Row i of sequence b goes to token position start_pos[b] + i
 * (start_pos: device [B]); positions >= capacity are dropped.
 * Returns KVS_NOOP without touching the GPU when the layer reads a donor's cache.
 */
int kvs_append_kv(const kvs_store* store, int layer, const void* k_new, const void* v_new,
                  const int32_t* start_pos, int B, int T_new, void* stream);

/*
 * Key/value projection fused with the append: the computation a sharing strategy removes for
 * every layer that reads a donor's cache (Sec. 3.2; the cache computation the abstract counts as saved).
 * For a layer that keeps its own cache, with x device [B][T_new][hidden] and the projection
 * weights w_k, w_v device [Hkv*head_dim][hidden] (row = output channel, bf16):
 *     k = x . w_k^T,   v = x . w_v^T                      (fp32 accumulation)
 *     k[c], k[c+h] <- k[c] cos - k[c+h] sin,  k[c+h] cos + k[c] sin      h = head_dim/2, c < h,
 *          cos = rope_cos[p][c], sin = rope_sin[p][c], p = start_pos[b] + i  (skipped if NULL)
 *     rounded to bf16 (nearest even) and stored at position p of the layer's slot (an fp8 store
 *     rounds that bf16 value on to E4M3, as kvs_append_kv of the bf16 row would).
 * rope_cos, rope_sin: device fp32 [rope_positions][head_dim/2], rope_positions >= capacity.
 * bf16 and fp8 stores (x and the weights are bf16 either way); hidden a multiple of 128.  workspace: device, >=
 * kvs_project_workspace_bytes(), zero-filled once by the caller; it has the layout of the attention
 * workspace (a 64 KiB region of arrival counters that every call leaves zero, then the partial sums
 * of the split contraction), so calls of any row count may take turns on it; calls sharing it must
 * not overlap in time.  Returns KVS_NOOP without touching the GPU when the layer reads a donor's cache.
 */
int kvs_project_append_kv(const kvs_store* store, int layer, const void* x, int hidden,
                          const void* w_k, const void* w_v,
                          const float* rope_cos, const float* rope_sin, int rope_positions,
                          const int32_t* start_pos, int B, int T_new,
                          void* workspace, size_t workspace_bytes, void* stream);

size_t kvs_project_workspace_bytes(const kvs_desc* desc, int hidden, int B, int T_new);

/*
 * Read back T tokens starting at t0 of every sequence from the cache `layer` attends to
 * (its donor's when it has one), in the order kvs_append_kv takes:
 * k_out, v_out device [B][T][Hkv][head_dim].  Inverse of kvs_append_kv; for checks, cache
 * migration and debugging.
 */
int kvs_gather_kv(const kvs_store* store, int layer, int t0, int T, int B,
                  void* k_out, void* v_out, void* stream);

/*
 * Debug aid for the share-map and page indexing of Sec. 3.2.  The kernels resolve
 * slot_of_layer[share_map[layer]] and the pages from the store's DEVICE arrays and clamp whatever
 * they find into the pool (memory safety), while argument checks and the KVS_NOOP decisions use
 * the HOST copies: the two must hold the same values, and a difference, or a page-table entry
 * outside [0, num_blocks), is otherwise silent (the call reads or writes some other slot or page
 * and returns KVS_OK).  This call makes it observable: report (device int32[2]) receives
 *   report[0] = entries of share_map / slot_of_layer whose device value differs from the host copy,
 *   report[1] = entries of the first B rows of the block table outside [0, num_blocks)
 * (0 for a contiguous store).  One small kernel on `stream`; L <= 256.
 */
int kvs_check_store(const kvs_store* store, int B, int32_t* report, void* stream);

/*
 * One decode step of `layer` (Sec. 3.2): out[b][h][:] = softmax_j(q[b][h] . K[b][g][j] /
 * sqrt(head_dim)) . V[b][g][j][:] over j < seq_lens[b], g = h / (Hq/Hkv), where K, V are
 * the cache of slot_of_layer[share_map[layer]] -- resolved on the device.  seq_lens counts
 * the token appended this step.  seq_lens[b] == 0 gives a zero row; values above the
 * capacity are clamped to it.
 *   q device [B][Hq][head_dim] of desc.dtype;  seq_lens device [B];  out device fp32
 *   [B][Hq][head_dim];  workspace device, >= kvs_workspace_bytes(desc, B, 1).
 */
int kvs_decode_attention(const kvs_store* store, int layer, const void* q,
                         const int32_t* seq_lens, int B, float* out,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * kvs_decode_attention for callers that cannot allocate device memory or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * without the workspace, same kernels, same result bit for bit; the scratch is an 8 MiB device
 * array inside the library (kvs_noalloc_scratch_bytes()), one copy per GPU, held until the process
 * ends.  The call allocates and frees nothing.  Shapes whose kvs_workspace_bytes(desc, B, 1)
 * exceeds the array are refused with KVS_ERR_CAPACITY before any launch.  All such calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 * race on it; calls in stream order do not.  The first call on a device looks up the array's
 * address there (hipGetSymbolAddress, no allocation) and should be made outside a graph capture.
 */
int kvs_decode_attention_noalloc(const kvs_store* store, int layer, const void* q,
                                 const int32_t* seq_lens, int B, float* out, void* stream);

size_t kvs_noalloc_scratch_bytes(void);

/*
 * One decode step in one launch: kvs_append_kv(k_new, v_new at position seq_lens[b] - 1) followed
 * by kvs_decode_attention(q, seq_lens), for the layers that keep their own cache; for a layer
 * that reads a donor's cache k_new and v_new are ignored and the call is kvs_decode_attention
 * (its donor stored this step's token when its own turn came).  On a bf16 or fp8 store the
 * attention kernel takes the new token from k_new / v_new directly -- it joins the softmax in the
 * merge of the context splits, with the values the store will hold (rounded to E4M3 for an fp8
 * store) -- and writes it to its place in the store on the side, so no second launch and no wait
 * for the write; on an fp32 store the call is the two launches.
 *   q device [B][Hq][head_dim], k_new, v_new device [B][1][Hkv][head_dim], all bf16 (fp32 for an
 *   fp32 store);  seq_lens device [B], counting the new token;  out, workspace as
 *   kvs_decode_attention.  Positions at or beyond the capacity are not stored.
 */
int kvs_decode_step(const kvs_store* store, int layer, const void* q, const void* k_new,
                    const void* v_new, const int32_t* seq_lens, int B, float* out,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Causal attention of T_new new query rows per sequence (the prefill side of Sec. 3.2):
 * row i of sequence b sits at position start_pos[b] + i and sees keys 0..start_pos[b] + i of
 * the cache `layer` attends to, which must already hold them (append first; a recipient's
 * donor, being nearer the input, has been appended earlier in the same pass).
 *   q device [B][T_new][Hq][head_dim];  out device fp32 [B][T_new][Hq][head_dim];
 *   workspace >= kvs_workspace_bytes(desc, B, T_new).
 */
int kvs_prefill_attention(const kvs_store* store, int layer, const void* q,
                          const int32_t* start_pos, int B, int T_new, float* out,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------- intra-layer sparsified slots (per-head token sets)
 *
 * Layer sharing composes with token-dropping methods such as H2O and PyramidInfer (Sec. 4.6,
 * "Compatibility with Intra-layer Compression", and the appendix on their reproduction): every
 * layer that keeps a cache sparsifies it by that method's own rule, and a layer that shares
 * reads the already sparsified cache of its donor.  Which tokens to keep is the caller's
 * policy; the three calls below are the storage and attention side.  A sparsified slot holds,
 * for every (sequence, kv head), its kept tokens at positions 0 .. n-1 of the head's pages, n
 * differing per head; the attention is the softmax over exactly those tokens and does not
 * depend on their order (positions are already inside the keys).
 */

/*
 * Keep, for every (sequence, kv head) of the slot `layer` owns, the tokens at positions
 * keep_idx[b][g][0 .. keep_count[b][g]) and move them to positions 0 .. keep_count[b][g], in
 * place.  keep_idx must be strictly increasing within a head and below the head's current
 * length (not checked: other values stay inside the store but give an unspecified token
 * set); counts are clamped to [0, max_keep].  Positions at and after the count keep stale data.
 *   keep_idx device int32 [B][Hkv][max_keep];  keep_count device int32 [B][Hkv].
 * Returns KVS_NOOP for a layer that reads a donor's cache (the donor's compaction is the one
 * it sees).  Cost: the workgroups of a (sequence, kv head) walk its kept tokens in order, 1024
 * at a time; a maintenance operation, not part of the decode step.
 */
int kvs_compact_kv(const kvs_store* store, int layer, const int32_t* keep_idx,
                   const int32_t* keep_count, int max_keep, int B, void* stream);

/*
 * kvs_append_kv with a write position per (sequence, kv head): rows i of head g of sequence b go
 * to positions pos[b][g] + i.  With per-head lengths this is both "extend the head by one
 * token" (pos = its length) and "overwrite the token the policy just evicted" (pos = its
 * index).  pos device int32 [B][Hkv]; everything else as kvs_append_kv.
 */
int kvs_append_kv_per_head(const kvs_store* store, int layer, const void* k_new, const void* v_new,
                           const int32_t* pos, int B, int T_new, void* stream);

/*
 * kvs_decode_attention over a sparsified slot: kv head g of sequence b attends to its first
 * kv_lens[slot][b][g] tokens, slot = slot_of_layer[share_map[layer]] (taken from the store's
 * host copies of the maps; pages are still resolved on the device).  A length of 0 gives zero
 * rows for the head's query heads; lengths above the capacity are clamped.
 *   kv_lens device int32 [n_slots][B][Hkv];  everything else as kvs_decode_attention.
 */
int kvs_decode_attention_per_head(const kvs_store* store, int layer, const void* q,
                                  const int32_t* kv_lens, int B, float* out,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------- calibration distance */

/*
 * Layer-dissimilarity matrix of the strategy search (Sec. 3.1.2, Algorithm 1).
 * kv_samples: device [S][L][2][N] of `dtype`: calibration sample, layer, keys(0)/values(1),
 * flattened [Hkv][T][head_dim] index; all samples have the same length.  The keys and the
 * values of a layer are averaged over the S samples, and
 *   dK2[a][b] = || meanK_a - meanK_b ||^2,  dV2 likewise,  D[a][b] = sqrt(dK2 + dV2)
 * i.e. the Euclidean distance between the flattened [mean K ; mean V] vectors.  Outputs are
 * device fp32 [L][L], symmetric with a zero diagonal; dK2 and dV2 are returned so that other
 * readings of the paper's separate averaging of keys and values can be formed by the caller.
 * Supported: L <= 128.  workspace >= kvs_distance_workspace_bytes(L).
 */
int kvs_layer_distance(const void* kv_samples, int S, int L, size_t N, int dtype,
                       float* dK2, float* dV2, float* D,
                       void* workspace, size_t workspace_bytes, void* stream);

size_t kvs_distance_workspace_bytes(int L);

/* ---------------------------------------------------------------- similarity test */

/*
 * Representation similarity of Algorithm 1 ("Avg_Cos_Sim") and Sec. 3.1.2: hidden_shared and
 * hidden_original are the last-layer hidden states of the model with the candidate strategy
 * and of the original model on the calibration set, device [S][N] of `dtype` (S sentences of
 * equal length, N = tokens x hidden size, flattened).  *similarity (device, one float):
 *   mode 0: cosine similarity of the two sentence-averaged vectors (the text of Sec. 3.1.2:
 *           the representations are averaged over the sentences first, then one cosine);
 *   mode 1: average over the sentences of the per-sentence cosine (the procedure's name).
 * A zero vector contributes a cosine of 0.  The caller compares the result with the
 * threshold T inside its kvs_accept_fn (keep the pair iff similarity > T).
 * workspace: device, >= kvs_cos_sim_workspace_bytes(S), zero-filled once by the caller (it starts
 * with an arrival counter that every call leaves at zero, followed by partial sums); calls that
 * share it must not overlap in time.  One kernel launch.
 */
int kvs_avg_cos_sim(const void* hidden_shared, const void* hidden_original, int S, size_t N,
                    int dtype, int mode, float* similarity,
                    void* workspace, size_t workspace_bytes, void* stream);

size_t kvs_cos_sim_workspace_bytes(int S);

#ifdef __cplusplus
}
#endif
#endif /* KVS_H */
