/*
 * CPU oracle for layer-shared-KV attention and the layer-dissimilarity matrix.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what the
 * GPU library must compute.  It shares no code with the GPU library and nothing in the
 * product path may call it; only the tests, the smoke check and the benchmark's CPU
 * baseline leg do.
 *
 * What it states:
 *   - Inference with a sharing strategy (paper Sec. 3.2 and the caption of the
 *     prefill/generation figure): a layer whose KV cache is replaced takes the cache of
 *     the donor layer the strategy names; everything after that is the host model's
 *     ordinary attention.  The ordinary attention is written out as its textbook
 *     definition: z_j = q.k_j / sqrt(d), p = softmax(z), out = sum_j p_j v_j, with
 *     grouped-query head mapping g = h / (Hq / Hkv).
 *   - The layer representation and distance of the strategy search (paper Sec. 3.1.2,
 *     "KV Cache Similarity Calculation", and Algorithm 1): per layer the
 *     keys and the values are averaged over the calibration samples, flattened, and the
 *     Euclidean distance between two layers is taken over the concatenated
 *     [mean K ; mean V] vector.
 *
 * All arithmetic is double precision.  Stored elements are either fp32 or bf16 bit
 * patterns; both convert to double exactly.  OpenMP spreads independent output rows
 * over host threads; there is no blocking, fusion or reordering of the sums.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };

/* A bf16 value is the upper 16 bits of the IEEE-754 binary32 with the same value. */
static double elem(const void* base, int64_t idx, int dtype)
{
    if (dtype == ORC_F32) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Where token j of sequence b lives in a layer's cache, as an element offset of the
 * (token, kv-head 0, channel 0) element.
 *   block_table == NULL : contiguous cache  [B][T_cap][Hkv][d]
 *   block_table != NULL : paged cache       [num_blocks][block_tokens][Hkv][d],
 *                         token j is row j % block_tokens of block
 *                         block_table[b][j / block_tokens].
 */
static int64_t token_offset(int b, int64_t j, int64_t T_cap, int Hkv, int d,
                            const int32_t* block_table, int max_blocks_per_seq,
                            int block_tokens)
{
    if (!block_table) return ((int64_t)b * T_cap + j) * Hkv * d;
    int64_t blk = block_table[(int64_t)b * max_blocks_per_seq + j / block_tokens];
    return (blk * block_tokens + j % block_tokens) * (int64_t)Hkv * d;
}

/* One query row against keys 0..n-1 of kv-head g of sequence b. */
static void attend_row(const void* q, int64_t q_off, int q_dtype,
                       const void* K, const void* V, int kv_dtype,
                       int b, int g, int64_t n, int64_t T_cap, int Hkv, int d,
                       const int32_t* block_table, int max_blocks_per_seq, int block_tokens,
                       double* z /* scratch, >= n */, double* out /* d */,
                       double* probs /* NULL or >= n */)
{
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    if (n <= 0) return;                       /* empty cache: the row is defined as zero */
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    double zmax = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        int64_t off = token_offset(b, j, T_cap, Hkv, d, block_table, max_blocks_per_seq,
                                   block_tokens) + (int64_t)g * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += elem(q, q_off + c, q_dtype) * elem(K, off + c, kv_dtype);
        z[j] = dot * inv_sqrt_d;
        if (z[j] > zmax) zmax = z[j];
    }
    double denom = 0.0;
    for (int64_t j = 0; j < n; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
    for (int64_t j = 0; j < n; ++j) {
        double p = z[j] / denom;
        if (probs) probs[j] = p;
        int64_t off = token_offset(b, j, T_cap, Hkv, d, block_table, max_blocks_per_seq,
                                   block_tokens) + (int64_t)g * d;
        for (int c = 0; c < d; ++c) out[c] += p * elem(V, off + c, kv_dtype);
    }
}

/*
 * Attention of `layer` for T_new query rows per sequence under sharing strategy
 * `share_map` (share_map[l] = the layer whose cache layer l reads; l itself when l is
 * not replaced).  K_layers/V_layers hold one cache pointer per layer; entries of
 * replaced layers are never dereferenced and may be NULL.
 *
 *   q         [B][T_new][Hq][d]
 *   out       [B][T_new][Hq][d] (double)
 *   n_keys    query row i of sequence b sees keys 0 .. start_pos[b] + i  (causal).
 *             A decode step is T_new = 1 with start_pos[b] = seq_lens[b] - 1.
 *   probs     NULL, or [B][T_new][Hq][T_cap]: the softmax weights (zero past n_keys).
 * Returns 0, or -1 on an inconsistent argument.
 */
int orc_shared_attention(int layer, const int32_t* share_map, int L,
                         const void* const* K_layers, const void* const* V_layers, int kv_dtype,
                         const int32_t* block_table, int max_blocks_per_seq, int block_tokens,
                         int64_t T_cap,
                         const void* q, int q_dtype, const int32_t* start_pos,
                         int B, int T_new, int Hq, int Hkv, int d,
                         double* out, double* probs)
{
    if (layer < 0 || layer >= L || Hkv <= 0 || Hq % Hkv != 0) return -1;
    const int donor = share_map[layer];
    if (donor < 0 || donor >= L) return -1;
    const void* K = K_layers[donor];
    const void* V = V_layers[donor];
    if (!K || !V) return -1;
    const int group = Hq / Hkv;
    int bad = 0;

#pragma omp parallel
    {
        double* z = (double*)malloc(sizeof(double) * (size_t)(T_cap > 0 ? T_cap : 1));
#pragma omp for collapse(3) schedule(dynamic, 1)
        for (int b = 0; b < B; ++b)
            for (int i = 0; i < T_new; ++i)
                for (int h = 0; h < Hq; ++h) {
                    int64_t n = (int64_t)start_pos[b] + i + 1;
                    if (n < 0) n = 0;
                    if (n > T_cap) {
#pragma omp atomic write
                        bad = 1;
                        continue;
                    }
                    int64_t row = (((int64_t)b * T_new + i) * Hq + h);
                    double* pr = probs ? probs + row * T_cap : NULL;
                    if (pr) for (int64_t j = 0; j < T_cap; ++j) pr[j] = 0.0;
                    attend_row(q, row * d, q_dtype, K, V, kv_dtype, b, h / group, n, T_cap,
                               Hkv, d, block_table, max_blocks_per_seq, block_tokens,
                               z, out + row * d, pr);
                }
        free(z);
    }
    return bad ? -1 : 0;
}

/*
 * Layer dissimilarity (paper Sec. 3.1.2 / Algorithm 1).
 *   kv   [S][L][2][N]   calibration caches: sample, layer, (0 = keys, 1 = values),
 *                       flattened [Hkv][T][d] index
 *   dK2, dV2, D  [L][L] (double):  dK2[a][b] = || meanK_a - meanK_b ||^2, dV2 likewise,
 *                       D = sqrt(dK2 + dV2)
 */
int orc_layer_distance(const void* kv, int dtype, int S, int L, int64_t N,
                       double* dK2, double* dV2, double* D)
{
    if (S <= 0 || L <= 0 || N <= 0) return -1;
    double* mean = (double*)malloc(sizeof(double) * (size_t)L * 2 * (size_t)N);
    if (!mean) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < (int64_t)L * 2; ++r) {
        double* m = mean + r * N;
        for (int64_t i = 0; i < N; ++i) {
            double acc = 0.0;
            for (int s = 0; s < S; ++s) acc += elem(kv, ((int64_t)s * L * 2 + r) * N + i, dtype);
            m[i] = acc / (double)S;
        }
    }
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int a = 0; a < L; ++a)
        for (int b = 0; b < L; ++b) {
            double sk = 0.0, sv = 0.0;
            const double* ka = mean + ((int64_t)a * 2 + 0) * N;
            const double* kb = mean + ((int64_t)b * 2 + 0) * N;
            const double* va = mean + ((int64_t)a * 2 + 1) * N;
            const double* vb = mean + ((int64_t)b * 2 + 1) * N;
            for (int64_t i = 0; i < N; ++i) {
                double dk = ka[i] - kb[i];
                double dv = va[i] - vb[i];
                sk += dk * dk;
                sv += dv * dv;
            }
            dK2[(int64_t)a * L + b] = sk;
            dV2[(int64_t)a * L + b] = sv;
            D[(int64_t)a * L + b] = sqrt(sk + sv);
        }
    free(mean);
    return 0;
}
