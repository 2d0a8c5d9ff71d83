// Layer-dissimilarity matrix of the strategy search (paper Sec. 3.1.2, Algorithm 1) on
// gfx950: per layer, keys and values are averaged over the calibration samples and
// the squared Euclidean distance of every layer pair is accumulated, keys and values apart.
//
// One pass over the samples: a workgroup takes chunks of kChunk consecutive positions of the
// flattened index of either the keys or the values, averages all L layers over the S samples
// into LDS (fp32), and adds the chunk's (mean_a - mean_b)^2 to register accumulators that live
// across all the chunks the workgroup visits.  Per-workgroup sums go to the workspace; a
// second, tiny kernel adds them in double and writes dK2, dV2 and D = sqrt(dK2 + dV2).
#include <hip/hip_runtime.h>

#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kChunk = 256;           // positions per chunk; L * kChunk * 4 B of LDS
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxWorkgroups = 2048;  // even; half visit key chunks, half value chunks
constexpr int kAccPerThread = 16;     // a 4 x 4 block of layer pairs
constexpr int kMaxBlocks = 136;       // 4 x 4 blocks in the upper triangle at L = 64
constexpr int kLoadsInFlight = 8;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// LDS index of (layer l, position e): rows are rotated by l so that threads reading the same
// position of different layers fall on different banks.
__device__ __forceinline__ int mean_index(int l, int e) { return l * kChunk + ((e + l) & (kChunk - 1)); }

// Sum over the samples of 8 consecutive bf16 positions (sum[0..7]); lanes 0-31 take the even
// samples and lanes 32-63 the odd ones, so one load instruction covers two 512-byte rows.
__device__ __forceinline__ void sum_samples_bf16(const unsigned short* row0, size_t stride, int S, int half,
                                                 float* sum)
{
    for (int s0 = half; s0 < S; s0 += 2 * kLoadsInFlight) {
        u32x4 w[kLoadsInFlight];
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u) {
            const int s = s0 + 2 * u;
            w[u] = u32x4{0u, 0u, 0u, 0u};
            if (s < S) w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row0 + (size_t)s * stride));
        }
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sum[2 * i] += __uint_as_float(w[u][i] << 16);
                sum[2 * i + 1] += __uint_as_float(w[u][i] & 0xffff0000u);
            }
    }
}

// Same for fp32 input: 4 consecutive positions per lane, every lane takes every sample.
__device__ __forceinline__ void sum_samples_f32(const float* row0, size_t stride, int S, float* sum)
{
    for (int s0 = 0; s0 < S; s0 += kLoadsInFlight) {
        f32x4 w[kLoadsInFlight];
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u) {
            const int s = s0 + u;
            w[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (s < S) w[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row0 + (size_t)s * stride));
        }
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) sum[i] += w[u][i];
    }
}

template <bool kBf16>
__global__ __launch_bounds__(kThreads) void distance_partial_kernel(const void* kv, int S, int L, size_t N,
                                                                    int chunks_per_wg, float* partial)
{
    extern __shared__ float lds[];                      // means [L][kChunk] (rotated rows); reused at the end
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int part = blockIdx.x & 1;                    // 0 = keys, 1 = values
    const int wg = blockIdx.x >> 1;
    const size_t n_chunks = (N + kChunk - 1) / kChunk;

    // pair blocks: upper-triangular 4 x 4 tiles of the L x L matrix, several position phases each
    const int T = (L + 3) / 4;
    const int n_blk = T * (T + 1) / 2;
    const int phases = kThreads / n_blk;
    const int blk = threadIdx.x % n_blk;
    const int phase = threadIdx.x / n_blk;
    int bi = 0, rem = blk;
    while (rem >= T - bi) { rem -= T - bi; ++bi; }
    const int bj = bi + rem;
    float acc[kAccPerThread];
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) acc[i] = 0.f;

    const float inv_S = 1.f / (float)S;
    const size_t stride = (size_t)L * 2 * N;            // elements between samples
    size_t chunk = (size_t)wg * chunks_per_wg;
    const size_t chunk_end = chunk + chunks_per_wg < n_chunks ? chunk + chunks_per_wg : n_chunks;
    for (; chunk < chunk_end; ++chunk) {
        for (int l = wave; l < L; l += kWaves) {
            const size_t row = ((size_t)l * 2 + part) * N + chunk * kChunk;
            if (kBf16) {
                const int half = lane >> 5, pl = lane & 31;
                float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                if (chunk * kChunk + (size_t)pl * 8 < N)          // N % 8 == 0: all 8 positions or none
                    sum_samples_bf16(static_cast<const unsigned short*>(kv) + row + pl * 8, stride, S, half, sum);
#pragma unroll
                for (int i = 0; i < 8; ++i) sum[i] += __shfl_xor(sum[i], 32);
#pragma unroll
                for (int i = 0; i < 4; ++i)                       // each half stores 4 of the 8 positions
                    lds[mean_index(l, pl * 8 + half * 4 + i)] = sum[half * 4 + i] * inv_S;
            } else {
                float sum[4] = {0.f, 0.f, 0.f, 0.f};
                if (chunk * kChunk + (size_t)lane * 4 < N)
                    sum_samples_f32(static_cast<const float*>(kv) + row + lane * 4, stride, S, sum);
#pragma unroll
                for (int i = 0; i < 4; ++i) lds[mean_index(l, lane * 4 + i)] = sum[i] * inv_S;
            }
        }
        __syncthreads();
        if (phase < phases) {
            for (int e = phase; e < kChunk; e += phases) {
                float x[4], y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int la = bi * 4 + r, lb = bj * 4 + r;
                    x[r] = la < L ? lds[mean_index(la, e)] : 0.f;
                    y[r] = lb < L ? lds[mean_index(lb, e)] : 0.f;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float d = x[r] - y[c];
                        acc[r * 4 + c] = fmaf(d, d, acc[r * 4 + c]);
                    }
            }
        }
        __syncthreads();
    }
    // fold the position phases of each pair block, then one record per block and workgroup
    float* red = lds;                                   // [kThreads][16]
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) red[threadIdx.x * kAccPerThread + i] = acc[i];
    __syncthreads();
    for (int idx = threadIdx.x; idx < n_blk * kAccPerThread; idx += kThreads) {
        const int b = idx / kAccPerThread, i = idx % kAccPerThread;
        float s = 0.f;
        for (int ph = 0; ph < phases; ++ph) s += red[(ph * n_blk + b) * kAccPerThread + i];
        partial[(size_t)blockIdx.x * kMaxBlocks * kAccPerThread + idx] = s;
    }
}

// One wavefront per ordered layer pair: add the partial sums of every workgroup.
__global__ __launch_bounds__(64) void distance_final_kernel(const float* partial, int n_workgroups, int L,
                                                            float* dK2, float* dV2, float* D)
{
    const int idx = blockIdx.x;
    const int a = idx / L, b = idx % L;
    if (a == b) {
        if (threadIdx.x == 0) { dK2[idx] = 0.f; dV2[idx] = 0.f; D[idx] = 0.f; }
        return;
    }
    const int lo = a < b ? a : b, hi = a < b ? b : a;
    const int T = (L + 3) / 4;
    const int bi = lo / 4, bj = hi / 4;
    const int blk = bi * T - bi * (bi - 1) / 2 + (bj - bi);
    const int slot = (lo % 4) * 4 + (hi % 4);
    double sum[2] = {0.0, 0.0};
    for (int w = threadIdx.x; w < n_workgroups; w += 64)
        sum[w & 1] += (double)partial[((size_t)w * kMaxBlocks + blk) * kAccPerThread + slot];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sum[0] += __shfl_xor(sum[0], o);
        sum[1] += __shfl_xor(sum[1], o);
    }
    if (threadIdx.x == 0) {
        dK2[idx] = (float)sum[0];
        dV2[idx] = (float)sum[1];
        D[idx] = (float)sqrt(sum[0] + sum[1]);
    }
}

size_t lds_bytes(int L)
{
    const size_t means = (size_t)L * kChunk * sizeof(float);
    const size_t fold = (size_t)kThreads * kAccPerThread * sizeof(float);
    return means > fold ? means : fold;
}

// Persistent grid: as many workgroups as are resident on the chip at once (asked of the
// runtime, since registers, LDS and wave slots all limit it), half of them on key chunks and
// half on value chunks, each with the same number of consecutive chunks.
template <bool kBf16>
void grid_for(size_t N, int L, int* n_wg, int* chunks_per_wg)
{
    const size_t n_chunks = (N + kChunk - 1) / kChunk;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, distance_partial_kernel<kBf16>, kThreads,
                                                     lds_bytes(L)) != hipSuccess || per_cu < 1)
        per_cu = 1;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    size_t per_part = (size_t)cus * per_cu / 2;
    if (per_part < 1) per_part = 1;
    if (per_part > kMaxWorkgroups / 2) per_part = kMaxWorkgroups / 2;
    if (per_part > n_chunks) per_part = n_chunks;
    const size_t k = (n_chunks + per_part - 1) / per_part;
    per_part = (n_chunks + k - 1) / k;
    *n_wg = (int)per_part * 2;
    *chunks_per_wg = (int)k;
}

}  // namespace

size_t distance_workspace_bytes(int L)
{
    (void)L;
    return (size_t)kMaxWorkgroups * kMaxBlocks * kAccPerThread * sizeof(float);
}

int launch_layer_distance(const void* kv, int S, int L, size_t N, int dtype, float* dK2, float* dV2, float* D,
                          void* workspace, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* partial = static_cast<float*>(workspace);
    int n_wg, chunks_per_wg;
    if (dtype == 1) grid_for<true>(N, L, &n_wg, &chunks_per_wg);
    else grid_for<false>(N, L, &n_wg, &chunks_per_wg);
    const size_t lds = lds_bytes(L);
    if (dtype == 1)
        hipLaunchKernelGGL(distance_partial_kernel<true>, dim3(n_wg), dim3(kThreads), lds, s, kv, S, L, N,
                           chunks_per_wg, partial);
    else
        hipLaunchKernelGGL(distance_partial_kernel<false>, dim3(n_wg), dim3(kThreads), lds, s, kv, S, L, N,
                           chunks_per_wg, partial);
    if (hipError_t e = hipGetLastError()) return (int)e;
    hipLaunchKernelGGL(distance_final_kernel, dim3(L * L), dim3(64), 0, s, partial, n_wg, L, dK2, dV2, D);
    return (int)hipGetLastError();
}

}  // namespace kvs
