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

// Positions per chunk: L * chunk * 4 B of LDS hold the chunk's means.  256 up to 64 layers; beyond
// that (up to 128 layers) 128, so that the means still fit 64 KiB.
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxWorkgroups = 2048;  // even; half visit key chunks, half value chunks
constexpr int kAccPerThread = 16;     // a 4 x 4 block of layer pairs
constexpr int kMaxLayers = 128;
constexpr int kLoadsInFlight = 8;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// LDS index of (layer l, position e): rows are rotated by l so that threads reading the same
// position of different layers fall on different banks.
template <int kChunk>
__device__ __forceinline__ int mean_index(int l, int e) { return l * kChunk + ((e + l) & (kChunk - 1)); }

// Sum over the samples of 8 consecutive bf16 positions (sum[0..7]); the lanes of a wavefront form
// kRows groups (2 at 256 positions per chunk: lanes 0-31 and 32-63), group r takes the samples
// r, r + kRows, ..., so one load instruction covers kRows rows of the chunk.
template <int kRows>
__device__ __forceinline__ void sum_samples_bf16(const unsigned short* row0, size_t stride, int S, int half,
                                                 float* sum)
{
    for (int s0 = half; s0 < S; s0 += kRows * kLoadsInFlight) {
        u32x4 w[kLoadsInFlight];
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u) {
            const int s = s0 + kRows * u;
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

// Same for fp32 input: 4 consecutive positions per lane, kRows groups of lanes (1 at 256 positions).
template <int kRows>
__device__ __forceinline__ void sum_samples_f32(const float* row0, size_t stride, int S, int first, float* sum)
{
    for (int s0 = first; s0 < S; s0 += kRows * kLoadsInFlight) {
        f32x4 w[kLoadsInFlight];
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u) {
            const int s = s0 + kRows * u;
            w[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (s < S) w[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row0 + (size_t)s * stride));
        }
#pragma unroll
        for (int u = 0; u < kLoadsInFlight; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) sum[i] += w[u][i];
    }
}

// kPer: pair blocks per thread: 1 while the 4 x 4 blocks of the upper triangle number at most
// kThreads (up to 124 layers), 2 beyond.
template <bool kBf16, int kChunk, int kPer>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4)))
void distance_partial_kernel(const void* kv, int S, int L, size_t N,
                                                                    int chunks_per_wg, float* partial)
{
    extern __shared__ float lds[];                      // means [L][kChunk] (rotated rows); reused at the end
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int part = blockIdx.x & 1;                    // 0 = keys, 1 = values
    const int wg = blockIdx.x >> 1;
    const size_t n_chunks = (N + kChunk - 1) / kChunk;

    // pair blocks: upper-triangular 4 x 4 tiles of the L x L matrix; with one block per thread,
    // several position phases each
    const int T = (L + 3) / 4;
    const int n_blk = T * (T + 1) / 2;
    const int phases = kPer == 1 ? kThreads / n_blk : 1;
    const int phase = kPer == 1 ? threadIdx.x / n_blk : 0;
    int bi[kPer], bj[kPer];
    bool has[kPer];
#pragma unroll
    for (int p = 0; p < kPer; ++p) {
        const int blk = kPer == 1 ? threadIdx.x % n_blk : threadIdx.x + p * kThreads;
        has[p] = blk < n_blk && phase < phases;
        int i = 0, rem = has[p] ? blk : 0;
        while (rem >= T - i) { rem -= T - i; ++i; }
        bi[p] = i;
        bj[p] = i + rem;
    }
    float acc[kPer][kAccPerThread];
#pragma unroll
    for (int p = 0; p < kPer; ++p)
#pragma unroll
        for (int i = 0; i < kAccPerThread; ++i) acc[p][i] = 0.f;

    const float inv_S = 1.f / (float)S;
    const size_t stride = (size_t)L * 2 * N;            // elements between samples
    size_t chunk = (size_t)wg * chunks_per_wg;
    const size_t chunk_end = chunk + chunks_per_wg < n_chunks ? chunk + chunks_per_wg : n_chunks;
    for (; chunk < chunk_end; ++chunk) {
        for (int l = wave; l < L; l += kWaves) {
            const size_t row = ((size_t)l * 2 + part) * N + chunk * kChunk;
            if (kBf16) {
                constexpr int kRowLanes = kChunk / 8, kRows = 64 / kRowLanes, kMine = 8 / kRows;
                const int half = lane / kRowLanes, pl = lane % kRowLanes;
                float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                if (chunk * kChunk + (size_t)pl * 8 < N)          // N % 8 == 0: all 8 positions or none
                    sum_samples_bf16<kRows>(static_cast<const unsigned short*>(kv) + row + pl * 8, stride, S, half, sum);
#pragma unroll
                for (int o = 32; o >= kRowLanes; o >>= 1)
#pragma unroll
                    for (int i = 0; i < 8; ++i) sum[i] += __shfl_xor(sum[i], o);
#pragma unroll
                for (int i = 0; i < kMine; ++i) {                 // each group of lanes stores its share of the 8 positions
                    float mine = sum[i];
#pragma unroll
                    for (int r = 1; r < kRows; ++r) mine = half == r ? sum[r * kMine + i] : mine;
                    lds[mean_index<kChunk>(l, pl * 8 + half * kMine + i)] = mine * inv_S;
                }
            } else {
                constexpr int kRowLanes = kChunk / 4, kRows = 64 / kRowLanes, kMine = 4 / kRows;
                const int half = lane / kRowLanes, pl = lane % kRowLanes;
                float sum[4] = {0.f, 0.f, 0.f, 0.f};
                if (chunk * kChunk + (size_t)pl * 4 < N)
                    sum_samples_f32<kRows>(static_cast<const float*>(kv) + row + pl * 4, stride, S, half, sum);
#pragma unroll
                for (int o = 32; o >= kRowLanes; o >>= 1)
#pragma unroll
                    for (int i = 0; i < 4; ++i) sum[i] += __shfl_xor(sum[i], o);
#pragma unroll
                for (int i = 0; i < kMine; ++i) {
                    float mine = sum[i];
#pragma unroll
                    for (int r = 1; r < kRows; ++r) mine = half == r ? sum[r * kMine + i] : mine;
                    lds[mean_index<kChunk>(l, pl * 4 + half * kMine + i)] = mine * inv_S;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < kPer; ++p) {
            if (!has[p]) continue;
            for (int e = phase; e < kChunk; e += phases) {
                float x[4], y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int la = bi[p] * 4 + r, lb = bj[p] * 4 + r;
                    x[r] = la < L ? lds[mean_index<kChunk>(la, e)] : 0.f;
                    y[r] = lb < L ? lds[mean_index<kChunk>(lb, e)] : 0.f;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float d = x[r] - y[c];
                        acc[p][r * 4 + c] = fmaf(d, d, acc[p][r * 4 + c]);
                    }
            }
        }
        __syncthreads();
    }
    // fold the position phases of each pair block, then one record per block and workgroup
    float* red = lds;                                   // [kPer][kThreads][16]
#pragma unroll
    for (int p = 0; p < kPer; ++p)
#pragma unroll
        for (int i = 0; i < kAccPerThread; ++i) red[(p * kThreads + threadIdx.x) * kAccPerThread + i] = acc[p][i];
    __syncthreads();
    for (int idx = threadIdx.x; idx < n_blk * kAccPerThread; idx += kThreads) {
        const int b = idx / kAccPerThread, i = idx % kAccPerThread;
        float s = 0.f;
        if (kPer == 1) {
            for (int ph = 0; ph < phases; ++ph) s += red[(ph * n_blk + b) * kAccPerThread + i];
        } else {
            s = red[b * kAccPerThread + i];             // block b sits at thread b % kThreads of pass b / kThreads
        }
        partial[(size_t)blockIdx.x * n_blk * kAccPerThread + idx] = s;
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
    const int n_blk = T * (T + 1) / 2;
    const int bi = lo / 4, bj = hi / 4;
    const int blk = bi * T - bi * (bi - 1) / 2 + (bj - bi);
    const int slot = (lo % 4) * 4 + (hi % 4);
    double sum[2] = {0.0, 0.0};
    for (int w = threadIdx.x; w < n_workgroups; w += 64)
        sum[w & 1] += (double)partial[((size_t)w * n_blk + blk) * kAccPerThread + slot];
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

int chunk_for(int L) { return L <= 64 ? 256 : 128; }

int blocks_for(int L)
{
    const int T = (L + 3) / 4;
    return T * (T + 1) / 2;
}

size_t lds_bytes(int L)
{
    const size_t means = (size_t)L * chunk_for(L) * sizeof(float);
    const size_t fold = (size_t)(blocks_for(L) <= kThreads ? 1 : 2) * kThreads * kAccPerThread * sizeof(float);
    return means > fold ? means : fold;
}

// Persistent grid: as many workgroups as are resident on the chip at once (asked of the
// runtime, since registers, LDS and wave slots all limit it), half of them on key chunks and
// half on value chunks, each with the same number of consecutive chunks.
template <typename Kernel>
void grid_for(Kernel kernel, size_t N, int L, int* n_wg, int* chunks_per_wg)
{
    const size_t n_chunks = (N + chunk_for(L) - 1) / chunk_for(L);
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, lds_bytes(L)) != hipSuccess || per_cu < 1)
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

template <bool kBf16, int kChunk, int kPer>
int launch_partial(const void* kv, int S, int L, size_t N, float* partial, int* n_wg, hipStream_t s)
{
    int chunks_per_wg;
    grid_for(distance_partial_kernel<kBf16, kChunk, kPer>, N, L, n_wg, &chunks_per_wg);
    hipLaunchKernelGGL((distance_partial_kernel<kBf16, kChunk, kPer>), dim3(*n_wg), dim3(kThreads), lds_bytes(L), s, kv, S,
                       L, N, chunks_per_wg, partial);
    return (int)hipGetLastError();
}

}  // namespace

size_t distance_workspace_bytes(int L)
{
    return (size_t)kMaxWorkgroups * blocks_for(L) * kAccPerThread * sizeof(float);
}

int launch_layer_distance(const void* kv, int S, int L, size_t N, int dtype, float* dK2, float* dV2, float* D,
                          void* workspace, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* partial = static_cast<float*>(workspace);
    static_assert(kMaxLayers == 128, "two pair blocks per thread cover the 528 blocks of 128 layers");
    int n_wg = 0, e;
    if (L <= 64) e = dtype == 1 ? launch_partial<true, 256, 1>(kv, S, L, N, partial, &n_wg, s)
                                : launch_partial<false, 256, 1>(kv, S, L, N, partial, &n_wg, s);
    else if (blocks_for(L) <= kThreads)          // up to 124 layers: still one pair block per thread
        e = dtype == 1 ? launch_partial<true, 128, 1>(kv, S, L, N, partial, &n_wg, s)
                       : launch_partial<false, 128, 1>(kv, S, L, N, partial, &n_wg, s);
    else e = dtype == 1 ? launch_partial<true, 128, 2>(kv, S, L, N, partial, &n_wg, s)
                        : launch_partial<false, 128, 2>(kv, S, L, N, partial, &n_wg, s);
    if (e) return e;
    hipLaunchKernelGGL(distance_final_kernel, dim3(L * L), dim3(64), 0, s, partial, n_wg, L, dK2, dV2, D);
    return (int)hipGetLastError();
}

}  // namespace kvs
