// Layer-dissimilarity matrix of the strategy search (paper Sec. 3.1.2, Algorithm 1 first
// step) on gfx950: per layer, keys and values are averaged over the calibration samples and
// the squared Euclidean distance of every layer pair is accumulated, keys and values apart.
//
// One pass over the samples: a workgroup takes a chunk of kChunk consecutive positions of the
// flattened index of either the keys or the values, averages all L layers over the S samples
// into LDS (fp32), and adds the chunk's (mean_a - mean_b)^2 to register accumulators that live
// across all the chunks the workgroup visits.  Per-workgroup sums go to the workspace; a
// second, tiny kernel adds them in double and writes dK2, dV2 and D = sqrt(dK2 + dV2).
#include <hip/hip_runtime.h>

#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kChunk = 256;           // positions per chunk; L * kChunk * 4 B of LDS
constexpr int kThreads = 256;
constexpr int kMaxWorkgroups = 1536;  // even; half visit key chunks, half value chunks
constexpr int kAccPerThread = 16;     // a 4 x 4 block of layer pairs

// LDS index of (layer l, position e): rows are rotated by l so that threads reading the same
// position of different layers fall on different banks.
__device__ __forceinline__ int mean_index(int l, int e) { return l * kChunk + ((e + l) & (kChunk - 1)); }

template <bool kBf16>
__global__ __launch_bounds__(kThreads) void distance_partial_kernel(const void* kv, int S, int L, size_t N,
                                                                    float* partial)
{
    extern __shared__ float mean[];                     // [L][kChunk], rotated rows
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int part = blockIdx.x & 1;                    // 0 = keys, 1 = values
    const int wg = blockIdx.x >> 1, n_wg = gridDim.x >> 1;
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
    for (size_t chunk = wg; chunk < n_chunks; chunk += n_wg) {
        const size_t e0 = chunk * kChunk + (size_t)lane * 4;
        const bool in_range = e0 < N;                    // N % 8 == 0: a lane's 4 positions share it
        for (int l = wave; l < L; l += 4) {
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            if (in_range) {
                const size_t stride = (size_t)L * 2 * N;
                const size_t off = ((size_t)l * 2 + part) * N + e0;
                if (kBf16) {
                    const unsigned short* p = static_cast<const unsigned short*>(kv) + off;
#pragma unroll 6
                    for (int s = 0; s < S; ++s) {
                        const uint2 w = *reinterpret_cast<const uint2*>(p + (size_t)s * stride);
                        s0 += __uint_as_float(w.x << 16);
                        s1 += __uint_as_float(w.x & 0xffff0000u);
                        s2 += __uint_as_float(w.y << 16);
                        s3 += __uint_as_float(w.y & 0xffff0000u);
                    }
                } else {
                    const float* p = static_cast<const float*>(kv) + off;
#pragma unroll 6
                    for (int s = 0; s < S; ++s) {
                        const float4 w = *reinterpret_cast<const float4*>(p + (size_t)s * stride);
                        s0 += w.x; s1 += w.y; s2 += w.z; s3 += w.w;
                    }
                }
            }
            mean[mean_index(l, lane * 4 + 0)] = s0 * inv_S;
            mean[mean_index(l, lane * 4 + 1)] = s1 * inv_S;
            mean[mean_index(l, lane * 4 + 2)] = s2 * inv_S;
            mean[mean_index(l, lane * 4 + 3)] = s3 * inv_S;
        }
        __syncthreads();
        if (phase < phases) {
            for (int e = phase; e < kChunk; e += phases) {
                float x[4], y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int la = bi * 4 + r, lb = bj * 4 + r;
                    x[r] = la < L ? mean[mean_index(la, e)] : 0.f;
                    y[r] = lb < L ? mean[mean_index(lb, e)] : 0.f;
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
    float* out = partial + ((size_t)blockIdx.x * kThreads + threadIdx.x) * kAccPerThread;
#pragma unroll
    for (int i = 0; i < kAccPerThread; i += 4)
        *reinterpret_cast<float4*>(out + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
}

// One wavefront per ordered layer pair: add the partial sums of every workgroup and phase.
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
    const int phases = kThreads / n_blk;
    const int bi = lo / 4, bj = hi / 4;
    const int blk = bi * T - bi * (bi - 1) / 2 + (bj - bi);
    const int slot = (lo % 4) * 4 + (hi % 4);
    double sum[2] = {0.0, 0.0};
    for (int i = threadIdx.x; i < n_workgroups * phases; i += 64) {
        const int w = i / phases, ph = i % phases;
        sum[w & 1] += (double)partial[((size_t)w * kThreads + ph * n_blk + blk) * kAccPerThread + slot];
    }
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

// Persistent grid: as many workgroups as fit on the chip at once (LDS-limited), half of them
// on key chunks and half on value chunks.
int workgroups_for(size_t N, int L)
{
    const size_t n_chunks = (N + kChunk - 1) / kChunk;
    const size_t lds = (size_t)L * kChunk * sizeof(float);
    size_t per_cu = (160 * 1024) / lds;
    per_cu = per_cu < 1 ? 1 : (per_cu > 6 ? 6 : per_cu);
    size_t per_part = 256 * per_cu / 2;
    if (per_part > n_chunks) per_part = n_chunks;
    if (per_part > kMaxWorkgroups / 2) per_part = kMaxWorkgroups / 2;
    return (int)per_part * 2;
}

}  // namespace

size_t distance_workspace_bytes(int L)
{
    (void)L;
    return (size_t)kMaxWorkgroups * kThreads * kAccPerThread * sizeof(float);
}

int launch_layer_distance(const void* kv, int S, int L, size_t N, int dtype, float* dK2, float* dV2, float* D,
                          void* workspace, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* partial = static_cast<float*>(workspace);
    const int n_wg = workgroups_for(N, L);
    const size_t lds = (size_t)L * kChunk * sizeof(float);
    if (dtype == 1)
        hipLaunchKernelGGL(distance_partial_kernel<true>, dim3(n_wg), dim3(kThreads), lds, s, kv, S, L, N, partial);
    else
        hipLaunchKernelGGL(distance_partial_kernel<false>, dim3(n_wg), dim3(kThreads), lds, s, kv, S, L, N, partial);
    if (hipError_t e = hipGetLastError()) return (int)e;
    hipLaunchKernelGGL(distance_final_kernel, dim3(L * L), dim3(64), 0, s, partial, n_wg, L, dK2,
                       dV2, D);
    return (int)hipGetLastError();
}

}  // namespace kvs
