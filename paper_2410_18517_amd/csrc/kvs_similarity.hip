// Similarity test of the strategy search (paper Sec. 3.1.2 and Algorithm 1, "Avg_Cos_Sim"): the
// last-layer hidden states of the model with the candidate sharing strategy and of the
// original model, one flattened vector per calibration sentence, are compared by cosine
// similarity.  Two readings are offered: the cosine of the sentence-averaged vectors (the
// text of Sec. 3.1.2) and the average over sentences of the per-sentence cosine (the
// procedure's name).  Both are one streaming pass: per "row" (the averaged vector, or each
// sentence) three sums  <a,b>, <a,a>, <b,b>  are reduced per workgroup, and a second tiny kernel
// adds the workgroup sums in double and forms the cosine(s).
#include <hip/hip_runtime.h>

#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxWorkgroupsPerRow = 256;

__device__ __forceinline__ float load_elem(const void* p, size_t i, bool bf16)
{
    if (bf16) return __uint_as_float((unsigned)static_cast<const unsigned short*>(p)[i] << 16);
    return static_cast<const float*>(p)[i];
}

// rows x inner: mode "mean first" = 1 row whose element i is the mean over `inner` sentences;
// mode "per sentence" = S rows with inner = 1.
__global__ __launch_bounds__(kThreads) void cos_partial_kernel(const void* a, const void* b, int inner, size_t N,
                                                               int bf16, float* partial)
{
    const int row = blockIdx.y;
    const size_t base = (size_t)row * (inner == 1 ? N : 0);
    const float inv = 1.f / (float)inner;
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < N; i += (size_t)gridDim.x * kThreads) {
        float xa = 0.f, xb = 0.f;
        for (int s = 0; s < inner; ++s) {
            xa += load_elem(a, base + (size_t)s * N + i, bf16);
            xb += load_elem(b, base + (size_t)s * N + i, bf16);
        }
        xa *= inv;
        xb *= inv;
        dot = fmaf(xa, xb, dot);
        na = fmaf(xa, xa, na);
        nb = fmaf(xb, xb, nb);
    }
    __shared__ float red[3][kThreads / 64];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        dot += __shfl_xor(dot, o);
        na += __shfl_xor(na, o);
        nb += __shfl_xor(nb, o);
    }
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = dot;
        red[1][threadIdx.x >> 6] = na;
        red[2][threadIdx.x >> 6] = nb;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        float s = 0.f;
        for (int w = 0; w < kThreads / 64; ++w) s += red[threadIdx.x][w];
        partial[((size_t)row * gridDim.x + blockIdx.x) * 3 + threadIdx.x] = s;
    }
}

__global__ __launch_bounds__(64) void cos_final_kernel(const float* partial, int rows, int n_wg, float* out)
{
    double acc = 0.0;
    for (int r = threadIdx.x; r < rows; r += 64) {
        double dot = 0.0, na = 0.0, nb = 0.0;
        for (int w = 0; w < n_wg; ++w) {
            const float* p = partial + ((size_t)r * n_wg + w) * 3;
            dot += p[0];
            na += p[1];
            nb += p[2];
        }
        acc += (na > 0.0 && nb > 0.0) ? dot / sqrt(na * nb) : 0.0;   // a zero vector has no direction
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (threadIdx.x == 0) out[0] = (float)(acc / rows);
}

int workgroups_per_row(size_t N)
{
    const size_t want = (N + kThreads * 8 - 1) / (kThreads * 8);
    return (int)(want < 1 ? 1 : (want > kMaxWorkgroupsPerRow ? kMaxWorkgroupsPerRow : want));
}

}  // namespace

size_t cos_sim_workspace_bytes(int S)
{
    return (size_t)S * kMaxWorkgroupsPerRow * 3 * sizeof(float);
}

int launch_cos_sim(const void* a, const void* b, int S, size_t N, int dtype, int mode, float* out, void* workspace,
                   void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* partial = static_cast<float*>(workspace);
    const int n_wg = workgroups_per_row(N);
    const int rows = mode == 0 ? 1 : S;
    const int inner = mode == 0 ? S : 1;
    hipLaunchKernelGGL(cos_partial_kernel, dim3(n_wg, rows), dim3(kThreads), 0, s, a, b, inner, N, dtype == 1, partial);
    if (hipError_t e = hipGetLastError()) return (int)e;
    hipLaunchKernelGGL(cos_final_kernel, dim3(1), dim3(64), 0, s, partial, rows, n_wg, out);
    return (int)hipGetLastError();
}

}  // namespace kvs
