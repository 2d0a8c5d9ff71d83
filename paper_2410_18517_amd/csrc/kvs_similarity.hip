// Similarity test of the strategy search (paper Sec. 3.1.2 and Algorithm 1, "Avg_Cos_Sim"): the
// last-layer hidden states of the model with the candidate sharing strategy and of the
// original model, one flattened vector per calibration sentence, are compared by cosine
// similarity.  Two readings are offered: the cosine of the sentence-averaged vectors (the
// text of Sec. 3.1.2) and the average over sentences of the per-sentence cosine (the
// procedure's name).
//
// One launch, one pass over the two inputs (roofline: HBM, 2 * S * N elements read once).  A
// "row" is the averaged vector (mean first: one row, every element the mean over the S sentences)
// or one sentence (per sentence: S rows).  A thread owns 16-byte pieces of the row: it streams the
// piece of every sentence that goes into the row, both inputs, with all those loads in flight at
// once, and keeps the three sums <a,b>, <a,a>, <b,b> of its elements.  The sums meet per wavefront,
// per workgroup and, through the workspace, per row: every workgroup publishes its three sums and
// the last one to arrive (a device counter, as the attention splits use) adds all of them in double
// in a fixed order and forms the cosine(s).  Nobody waits for anybody; the counter is left at zero.
#include <hip/hip_runtime.h>

#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr int kThreadsOneRow = 64;           // mean first: a piece per thread, so small workgroups to have enough of them
constexpr int kThreadsRows = 256;           // per sentence
constexpr int kMaxChunksPerRow = 1024;      // workgroups per row at most (their sums are added by one workgroup)
constexpr int kInFlightOneRow = 16;          // pieces of either input a thread requests before it adds any
constexpr int kInFlightRows = 8;
constexpr int kArrivalGroup = 16;           // workgroups per first-level arrival counter
constexpr int kMaxWorkgroups = 2048;        // workgroups of a launch with several rows, about
constexpr int kCounterLine = 32;            // ints per 128-byte line: every counter sits on a line of its own

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of a row as floats: 8 bf16 elements or 4 fp32 elements (the unused upper half stays zero)
template <bool kBf16>
__device__ __forceinline__ void widen(const u32x4 w, float (&x)[8])
{
    if constexpr (kBf16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[2 * e] = __uint_as_float(w[e] << 16);
            x[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = __uint_as_float(w[e]);
            x[4 + e] = 0.f;
        }
    }
}

// grid (chunks, rows).  inner: sentences averaged into a row (S for "mean first" with one row, 1 for
// "per sentence" with S rows).  workspace: int counter, then [rows][chunks][3] floats.
template <bool kBf16, int kThreads, int kInFlight>
__global__ __launch_bounds__(kThreads) void cos_sim_kernel(const void* a, const void* b, int inner, size_t N, int rows,
                                                           int* counter, float* partial, float* out)
{
    constexpr int kPer = kBf16 ? 8 : 4;                    // elements per 16-byte piece
    const int row = blockIdx.y, chunks = gridDim.x;
    const size_t row_base = inner == 1 ? (size_t)row * N : 0;
    const size_t pieces = N / kPer;                        // whole pieces of a row; the tail is handled element by element
    const u32x4* pa = reinterpret_cast<const u32x4*>(a);   // rows start at multiples of N elements: aligned when N % kPer == 0
    const u32x4* pb = reinterpret_cast<const u32x4*>(b);
    const bool aligned = N % kPer == 0 && ((reinterpret_cast<size_t>(a) | reinterpret_cast<size_t>(b)) & 15) == 0;
    const float inv = 1.f / (float)inner;
    float dot = 0.f, na = 0.f, nb = 0.f;
    if (aligned && inner > 1) {
        // mean first: a thread's piece of every sentence, kInFlight sentences of both inputs at a time
        for (size_t p = (size_t)blockIdx.x * kThreads + threadIdx.x; p < pieces; p += (size_t)chunks * kThreads) {
            float xa[8] = {0, 0, 0, 0, 0, 0, 0, 0}, xb[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int s0 = 0; s0 < inner; s0 += kInFlight) {
                u32x4 wa[kInFlight], wb[kInFlight];
#pragma unroll
                for (int u = 0; u < kInFlight; ++u) {
                    const bool in = s0 + u < inner;
                    const size_t at = ((size_t)(in ? s0 + u : s0) * N) / kPer + p;
                    wa[u] = __builtin_nontemporal_load(pa + at);        // read once: streamed past the caches
                    wb[u] = __builtin_nontemporal_load(pb + at);
                }
#pragma unroll
                for (int u = 0; u < kInFlight; ++u) {
                    if (s0 + u >= inner) continue;                      // (a repeated load of sentence s0: not added)
                    float ya[8], yb[8];
                    widen<kBf16>(wa[u], ya);
                    widen<kBf16>(wb[u], yb);
#pragma unroll
                    for (int e = 0; e < kPer; ++e) {
                        xa[e] += ya[e];
                        xb[e] += yb[e];
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < kPer; ++e) {
                const float ma = xa[e] * inv, mb = xb[e] * inv;
                dot = fmaf(ma, mb, dot);
                na = fmaf(ma, ma, na);
                nb = fmaf(mb, mb, nb);
            }
        }
    } else if (aligned) {
        // per sentence: kInFlight pieces of the row at a time
        const size_t stride = (size_t)chunks * kThreads;
        for (size_t p0 = (size_t)blockIdx.x * kThreads + threadIdx.x; p0 < pieces; p0 += stride * kInFlight) {
            u32x4 wa[kInFlight], wb[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const size_t p = p0 + u * stride;
                const size_t at = row_base / kPer + (p < pieces ? p : p0);
                wa[u] = __builtin_nontemporal_load(pa + at);
                wb[u] = __builtin_nontemporal_load(pb + at);
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                if (p0 + u * stride >= pieces) continue;
                float ya[8], yb[8];
                widen<kBf16>(wa[u], ya);
                widen<kBf16>(wb[u], yb);
#pragma unroll
                for (int e = 0; e < kPer; ++e) {
                    dot = fmaf(ya[e], yb[e], dot);
                    na = fmaf(ya[e], ya[e], na);
                    nb = fmaf(yb[e], yb[e], nb);
                }
            }
        }
    }
    // elements no 16-byte piece covers: the row's last N % kPer, or all of it when rows are not 16-byte aligned
    for (size_t i = (aligned ? pieces * kPer : 0) + (size_t)blockIdx.x * kThreads + threadIdx.x; i < N;
         i += (size_t)chunks * kThreads) {
        float ma = 0.f, mb = 0.f;
        for (int s = 0; s < inner; ++s) {
            const size_t at = row_base + (size_t)s * N + i;
            if constexpr (kBf16) {
                ma += __uint_as_float((unsigned)static_cast<const unsigned short*>(a)[at] << 16);
                mb += __uint_as_float((unsigned)static_cast<const unsigned short*>(b)[at] << 16);
            } else {
                ma += static_cast<const float*>(a)[at];
                mb += static_cast<const float*>(b)[at];
            }
        }
        ma *= inv;
        mb *= inv;
        dot = fmaf(ma, mb, dot);
        na = fmaf(ma, ma, na);
        nb = fmaf(mb, mb, nb);
    }

    __shared__ float red[3][kThreads / 64 > 0 ? kThreads / 64 : 1];
    __shared__ int s_is_last;
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
    // Publish this workgroup's sums with device-scope stores, wait until they are acknowledged, then
    // arrive; the workgroup that finds every other one arrived reads all sums with device-scope loads.
    if (threadIdx.x < 3) {
        float s = 0.f;
        for (int w = 0; w < kThreads / 64; ++w) s += red[threadIdx.x][w];
        __hip_atomic_store(partial + ((size_t)row * chunks + blockIdx.x) * 3 + threadIdx.x, s, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0)
    __syncthreads();
    // Arrival in two levels, so that no counter is bumped by more than a few workgroups at about the
    // same time (device-scope atomics on one address are served one after another): sixteen
    // workgroups share a first-level counter, and the last of each sixteen arrives at the launch's.
    if (threadIdx.x == 0) {
        const int total = chunks * rows;
        const int wg = row * chunks + blockIdx.x;
        const int grp = wg / kArrivalGroup, n_groups = (total + kArrivalGroup - 1) / kArrivalGroup;
        const int in_group = grp == n_groups - 1 ? total - grp * kArrivalGroup : kArrivalGroup;
        int* first = counter + (1 + grp) * kCounterLine;
        int last = atomicAdd(first, 1) == in_group - 1;
        if (last) {
            atomicExch(first, 0);                         // ready for the next call
            last = atomicAdd(counter, 1) == n_groups - 1;
            if (last) atomicExch(counter, 0);
        }
        s_is_last = last;
    }
    __syncthreads();
    if (!s_is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    // Everything in double and in a fixed order.  One row: the chunks in turn over the threads, the
    // threads' sums folded in thread order.  Several rows: the rows in turn over the threads, each
    // row's chunks in order, four triples requested at a time.
    auto triple = [&](int r, int w, double& d, double& xa, double& xb) {
        const float* p = partial + ((size_t)r * chunks + w) * 3;
        d += (double)__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        xa += (double)__hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        xb += (double)__hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    __shared__ double fold[3][kThreads];
    if (rows == 1) {
        double d = 0.0, xa = 0.0, xb = 0.0;
        for (int w = threadIdx.x; w < chunks; w += kThreads) triple(0, w, d, xa, xb);
        fold[0][threadIdx.x] = d;
        fold[1][threadIdx.x] = xa;
        fold[2][threadIdx.x] = xb;
        __syncthreads();
        if (threadIdx.x == 0) {
            d = xa = xb = 0.0;
            for (int t = 0; t < kThreads; ++t) {
                d += fold[0][t];
                xa += fold[1][t];
                xb += fold[2][t];
            }
            out[0] = (float)((xa > 0.0 && xb > 0.0) ? d / sqrt(xa * xb) : 0.0);   // a zero vector has no direction
        }
        return;
    }
    double acc = 0.0;
    for (int r = threadIdx.x; r < rows; r += kThreads) {
        double d = 0.0, xa = 0.0, xb = 0.0;
        int w = 0;
        for (; w + 4 <= chunks; w += 4) {
            double d4[4] = {0, 0, 0, 0}, a4[4] = {0, 0, 0, 0}, b4[4] = {0, 0, 0, 0};
#pragma unroll
            for (int u = 0; u < 4; ++u) triple(r, w + u, d4[u], a4[u], b4[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                d += d4[u];
                xa += a4[u];
                xb += b4[u];
            }
        }
        for (; w < chunks; ++w) triple(r, w, d, xa, xb);
        acc += (xa > 0.0 && xb > 0.0) ? d / sqrt(xa * xb) : 0.0;
    }
    fold[0][threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double sum = 0.0;
        for (int t = 0; t < kThreads; ++t) sum += fold[0][t];
        out[0] = (float)(sum / rows);
    }
}

// Workgroups per row: one 16-byte piece per thread (mean first; per sentence: kInFlightRows of them)
// while that gives at most kMaxChunksPerRow workgroups for one row, or about kMaxWorkgroups in all
// for several rows.
int chunks_per_row(size_t N, int rows, bool bf16)
{
    const size_t pieces = N / (bf16 ? 8 : 4) + 1;
    const size_t per_wg = rows == 1 ? (size_t)kThreadsOneRow : (size_t)kThreadsRows * kInFlightRows;
    size_t want = (pieces + per_wg - 1) / per_wg;
    const size_t cap = rows == 1 ? (size_t)kMaxChunksPerRow : (size_t)(kMaxWorkgroups / rows > 0 ? kMaxWorkgroups / rows : 1);
    want = want > cap ? cap : want;
    return (int)(want < 1 ? 1 : want);
}

// workgroups a launch can have: rows * chunks <= max(kMaxWorkgroups, rows), or kMaxChunksPerRow for one row
size_t max_workgroups(int S)
{
    return (size_t)(S > kMaxWorkgroups ? S : kMaxWorkgroups) + kMaxChunksPerRow;
}

}  // namespace

// a line per arrival counter (the launch's, then one per sixteen workgroups), then a triple of
// sums per (row, chunk)
size_t cos_sim_workspace_bytes(int S)
{
    const size_t wgs = max_workgroups(S);
    return (1 + (wgs + kArrivalGroup - 1) / kArrivalGroup) * kCounterLine * sizeof(int) + wgs * 3 * sizeof(float);
}

int launch_cos_sim(const void* a, const void* b, int S, size_t N, int dtype, int mode, float* out, void* workspace,
                   void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    int* counter = static_cast<int*>(workspace);
    const size_t wgs = max_workgroups(S);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                              (1 + (wgs + kArrivalGroup - 1) / kArrivalGroup) * kCounterLine * sizeof(int));
    const int rows = mode == 0 ? 1 : S;
    const int inner = mode == 0 ? S : 1;
    const int chunks = chunks_per_row(N, rows, dtype == 1);
    const dim3 grid(chunks, rows);
    if (rows == 1) {
        if (dtype == 1)
            hipLaunchKernelGGL((cos_sim_kernel<true, kThreadsOneRow, kInFlightOneRow>), grid, dim3(kThreadsOneRow), 0, s, a, b, inner, N,
                               rows, counter, partial, out);
        else
            hipLaunchKernelGGL((cos_sim_kernel<false, kThreadsOneRow, kInFlightOneRow>), grid, dim3(kThreadsOneRow), 0, s, a, b, inner, N,
                               rows, counter, partial, out);
    } else {
        if (dtype == 1)
            hipLaunchKernelGGL((cos_sim_kernel<true, kThreadsRows, kInFlightRows>), grid, dim3(kThreadsRows), 0, s, a, b, inner, N, rows,
                               counter, partial, out);
        else
            hipLaunchKernelGGL((cos_sim_kernel<false, kThreadsRows, kInFlightRows>), grid, dim3(kThreadsRows), 0, s, a, b, inner, N, rows,
                               counter, partial, out);
    }
    return (int)hipGetLastError();
}

}  // namespace kvs
