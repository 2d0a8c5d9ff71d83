// Tile arithmetic shared by the bf16 / fp8 attention kernels (gfx950): pages as MFMA operand
// registers, the score, softmax and value steps over a pair of pages, and the device-scope
// accesses and the arrival counter the context splits are merged with.
#pragma once
#include <hip/hip_runtime.h>

#include "kvs_device.h"
#include "kvs_internal.h"

namespace kvs {
namespace {

constexpr float kRefSlack = 8.f;       // log2 units a score may exceed the softmax reference by

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int D>
struct PageRegs {          // native vectors: they stay in registers when passed by reference
    u32x4 k[D / 32];
    u32x4 v[D / 32];
};

template <int D>
__device__ __forceinline__ void load_page(PageRegs<D>& r, const void* pool, size_t page_off, int lane)
{
    // Every key and value is read once per launch: stream them past the caches.
    const u32x4* kp = reinterpret_cast<const u32x4*>(static_cast<const unsigned short*>(pool) + page_off) + lane;
    const u32x4* vp = kp + (kPageTokens * D * 2) / 16;
#pragma unroll
    for (int s = 0; s < D / 32; ++s) r.k[s] = __builtin_nontemporal_load(kp + s * 64);
#pragma unroll
    for (int s = 0; s < D / 32; ++s) r.v[s] = __builtin_nontemporal_load(vp + s * 64);
}

// The same page in the fp8 store: half the registers, and one 16-byte load carries two
// contraction steps of K (or four channel tiles of V).
template <int D>
struct PageRegs8 {
    u32x4 k[D / 64];
    u32x4 v[D / 64];
};

template <int D>
__device__ __forceinline__ void load_page(PageRegs8<D>& r, const void* pool, size_t page_off, int lane)
{
    const u32x4* kp = reinterpret_cast<const u32x4*>(static_cast<const unsigned char*>(pool) + page_off) + lane;
    const u32x4* vp = kp + (kPageTokens * D) / 16;
#pragma unroll
    for (int s = 0; s < D / 64; ++s) r.k[s] = __builtin_nontemporal_load(kp + s * 64);
#pragma unroll
    for (int s = 0; s < D / 64; ++s) r.v[s] = __builtin_nontemporal_load(vp + s * 64);
}

// Four E4M3 bytes -> four bf16 (two words), exactly: every E4M3 value is a bf16 value.
__device__ __forceinline__ void widen4(unsigned w, unsigned& lo, unsigned& hi)
{
    const floatx2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    const floatx2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    lo = __builtin_bit_cast(unsigned, __builtin_convertvector(a, bf16x2));
    hi = __builtin_bit_cast(unsigned, __builtin_convertvector(b, bf16x2));
}

// One 16-byte piece of an fp8 page -> the two 16-byte pieces of the bf16 page it stands for (same
// lane, consecutive 64-piece blocks).  Keys: words x, y are one contraction step (channels
// 8*quad .. +3, then +4 .. +7), words z, w the next.  Values: channel tiles 2s and 2s + 1 (tokens
// 4*quad .. +3 each) in x, y, the next two in z, w.
__device__ __forceinline__ void widen_piece(const u32x4 raw, u32x4& first, u32x4& second)
{
    unsigned a0, a1, b0, b1;
    widen4(raw.x, a0, a1);
    widen4(raw.y, b0, b1);
    first = u32x4{a0, a1, b0, b1};
    widen4(raw.z, a0, a1);
    widen4(raw.w, b0, b1);
    second = u32x4{a0, a1, b0, b1};
}

// fp8 page registers -> the bf16 operand registers the arithmetic below works on.
template <int D>
__device__ __forceinline__ void widen(const PageRegs8<D>& r, PageRegs<D>& o)
{
#pragma unroll
    for (int s = 0; s < D / 64; ++s) {
        widen_piece(r.k[s], o.k[2 * s], o.k[2 * s + 1]);
        widen_piece(r.v[s], o.v[2 * s], o.v[2 * s + 1]);
    }
}

// Zero the values of tokens `first`.. of this lane's four (first <= 0 clears all four): the
// lane holds tokens 4*quad..4*quad+3 of the page, two per 32-bit word, for two channel tiles.
template <int D>
__device__ __forceinline__ void clear_values_from(u32x4 (&v)[D / 32], int first)
{
    const unsigned m01 = (0 < first ? 0x0000ffffu : 0u) | (1 < first ? 0xffff0000u : 0u);
    const unsigned m23 = (2 < first ? 0x0000ffffu : 0u) | (3 < first ? 0xffff0000u : 0u);
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        v[s].x &= m01; v[s].y &= m23; v[s].z &= m01; v[s].w &= m23;
    }
}

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}

// Split states cross compute units, and on this chip each group of compute units has its own
// L2.  They are therefore written and read with device-scope atomic accesses, which go to
// the memory side of the L2s, instead of flushing and invalidating whole caches around
// ordinary accesses.  A writer waits for its stores to complete before its workgroup bumps
// the arrival counter; the reader issues its loads only after it has read the final count.
__device__ __forceinline__ void publish_pair(float* p, float x, float y)
{
    const floatx2 v = {x, y};
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ floatx2 fetch_pair(const float* p)
{
    const unsigned long long w = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(floatx2, w);
}

// The end of a workgroup that has published its partial states: the one that arrives last at
// its (sequence, kv head, column group) merges the splits.  Nobody waits: each workgroup publishes
// its partial state, bumps the counter and leaves; the one that reads (live splits - 1) finds every
// other state already published.  Returns whether this workgroup is that last one.
__device__ __forceinline__ bool arrived_last(int* counter, int live_splits)
{
    __shared__ int s_is_last;
    // vmcnt(0): every device-scope store this wavefront issued has been acknowledged.  A
    // workgroup-scope fence would not wait for that (the compute unit orders its own accesses).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (threadIdx.x == 0) {
        const int arrived = atomicAdd(counter, 1);
        s_is_last = arrived == live_splits - 1;
        if (s_is_last) atomicExch(counter, 0);          // leave the counter ready for the next call
    }
    __syncthreads();
    if (!s_is_last) return false;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return true;
}

// Merge of the published states of `live_splits` splits for the columns [first_col, first_col +
// n_cols) of (sequence b, kv head g): the normalised output rows.  The record of (output row,
// split s) is number row * rec_per_row + s * rec_per_split + rec_first.
template <int D>
__device__ __forceinline__ void merge_splits(const AttnArgs& a, int b, int g, int first_col, int n_cols, int ncols,
                                             int group, int live_splits, int n_threads,
                                             int rec_per_row, int rec_per_split, size_t rec_first)
{
    const StoreView& st = a.st;
    for (int idx = threadIdx.x; idx < n_cols * (D / 4); idx += n_threads) {
        const int cidx = first_col + idx / (D / 4);
        const int d4 = (idx % (D / 4)) * 4;
        if (cidx >= ncols) break;
        const int r = cidx / group, hc = cidx % group;
        const size_t row = ((size_t)b * a.T_new + r) * st.Hq + g * group + hc;
        const float* part = a.partials + (row * rec_per_row + rec_first) * (size_t)(D + 2);
        const size_t step = (size_t)rec_per_split * (D + 2);
        // Eight records at a time, all their loads issued before any is used: one memory round trip
        // per eight parts (a pass for the maximum and a pass for the sums were two to three per
        // eight).  Beyond eight parts the running reference moves as in the online softmax.
        constexpr int kAtOnce = 8;
        float M = -INFINITY;
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        float lt = 0.f;
        for (int s0 = 0; s0 < live_splits; s0 += kAtOnce) {
            floatx2 ml[kAtOnce], lo[kAtOnce], hi[kAtOnce];
#pragma unroll
            for (int u = 0; u < kAtOnce; ++u) {
                const float* ps = part + (size_t)(s0 + u < live_splits ? s0 + u : s0) * step;   // past the end: a record that exists
                ml[u] = fetch_pair(ps + D);
                lo[u] = fetch_pair(ps + d4);
                hi[u] = fetch_pair(ps + d4 + 2);
            }
            float Mc = M;
#pragma unroll
            for (int u = 0; u < kAtOnce; ++u) {
                if (s0 + u >= live_splits) ml[u][0] = -INFINITY;     // weight 0
                Mc = fmaxf(Mc, ml[u][0]);
            }
            const float M_use = Mc == -INFINITY ? 0.f : Mc;
            const float keep = __builtin_amdgcn_exp2f(M - M_use);    // 0 while nothing has been added (M = -inf)
            acc *= keep;
            lt *= keep;
#pragma unroll
            for (int u = 0; u < kAtOnce; ++u) {
                const float wgt = __builtin_amdgcn_exp2f(ml[u][0] - M_use);   // empty parts carry m = -inf
                acc += wgt * floatx4{lo[u][0], lo[u][1], hi[u][0], hi[u][1]};
                lt += wgt * ml[u][1];
            }
            M = Mc;
        }
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        *reinterpret_cast<floatx4*>(a.out + row * D + d4) = acc * inv;
    }
}

// Reductions over the four lanes l, l^16, l^32, l^48 that hold one query column, with the
// gfx950 lane-swap instructions: permlane16_swap(x, x) returns the pair (rows 0,0,2,2 of x,
// rows 1,1,3,3 of x) for 16-lane rows, permlane32_swap the same for 32-lane halves, so two
// swaps and two combines replace two round trips through the LDS crossbar.
__device__ __forceinline__ float column_max(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float column_sum(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// One softmax / accumulation step over a pair of pages (32 tokens) for the NT column tiles of a
// wavefront, in three parts so that a caller whose pages sit in LDS can fetch the value operands
// while the scores are being turned into probabilities.  ka / kb and va / vb hold the key and
// value operands of the two pages (second page absent: have_b false), tok_a / tok_b are their
// first token positions, n_col[ct] the number of keys the lane's column of tile ct sees, n_min /
// n_max the fewest / most keys any column of the wavefront sees.
//
// Scores of the 32 tokens against the wavefront's columns: sa / sb, one accumulator per page and tile.
template <int D, int NT>
__device__ __forceinline__ void pair_qk(const u32x4 (&ka)[D / 32], u32x4 (&kb)[D / 32], bool have_b,
                                        const bf16x8 (&qf)[NT][D / 32], floatx4 (&sa)[NT], floatx4 (&sb)[NT])
{
    constexpr int KS = D / 32;
    if (!have_b) {
#pragma unroll
        for (int s = 0; s < KS; ++s) kb[s] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) sa[ct] = sb[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            sa[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[s]), qf[ct][s], sa[ct], 0, 0, 0);
            sb[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[s]), qf[ct][s], sb[ct], 0, 0, 0);
        }
}

// Masking, the softmax update of m, l and o, and the probabilities as bf16 operands.
template <int D, int NT>
__device__ __forceinline__ void pair_softmax(const floatx4 (&sa)[NT], const floatx4 (&sb)[NT], bool have_b, int tok_a,
                                             int tok_b, int n_min, const int (&n_col)[NT], float (&m)[NT],
                                             float (&l)[NT], floatx4 (&o)[NT][D / 16], int quad, float scale_log2,
                                             bf16x8 (&pf)[NT])
{
    constexpr int DT = D / 16;
    const bool need_mask = !have_b || tok_b + kPageTokens > n_min || tok_a + kPageTokens > n_min;
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        float z[8];                                          // raw scores; the scale is applied inside the exponent
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            z[i] = sa[ct][i];
            z[4 + i] = sb[ct][i];
        }
        if (need_mask) {
            const int ta = tok_a + quad * 4, tb = tok_b + quad * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                z[i] = (ta + i < n_col[ct]) ? z[i] : -INFINITY;
                z[4 + i] = (have_b && tb + i < n_col[ct]) ? z[4 + i] : -INFINITY;
            }
        }
        // m is the reference of the exponentials, not necessarily the running maximum:
        // softmax is shift invariant, so the reference only moves (and o, l are only
        // rescaled) when a score exceeds it by more than kRefSlack; until then weights
        // may reach 2^kRefSlack, which fp32 sums and bf16 operands hold without loss.
        // Whether any column must move is decided from the lanes' own maxima; the reduction
        // over the four lanes of a column is only paid for on the pairs where one does.
        const float lane_max = scale_log2 * fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])),
                                                  fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
        if (__any(lane_max > m[ct] + kRefSlack)) {           // false while everything is masked
            const float mx = column_max(lane_max);
            const bool up = mx > m[ct] + kRefSlack;
            const float m_new = up ? mx : m[ct];
            const float alpha = __builtin_amdgcn_exp2f(m[ct] - (m_new == -INFINITY ? 0.f : m_new));   // 1 in lanes that keep their reference
            l[ct] *= alpha;
#pragma unroll
            for (int c = 0; c < DT; ++c) o[ct][c] *= alpha;
            m[ct] = m_new;
        }
        const float m_use = m[ct] == -INFINITY ? 0.f : m[ct];   // column sees nothing yet
        float p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(z[i], scale_log2, -m_use));
        l[ct] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        const uint4 pw = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]),
                                    pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
        pf[ct] = __builtin_bit_cast(bf16x8, pw);
    }
}

// The same update for kernels bound by their own arithmetic (prefill with many query columns),
// where every vector instruction counts: on this part the vector instructions of a wavefront do
// not run beside the matrix instructions of the other wavefront of its SIMD, the two add up.
// The reference m starts at kNoReference, finite and far below any score, instead of minus
// infinity, so no case needs a guard (the first score a column sees overflows its weight, which
// moves the reference to that pair's maximum); the weights are formed against the reference first,
// and whether it has to move is read off their sum, which the update needs anyway: a lane's eight
// weights sum to more than 2^kRefSlack only if one of them exceeds 2^(kRefSlack - 3), and a column
// whose maximum is that far above the reference moves (then its weights are formed again, all at
// most 1).  The maxima are computed only then.
constexpr float kMoveAt = kRefSlack - 3.5f;      // log2 units above the reference from which a column moves once a sum trips
constexpr float kNoReference = -1e30f;

template <int D, int NT>
__device__ __forceinline__ void pair_softmax_by_sum(const floatx4 (&sa)[NT], const floatx4 (&sb)[NT], bool have_b, int tok_a,
                                                    int tok_b, int n_min, const int (&n_col)[NT], float (&m)[NT],
                                                    float (&l)[NT], floatx4 (&o)[NT][D / 16], int quad, float scale_log2,
                                                    bf16x8 (&pf)[NT])
{
    constexpr int DT = D / 16;
    const bool need_mask = !have_b || tok_b + kPageTokens > n_min || tok_a + kPageTokens > n_min;
    const float sum_limit = __builtin_amdgcn_exp2f(kRefSlack);
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        float z[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            z[i] = sa[ct][i];
            z[4 + i] = sb[ct][i];
        }
        if (need_mask) {
            const int ta = tok_a + quad * 4, tb = tok_b + quad * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                z[i] = (ta + i < n_col[ct]) ? z[i] : -INFINITY;
                z[4 + i] = (have_b && tb + i < n_col[ct]) ? z[4 + i] : -INFINITY;
            }
        }
        float p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(z[i], scale_log2, -m[ct]));
        float ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        if (__any(!(ps <= sum_limit))) {                     // some weight is too large (or overflowed): rare
            const float lane_max = scale_log2 * fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])),
                                                      fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
            const float mx = column_max(lane_max);           // minus infinity while the column sees nothing
            const bool up = mx > m[ct] + kMoveAt;
            const float m_new = up ? mx : m[ct];
            const float alpha = __builtin_amdgcn_exp2f(m[ct] - m_new);   // 1 in columns that keep their reference
            l[ct] *= alpha;
#pragma unroll
            for (int c = 0; c < DT; ++c) o[ct][c] *= alpha;
            m[ct] = m_new;
#pragma unroll
            for (int i = 0; i < 8; ++i) p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(z[i], scale_log2, -m_new));
            ps = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
        }
        l[ct] += ps;
        const uint4 pw = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]),
                                    pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
        pf[ct] = __builtin_bit_cast(bf16x8, pw);
    }
}

// o += V^T . P^T.  Tokens past the stored length hold whatever the allocation held:
// their values are cleared first, so that a zero probability cannot meet a NaN.
template <int D, int NT>
__device__ __forceinline__ void pair_values(u32x4 (&va)[D / 32], u32x4 (&vb)[D / 32], bool have_b, int tok_a, int tok_b,
                                            int n_max, int quad, const bf16x8 (&pf)[NT], floatx4 (&o)[NT][D / 16])
{
    constexpr int KS = D / 32, DT = D / 16;
    if (tok_a + kPageTokens > n_max) clear_values_from<D>(va, n_max - tok_a - quad * 4);
    if (!have_b) {
#pragma unroll
        for (int s = 0; s < KS; ++s) vb[s] = u32x4{0u, 0u, 0u, 0u};
    } else if (tok_b + kPageTokens > n_max) {
        clear_values_from<D>(vb, n_max - tok_b - quad * 4);
    }
#pragma unroll
    for (int c = 0; c < DT; ++c) {
        const u32x4 xa = va[c >> 1], xb = vb[c >> 1];
        // contraction slots 0-3: tokens 4*quad.. of the first page, 4-7: of the second
        const u32x4 vcat = (c & 1) ? u32x4{xa.z, xa.w, xb.z, xb.w} : u32x4{xa.x, xa.y, xb.x, xb.y};
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
            o[ct][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vcat), pf[ct],
                                                               o[ct][c], 0, 0, 0);
    }
}

// The same for value operands that already arrive as the eight-token operands of a pair (the
// shared-page kernels lay them out that way in LDS): words x, y of vcat[c] are the first page's
// four tokens of channel tile c, words z, w the second page's.
template <int D, int NT>
__device__ __forceinline__ void pair_values_cat(u32x4 (&vcat)[D / 16], bool have_b, int tok_a, int tok_b, int n_max,
                                                int quad, const bf16x8 (&pf)[NT], floatx4 (&o)[NT][D / 16])
{
    constexpr int DT = D / 16;
    if (!have_b || tok_b + kPageTokens > n_max) {            // some token of the pair lies past the stored length
        const int fa = n_max - tok_a - quad * 4, fb = have_b ? n_max - tok_b - quad * 4 : 0;
        const unsigned a01 = (0 < fa ? 0x0000ffffu : 0u) | (1 < fa ? 0xffff0000u : 0u);
        const unsigned a23 = (2 < fa ? 0x0000ffffu : 0u) | (3 < fa ? 0xffff0000u : 0u);
        const unsigned b01 = (0 < fb ? 0x0000ffffu : 0u) | (1 < fb ? 0xffff0000u : 0u);
        const unsigned b23 = (2 < fb ? 0x0000ffffu : 0u) | (3 < fb ? 0xffff0000u : 0u);
#pragma unroll
        for (int c = 0; c < DT; ++c) {
            vcat[c].x &= a01; vcat[c].y &= a23; vcat[c].z &= b01; vcat[c].w &= b23;
        }
    }
#pragma unroll
    for (int c = 0; c < DT; ++c)
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
            o[ct][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vcat[c]), pf[ct], o[ct][c], 0, 0, 0);
}

template <int D, int NT>
__device__ __forceinline__ void consume_pair(PageRegs<D>& pa, PageRegs<D>& pb, bool have_b, int tok_a, int tok_b,
                                             int n_min, int n_max, const int (&n_col)[NT],
                                             const bf16x8 (&qf)[NT][D / 32], float (&m)[NT], float (&l)[NT],
                                             floatx4 (&o)[NT][D / 16], int quad, float scale_log2)
{
    floatx4 sa[NT], sb[NT];
    bf16x8 pf[NT];
    pair_qk<D, NT>(pa.k, pb.k, have_b, qf, sa, sb);
    pair_softmax<D, NT>(sa, sb, have_b, tok_a, tok_b, n_min, n_col, m, l, o, quad, scale_log2, pf);
    pair_values<D, NT>(pa.v, pb.v, have_b, tok_a, tok_b, n_max, quad, pf, o);
}

}  // namespace
}  // namespace kvs
