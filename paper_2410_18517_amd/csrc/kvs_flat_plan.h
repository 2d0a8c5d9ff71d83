// How a decode launch shares out its keys and values by tokens: plain integer arithmetic used by
// the kernel (every workgroup derives the whole plan from the sequence lengths it reads on the
// device) and, through the library's testing hooks, checked on the host against brute force.
//
// A sequence of p pages occupies ceil(p / 8) octets; an octet is the eight pages the four
// wavefronts of a workgroup take in one step, a pair each.  The octets of all (kv head, sequence)
// segments, kv head by kv head and sequence by sequence, form one line; the launch's n workgroups
// cut that line into n shares that differ by at most one octet.  A share may begin and end in the
// middle of a segment and may hold several whole segments.
#pragma once

#if defined(__HIPCC__)
#define KVS_PLAN_FN __host__ __device__ inline
#else
#define KVS_PLAN_FN inline
#endif

namespace kvs {

constexpr int kOctetPages = 8;

struct FlatShare {
    int lo, count;      // octets [lo, lo + count) of the line
};

// Share of workgroup i of n over a line of `total` octets: the first total % n workgroups take
// one octet more than the others.
KVS_PLAN_FN FlatShare flat_share(int i, int n, int total)
{
    const int base = total / n, rem = total % n;
    FlatShare s;
    s.lo = i * base + (i < rem ? i : rem);
    s.count = base + (i < rem ? 1 : 0);
    return s;
}

// The workgroup whose share holds octet o (0 <= o < total).
KVS_PLAN_FN int flat_owner(int o, int n, int total)
{
    const int base = total / n, rem = total % n;
    const int big = rem * (base + 1);          // octets held by the larger shares
    return o < big ? o / (base + 1) : rem + (o - big) / base;   // base > 0 whenever o >= big
}

}  // namespace kvs
