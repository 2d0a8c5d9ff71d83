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

// The cut of a line of `total` octets into n shares (n <= 65535).  Share i begins at octet
// floor(total * i / n), so the shares differ by at most one octet and the longer ones are spread
// evenly over the workgroups.  A line shorter than n gives its octets to the first `total`
// workgroups, one each: the workgroups that hold the parts of a segment are then always consecutive,
// none of them empty, which the kernel's count of a segment's parts relies on.
// All in 32-bit arithmetic ((total % n) * i stays below 2^32), the two divisions by n that depend on
// the line alone done once.
struct FlatPlan {
    int n, total;
    unsigned base, rem;      // total = base * n + rem
    float per_octet;         // n / total: the owner of an octet, up to rounding

    KVS_PLAN_FN FlatPlan(int n_, int total_) : n(n_), total(total_)
    {
        base = (unsigned)total / (unsigned)n;
        rem = (unsigned)total - base * (unsigned)n;
        per_octet = total > 0 ? (float)n / (float)total : 0.f;
    }
    // first octet of workgroup i's share, i = 0 .. n (i = n: the end of the line)
    KVS_PLAN_FN int bound(int i) const
    {
        if (total < n) return i < total ? i : total;
        return (int)(base * (unsigned)i + (rem ? rem * (unsigned)i / (unsigned)n : 0u));
    }
    KVS_PLAN_FN FlatShare share(int i) const
    {
        FlatShare s;
        s.lo = bound(i);
        s.count = bound(i + 1) - s.lo;
        return s;
    }
    // the workgroup whose share holds octet o (0 <= o < total)
    KVS_PLAN_FN int owner(int o) const
    {
        int i = (int)(((float)o + 0.5f) * per_octet);
        i = i < 0 ? 0 : (i > n - 1 ? n - 1 : i);
        while (bound(i) > o) --i;
        while (bound(i + 1) <= o) ++i;
        return i;
    }
};

KVS_PLAN_FN FlatShare flat_share(int i, int n, int total) { return FlatPlan(n, total).share(i); }
KVS_PLAN_FN int flat_owner(int o, int n, int total) { return FlatPlan(n, total).owner(o); }

}  // namespace kvs
