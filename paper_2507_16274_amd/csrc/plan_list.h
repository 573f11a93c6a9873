// The sorted list of placed blocks that the list-based placement kernels keep per plan, and the
// pass that merges newly settled blocks into it (shared by the sorted-list kernel and the kernel
// that keeps only long-lived blocks in the list).
#pragma once

#include "host_util.h"
#include "wave.h"

namespace stalloc {

template <typename Addr> struct Span { Addr lo, hi; };     // [lo, hi) in address units

template <typename Addr> struct Top;
template <> struct Top<uint32_t> { static constexpr uint32_t value = 0xffffffffu; };
template <> struct Top<uint64_t> { static constexpr uint64_t value = ~0ull; };

// The sorted list of placed blocks.  Two storage layouts:
//   wide     (lo, hi) in address units of type Addr plus (t_alloc, t_free) as 32-bit values
//   compact  lo, hi, t_alloc, t_free as 16-bit fields of one 8-byte cell; usable when the sum of
//            sizes in granules and the number of timestamps both stay below 2^16
template <typename Addr, bool kCompact>
struct BlockList;

template <typename Addr>
struct BlockList<Addr, false> {
    typedef Addr addr_type;
    static constexpr size_t kEntryBytes = sizeof(Span<Addr>) + sizeof(uint2);
    struct Entry {
        Span<Addr> sp;
        uint2 lf;
        __device__ __forceinline__ Addr lo() const { return sp.lo; }
        __device__ __forceinline__ Addr hi() const { return sp.hi; }
        __device__ __forceinline__ uint32_t ta() const { return lf.x; }
        __device__ __forceinline__ uint32_t tf() const { return lf.y; }
    };
    Span<Addr>* span;
    uint2* life;
    __device__ __forceinline__ void bind(unsigned char* base, uint32_t cap)
    {
        span = reinterpret_cast<Span<Addr>*>(base);
        life = reinterpret_cast<uint2*>(span + cap);
    }
    __device__ __forceinline__ Entry load(uint32_t k) const { return Entry{span[k], life[k]}; }
    __device__ __forceinline__ void store(uint32_t k, const Entry& e) const { span[k] = e.sp; life[k] = e.lf; }
    static __device__ __forceinline__ Entry make(Addr lo, Addr hi, uint32_t ta, uint32_t tf)
    {
        return Entry{Span<Addr>{lo, hi}, make_uint2(ta, tf)};
    }
    static __device__ __forceinline__ Entry none() { return make(0, 0, 0, 0); }
};

template <>
struct BlockList<uint32_t, true> {
    typedef uint32_t addr_type;
    static constexpr size_t kEntryBytes = sizeof(uint2);
    struct Entry {
        uint2 c;
        __device__ __forceinline__ uint32_t lo() const { return c.x & 0xffffu; }
        __device__ __forceinline__ uint32_t hi() const { return c.x >> 16; }
        __device__ __forceinline__ uint32_t ta() const { return c.y & 0xffffu; }
        __device__ __forceinline__ uint32_t tf() const { return c.y >> 16; }
    };
    uint2* cell;
    __device__ __forceinline__ void bind(unsigned char* base, uint32_t) { cell = reinterpret_cast<uint2*>(base); }
    __device__ __forceinline__ Entry load(uint32_t k) const { return Entry{cell[k]}; }
    __device__ __forceinline__ void store(uint32_t k, const Entry& e) const { cell[k] = e.c; }
    static __device__ __forceinline__ Entry make(uint32_t lo, uint32_t hi, uint32_t ta, uint32_t tf)
    {
        return Entry{make_uint2(lo | (hi << 16), ta | (tf << 16))};
    }
    static __device__ __forceinline__ Entry none() { return Entry{make_uint2(0, 0)}; }
};

template <typename Addr> constexpr size_t entry_bytes() { return BlockList<Addr, false>::kEntryBytes; }

// The side buffer in registers: block q in lane q, ascending start address.
template <typename Addr>
struct Pending {
    Addr lo, hi;
    uint32_t ta, tf;
};

template <typename Addr, typename Lds>
__device__ __forceinline__ Pending<Addr> load_pending(const Lds& sh, uint32_t pending)
{
    Pending<Addr> pd = {0, 0, 0, 0};
    const int lane = lane_id();
    if (lane < (int)pending) {
        const Span<Addr> sp = sh.pend_span[lane];
        const uint2 lf = sh.pend_life[lane];
        pd.lo = sp.lo; pd.hi = sp.hi; pd.ta = lf.x; pd.tf = lf.y;
    }
    return pd;
}

// Number of pending blocks (sorted by start address, one per lane) whose start address is
// <= lo, for a wave-uniform lo; `from` of them are already known to be.
template <typename Addr>
__device__ __forceinline__ uint32_t pending_at_or_below(const Pending<Addr>& pd, uint32_t pending, Addr lo, uint32_t from)
{
    uint32_t q = from;
    while (q < pending && read_lane(pd.lo, (int)q) <= lo) ++q;
    return q;
}

// One merge pass over the list entries [base, base + kThreads * kSub) and, if it falls into that
// range, the position just past the end: listed block k moves to k + c_k, where c_k is the
// number of pending blocks at or below its start address; pending block q lands at k + q in
// front of the first listed block k with c_k > q (or behind the last one).  kSub is a template
// parameter so that the per-lane copies of the entries stay in registers.
template <typename Addr, bool kLds, int kThreads, int kSub, typename List, typename Lds>
__device__ __forceinline__ void merge_pass(const List& list, const List& dst, uint32_t count,
                                           uint32_t base, const Pending<Addr>& pd, uint32_t pending, Lds& sh)
{
    const int lane = lane_id(), wave = wave_id();
    const uint32_t chunk0 = base + (uint32_t)wave * kWave * kSub;
    typename List::Entry en[kSub];
    uint32_t c_here[kSub], c_prev[kSub];
    // pending blocks at or below the entry in front of this wave's chunk
    uint32_t carry = 0;
    if (chunk0 > 0 && chunk0 - 1 < count) {
        const Addr lo_before = read_lane((Addr)list.load(chunk0 - 1).lo(), 0);
        for (uint32_t step = 32; step > 0; step >>= 1)           // (the one place without a known starting point)
            if (carry + step <= pending && read_lane(pd.lo, (int)(carry + step - 1)) <= lo_before) carry += step;
        if (carry < pending && read_lane(pd.lo, (int)carry) <= lo_before) ++carry;
    } else if (chunk0 > count) {
        carry = pending;
    }
#pragma unroll
    for (int j = 0; j < kSub; ++j) {
        const uint32_t k0 = chunk0 + j * kWave;
        const uint32_t k = k0 + lane;
        const bool valid = k < count;
        en[j] = List::none();
        if (valid) en[j] = list.load(k);
        const Addr lo_j = en[j].lo();
        // Both sequences ascend, so the counts of a step lie between those of its first and last
        // block, and the first one starts from the previous step's last: the pending blocks are
        // walked once per chunk, and only the few that fall inside a step are compared per lane.
        uint32_t c = pending;
        if (k0 < count) {
            const int last_lane = count - k0 >= (uint32_t)kWave ? kWave - 1 : (int)(count - k0 - 1);
            const uint32_t c_first = pending_at_or_below(pd, pending, read_lane(lo_j, 0), carry);
            const uint32_t c_last = pending_at_or_below(pd, pending, read_lane(lo_j, last_lane), c_first);
            uint32_t mine = c_first;
            for (uint32_t q = c_first; q < c_last; ++q) mine += read_lane(pd.lo, (int)q) <= lo_j;
            c = valid ? mine : pending;
        }
        c_here[j] = c;
        c_prev[j] = wave_shift_up(c, carry);
        carry = read_lane(c, kWave - 1);
    }
    if constexpr (kLds) __syncthreads();     // in place: every block is in registers before any moves
#pragma unroll
    for (int j = 0; j < kSub; ++j) {
        const uint32_t k = chunk0 + j * kWave + lane;
        if (k < count && (!kLds || c_here[j] > 0)) {
            dst.store(k + c_here[j], en[j]);
        }
        if (k <= count) {
            for (uint32_t q = c_prev[j]; q < c_here[j]; ++q) {
                const Span<Addr> ps = sh.pend_span[q];
                const uint2 pl = sh.pend_life[q];
                dst.store(k + q, List::make(ps.lo, ps.hi, pl.x, pl.y));
            }
        }
    }
}

#ifndef STALLOC_MERGE_SUB
#define STALLOC_MERGE_SUB 4
#endif
constexpr int kMergeSub = STALLOC_MERGE_SUB;     // 64-entry steps one wave handles per merge segment

// Merges the side buffer (sh.pend_*, sorted, `pending` >= 1 blocks, already visible to the whole
// workgroup) into the sorted list.  The list is cut into segments of kThreads * kSub
// entries which are handled from the top down: blocks only move up, so a segment's writes
// never touch entries of the segments below it, which are read later.  When the list is in LDS
// the merge is in place (a barrier separates a segment's reads from its writes); otherwise
// it goes into the spare slab.
template <typename Addr, bool kLds, int kThreads, int kSub = kMergeSub, typename List, typename Lds>
__device__ __forceinline__ void merge_pending(List& list, List& spare, uint32_t count, uint32_t pending, Lds& sh)
{
    constexpr uint32_t kSegment = (uint32_t)kThreads * kSub;
    const Pending<Addr> pd = load_pending<Addr>(sh, pending);
    const List& dst = kLds ? list : spare;
    const uint32_t segments = count / kSegment + 1;          // the position just past the end counts too
    for (uint32_t g = segments; g-- > 0;) {
        merge_pass<Addr, kLds, kThreads, kSub>(list, dst, count, g * kSegment, pd, pending, sh);
        // In place, a block stays where it is when no pending block starts at or below it: once the
        // block in front of a segment starts below the lowest pending block, the rest is done.
        if constexpr (kLds) {
            if (g > 0 && read_lane((Addr)list.load(g * kSegment - 1).lo(), 0) < read_lane(pd.lo, 0)) break;
        }
    }
    if constexpr (!kLds) { List t = list; list = spare; spare = t; }
    __syncthreads();
}

}  // namespace stalloc
