// stalloc_plan: batched greedy placement, one workgroup per candidate placement order; the
// entry point, and the placement kernel for traces the occupancy-bitmap kernel does not take.
//
// Rule (Sec. 5.1): requests are taken in the given order; each gets the lowest address at
// which it conflicts with no earlier request of the same plan in lifespan and address
// range at once.  Extent of a plan = max(a + s) (Eq. 2).
//
// Per plan the workgroup keeps the list of placed blocks SORTED BY ADDRESS, so that no
// sorting is needed when a request is placed.  Requests are handled in batches of K:
//
//   scan     One pass over the sorted list serves the whole batch, because the list only
//            changes between batches.  Each wave owns a run of consecutive entries (its
//            chunk); every entry is loaded once and tested against the K requests: two
//            compares keep the blocks whose lifetime conflicts with request r, the running
//            maximum of their end addresses is "covered so far", and a conflicting block that
//            starts at least size_r above it closes a hole [covered, start) in which r could
//            fit.  Per (wave, request) the wave publishes its chunk maximum and its first
//            few holes (with chunk-local "covered") to LDS.  Two forms: with the list in LDS
//            (K = 16) a lane holds a listed block and the running maximum is a wave64 DPP
//            scan per request; with the list in the workspace (K = 64) a lane holds a
//            request and the blocks are taken one by one as wave-uniform values, which needs
//            no cross-lane step at all.
//   survey   After a barrier, wave r gathers what all waves published for request r into its
//            64 lanes in address order; the true "covered" of a hole is the maximum of its
//            local value and the chunk maxima of the waves below.  It lists the first holes
//            that are large enough as such.
//   resolve  After another barrier, wave 0 settles the K requests in order.  The blocks
//            settled earlier in the batch (the side buffer, sorted, one per lane) are honoured
//            through f(c) = lowest address >= c that clears the side-buffer blocks conflicting
//            with r: r takes the first surveyed hole with f(covered) + size_r <= hole end, else
//            goes on top at f(maximum).  If the surveyed holes run out while more were
//            published, all published holes are looked at with f evaluated over "zones" --
//            maximal groups of conflicting side-buffer blocks whose holes are too small for r.
//            If a wave had more holes than it could publish and none of the earlier ones
//            fits, wave 0 walks that wave's chunk again for this one request, with
//            everything below the chunk known, and takes the chunk's first hole that fits.
//   merge    The settled blocks are merged into the sorted list in one pass: listed block k
//            moves up by the number of new blocks at or below its start address and the new
//            blocks drop into the gaps (in place through registers when the list is in LDS,
//            ping-pong between two slabs when it is in the workspace).
//
// Addresses are multiples of the largest power of two dividing all sizes.  When the sum of
// sizes, in those granules, stays below 2^31 the list holds 32-bit granule counts (16-byte
// entries, single-instruction max/compare/DPP), below 2^16 (and with 16-bit timestamps) 8-byte
// cells; otherwise 64-bit byte addresses.  The sum of sizes is a bound no sensible plan comes
// near, so when only the sum is too large (no single size reaches 2^30 granules) the 32-bit
// instantiation still takes every plan, as far as the extent so far plus the sizes of the next
// batch stays below 2^32 granules, and marks the plans that fail the check for the 64-bit
// instantiation enqueued behind it.  Only the device knows which case applies (the trace
// check leaves it in the mode word), so every instantiation that could apply is enqueued and
// those with nothing to do return at once.  The list lives in LDS when it fits and in the
// workspace otherwise.
#include "host_util.h"
#include "plan_list.h"
#include "plan_params.h"
#include "wave.h"

namespace stalloc {

constexpr int kBatch = 256;          // requests fetched per refill

template <typename Addr, int kPend, int kThreads>
struct PlanLds {
    static constexpr int kWaves = kThreads / kWave;
#ifdef STALLOC_HOLE_SLOTS
    static constexpr int kSlots = STALLOC_HOLE_SLOTS;      // (test builds shrink this to exercise the second walk of a chunk)
#else
    // holes a wave can publish per request; three when 64 requests with 64-bit addresses share
    // a pass, so that two workgroups still fit the LDS of a CU
    static constexpr int kSlots = (sizeof(Addr) == 8 && kPend > 32 && kWaves == 16) ? 3 : kWave / kWaves;
#endif
    uint64_t rq_size[kBatch];
    uint64_t rq_addr[kBatch];
    uint32_t rq_ta[kBatch];
    uint32_t rq_tf[kBatch];
    uint32_t rq_id[kBatch];
    Addr top[kWaves][kPend];                               // chunk maximum per (wave, request)
    uint32_t holes[kWaves][kPend];                         // holes found per (wave, request), may exceed kSlots
    Span<Addr> hole[kWaves][kPend][kSlots];                // {hole end, chunk-local covered}
    Span<Addr> surveyed[kPend][4];                         // survey: first holes large enough as such {end, covered}
    uint32_t listed[kPend];                                // survey: how many, bit 8 = more to look at behind them
    Addr top_of[kPend];                                    // survey: maximum over all chunks
    Span<Addr> pend_span[kPend];                           // blocks settled in this batch, sorted
    uint2 pend_life[kPend];
    uint32_t settled;
    Addr extent_now;                                       // extent of the plan after the last settled batch
};

// Zones of the side buffer for one request: groups of lifetime-conflicting pending blocks.
// A zone starts at a conflicting block that leaves a hole of at least `s` above everything
// conflicting before it; it ends at the running maximum of end addresses.
template <typename Addr>
struct Zones {
    uint64_t starts;     // lanes that open a zone
    Addr lo;             // per lane: start address of the pending block
    Addr reach_before;   // per lane: max end of conflicting pending blocks in lower lanes
    Addr reach_all;      // uniform: max end of all conflicting pending blocks
};

template <typename Addr>
__device__ __forceinline__ Zones<Addr> make_zones(const Pending<Addr>& pd, uint32_t pending, Addr s,
                                                  uint32_t ta, uint32_t tf)
{
    const int lane = lane_id();
    const bool conflict = lane < (int)pending && pd.ta < tf && ta < pd.tf;
    const Addr incl = wave_scan_max(conflict ? pd.hi : (Addr)0);
    Zones<Addr> z;
    z.lo = pd.lo;
    z.reach_before = wave_shift_up(incl, (Addr)0);
    z.reach_all = read_lane(incl, kWave - 1);
    const uint64_t conflicts = __builtin_amdgcn_ballot_w64(conflict);
    const uint64_t lower = conflicts & ((1ull << lane) - 1);
    z.starts = __builtin_amdgcn_ballot_w64(conflict && (lower == 0 || pd.lo >= z.reach_before + s));
    return z;
}

// f(e): lowest address >= e at which [e, e + s) clears every zone.
template <typename Addr>
__device__ __forceinline__ Addr clear_zones(Addr e, Addr s, const Zones<Addr>& z)
{
    uint64_t m = z.starts;
    if (m == 0) return e;
    const Addr es = e + s;
    while (m) {
        const int q = __builtin_ctzll(m);
        m &= m - 1;
        const Addr zone_lo = read_lane(z.lo, q);
        const Addr zone_hi = m ? read_lane(z.reach_before, __builtin_ctzll(m)) : z.reach_all;
        if (es > zone_lo && e < zone_hi) e = zone_hi;
    }
    return e;
}

// Sorted insertion of the block [x, x + s) into the register-held side buffer.
template <typename Addr>
__device__ __forceinline__ void pending_insert(Pending<Addr>& pd, uint32_t pending, Addr x, Addr s, uint32_t ta,
                                               uint32_t tf)
{
    const int lane = lane_id();
    const uint64_t keep = __builtin_amdgcn_ballot_w64(lane < (int)pending && pd.lo <= x);
    const int pos = __builtin_popcountll(keep);
    const Addr up_lo = wave_shift_up(pd.lo, (Addr)0), up_hi = wave_shift_up(pd.hi, (Addr)0);
    const uint32_t up_ta = wave_shift_up(pd.ta, 0u), up_tf = wave_shift_up(pd.tf, 0u);
    if (lane > pos) { pd.lo = up_lo; pd.hi = up_hi; pd.ta = up_ta; pd.tf = up_tf; }
    if (lane == pos) { pd.lo = x; pd.hi = x + s; pd.ta = ta; pd.tf = tf; }
}

// One pass over the sorted list for the requests b0 .. b0+nb-1 of the staged batch: publishes,
// per (wave, request), the chunk maximum of conflicting end addresses and the first holes.
template <typename Addr, int kPend, int kThreads, typename List, typename Lds>
__device__ __forceinline__ void scan_batch(const List& list, uint32_t count, uint32_t b0, uint32_t nb,
                                           uint32_t shift, Lds& sh)
{
    constexpr int kSlots = Lds::kSlots;
    const int lane = lane_id(), wave = wave_id();
    // lane r holds request r of the batch; unused lanes get an empty lifetime (conflicts with nothing)
    Addr rq_s = 0;
    uint32_t rq_ta = 0, rq_tf = 0;
    if (lane < (int)nb) {
        rq_s = (Addr)(sh.rq_size[b0 + lane] >> shift);
        rq_ta = sh.rq_ta[b0 + lane];
        rq_tf = sh.rq_tf[b0 + lane];
    }
    Addr run[kPend];        // uniform: running maximum for request r inside this wave's chunk
    uint32_t found[kPend];  // uniform: holes found for request r
    Addr s_of[kPend];       // uniform copies of the request parameters
    uint32_t ta_of[kPend], tf_of[kPend];
#pragma unroll
    for (int r = 0; r < kPend; ++r) {
        run[r] = 0; found[r] = 0;
        s_of[r] = read_lane(rq_s, r); ta_of[r] = read_lane(rq_ta, r); tf_of[r] = read_lane(rq_tf, r);
    }
    const uint32_t sub = (count + kThreads - 1) / kThreads;     // 64-entry steps per wave
    uint32_t k = (uint32_t)wave * kWave * sub + lane;
    for (uint32_t j = 0; j < sub; ++j, k += kWave) {
        const bool valid = k < count;
        const uint32_t kc = valid ? k : count - 1;
        const typename List::Entry en = list.load(kc);
        const Span<Addr> sp = {en.lo(), en.hi()};
        // lanes past the end of the list get a lifetime that conflicts with nothing
        const uint2 lf = make_uint2(valid ? en.ta() : 0xffffffffu, valid ? en.tf() : 0u);
        // requests in groups of kGroup: their running-maximum chains are independent, so the
        // compiler can interleave the DPP steps of one chain into the wait states of the others
        constexpr int kGroup = 4;
#pragma unroll
        for (int g = 0; g < kPend; g += kGroup) {
            Addr incl[kGroup], covered[kGroup];
            uint64_t conflict_m[kGroup], closers[kGroup];
            uint64_t any_closer = 0;
            Addr ends[kGroup];
#pragma unroll
            for (int q = 0; q < kGroup; ++q) {
                const int r = g + q;
                conflict_m[q] = lanes_lt(lf.x, tf_of[r]) & lanes_lt(ta_of[r], lf.y);   // lanes past the end: see above
            }
            keep_lanes4(conflict_m, sp.hi, ends);
#pragma unroll
            for (int q = 0; q < kGroup; ++q) incl[q] = wave_scan_max(ends[q]);
#pragma unroll
            for (int q = 0; q < kGroup; ++q) {
                const int r = g + q;
                covered[q] = umax(run[r], wave_shift_up(incl[q], (Addr)0));
                closers[q] = conflict_m[q] & lanes_ge(sp.lo, (Addr)(covered[q] + s_of[r]));
                any_closer |= closers[q];
                run[r] = umax(run[r], read_lane(incl[q], kWave - 1));
            }
            if (any_closer) {
#pragma unroll
                for (int q = 0; q < kGroup; ++q) {
                    const int r = g + q;
                    uint64_t m = closers[q];                     // holes [covered, sp.lo) in front of conflicting blocks
                    while (m && found[r] < (uint32_t)kSlots) {
                        const int f = __builtin_ctzll(m);
                        m &= m - 1;
                        // uniform address and data: every lane stores the same record
                        sh.hole[wave][r][found[r]] = Span<Addr>{read_lane(sp.lo, f), read_lane(covered[q], f)};
                        ++found[r];
                    }
                    if (m) found[r] = kSlots + 1;                // more holes than slots
                }
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < kPend; ++r) {
            sh.top[wave][r] = run[r];
            sh.holes[wave][r] = found[r];
        }
    }
}

// The same pass with the roles of lanes and loop exchanged, for lists in the workspace: lane r
// holds request r of the batch (up to 64 of them) and the listed blocks of the wave's chunk
// are taken one at a time, in address order, as wave-uniform values.  A block costs two
// lifetime compares, an add and two address compares for all requests at once -- no
// cross-lane running maximum, which is what the lane-per-block form spends its time on when
// one pass serves many requests.  What is published per (wave, request) is identical.
template <typename Addr, int kPend, int kThreads, typename List, typename Lds>
__device__ __forceinline__ void scan_batch_by_request(const List& list, uint32_t count, uint32_t b0, uint32_t nb,
                                                      uint32_t shift, Lds& sh)
{
    constexpr int kSlots = Lds::kSlots;
    static_assert(kPend <= kWave, "one lane per request of the batch");
    const int lane = lane_id(), wave = wave_id();
    // unused lanes get an empty lifetime (conflicts with nothing)
    Addr rq_s = 0;
    uint32_t rq_ta = 0, rq_tf = 0;
    if (lane < (int)nb) {
        rq_s = (Addr)(sh.rq_size[b0 + lane] >> shift);
        rq_ta = sh.rq_ta[b0 + lane];
        rq_tf = sh.rq_tf[b0 + lane];
    }
    Addr covered = 0;        // per request: maximum end of the conflicting blocks of this chunk so far
    uint32_t found = 0;      // per request: holes found in this chunk
    const uint32_t sub = (count + kThreads - 1) / kThreads;     // 64-entry steps per wave
    const uint32_t chunk0 = (uint32_t)wave * kWave * sub;
    for (uint32_t j = 0; j < sub; ++j) {
        const uint32_t k0 = chunk0 + j * kWave;
        if (k0 >= count) break;                                  // (uniform)
        const uint32_t k = k0 + lane;
        const bool valid = k < count;
        const typename List::Entry en = list.load(valid ? k : count - 1);
        const Addr e_lo = en.lo(), e_hi = en.hi();
        // lanes past the end of the list get a lifetime that conflicts with nothing
        const uint32_t e_ta = valid ? en.ta() : 0xffffffffu, e_tf = valid ? en.tf() : 0u;
#pragma unroll
        for (int q = 0; q < kWave; ++q) {
            const uint32_t ta_q = read_lane(e_ta, q), tf_q = read_lane(e_tf, q);
            const bool conflict = ta_q < rq_tf && rq_ta < tf_q;
            if (__builtin_amdgcn_ballot_w64(conflict) == 0) continue;   // (uniform) the block concerns no request of the batch
            const Addr lo_q = read_lane(e_lo, q), hi_q = read_lane(e_hi, q);
            if (conflict && lo_q >= (Addr)(covered + rq_s)) {    // a hole [covered, lo_q) in front of this block
                if (found < (uint32_t)kSlots) sh.hole[wave][lane][found] = Span<Addr>{lo_q, covered};
                found = found < (uint32_t)kSlots ? found + 1 : (uint32_t)kSlots + 1;   // kSlots + 1: more holes than slots
            }
            const Addr reach = umax(covered, hi_q);
            covered = conflict ? reach : covered;
        }
    }
    if (lane < kPend) {
        sh.top[wave][lane] = covered;
        sh.holes[wave][lane] = found;
    }
}

// What the waves published for request r, gathered into the 64 lanes of one wave in address
// order (lane = wave * kSlots + slot), with the true "covered" of every hole.
template <typename Addr>
struct HoleView {
    Addr covered;        // per lane: covered in front of this hole (chunk maxima of lower waves included)
    Addr end;            // per lane: address at which the hole ends
    Addr top;            // uniform: maximum over all chunks (where the request goes if no hole fits)
    Addr below;          // per lane: maximum over the chunks of the waves below this lane's wave
    uint64_t published;  // lanes that hold a hole
    uint64_t crowded;    // lanes of waves that found more holes than they could publish
};

template <typename Addr, typename Lds>
__device__ __forceinline__ HoleView<Addr> view_holes(const Lds& sh, uint32_t r)
{
    constexpr int kSlots = Lds::kSlots;
    const int lane = lane_id();
    const int w = lane / kSlots, c = lane % kSlots;
    const bool live = w < Lds::kWaves;                  // (always true unless kSlots was shrunk)
    const int wc = live ? w : 0;
    const Addr topv = live ? sh.top[wc][r] : (Addr)0;
    const uint32_t found = live ? sh.holes[wc][r] : 0u;
    const Span<Addr> hl = sh.hole[wc][r][c];
    const Addr incl = wave_scan_max(topv);
    const Addr below = lane_gather(wave_shift_up(incl, (Addr)0), wc * kSlots);
    HoleView<Addr> v;
    v.covered = umax(below, hl.hi);
    v.below = below;
    v.end = hl.lo;
    v.top = read_lane(incl, kWave - 1);
    v.published = lanes_lt((uint32_t)c, found);
    v.crowded = __builtin_amdgcn_ballot_w64(found > (uint32_t)kSlots);
    return v;
}

// True if a wave with unpublished holes lies below lane h (h < 0: the request would go on top).
template <typename Lds>
__device__ __forceinline__ bool unpublished_below(uint64_t crowded, int h)
{
    return crowded && (h < 0 || __builtin_ctzll(crowded) / Lds::kSlots < h / Lds::kSlots);
}

constexpr int kSurveyed = 4;     // holes the survey lists per request

// Survey (all waves, request r handled by wave r mod #waves): lists, in address order, the
// first holes that are large enough as such, and says what follows the list: the top of the
// plan (every usable hole is listed) or a closer look at everything that was published.
template <typename Addr, int kPend, int kThreads, typename Lds>
__device__ __forceinline__ void survey_batch(uint32_t b0, uint32_t nb, uint32_t shift, Lds& sh)
{
    for (uint32_t r = (uint32_t)wave_id(); r < nb; r += Lds::kWaves) {
        const Addr s = (Addr)(sh.rq_size[b0 + r] >> shift);
        const HoleView<Addr> v = view_holes<Addr>(sh, r);
        uint64_t raw = v.published & lanes_ge(v.end, (Addr)(v.covered + s));
        uint32_t listed = 0;
        while (raw && listed < (uint32_t)kSurveyed) {
            const int h = __builtin_ctzll(raw);
            if (unpublished_below<Lds>(v.crowded, h)) break;          // an unpublished hole may lie lower
            raw &= raw - 1;
            sh.surveyed[r][listed] = Span<Addr>{read_lane(v.end, h), read_lane(v.covered, h)};   // uniform store
            ++listed;
        }
        if (lane_id() == 0) {
            sh.listed[r] = listed | ((raw || v.crowded) ? 0x100u : 0u);     // bit 8: more to look at after the list
            sh.top_of[r] = v.top;
        }
    }
}

// Lowest address >= c at which [c, c + s) clears the pending blocks selected by `rivals`
// (lanes of the side buffer whose lifetime conflicts with the request).
template <typename Addr>
__device__ __forceinline__ Addr clear_rivals(Addr c, Addr s, uint64_t rivals, const Pending<Addr>& pd)
{
    if (rivals == 0) return c;
    for (;;) {
        const uint64_t hit = rivals & lanes_lt(pd.lo, (Addr)(c + s)) & lanes_lt(c, pd.hi);
        if (hit == 0) return c;
        c = read_lane(wave_scan_max(keep_lanes(hit, pd.hi)), kWave - 1);   // every address in [c, that end) is blocked
    }
}

// One wave walks the chunk of the list that wave `w` scanned, for one request, with everything
// below the chunk known (`below` = maximum end of the conflicting blocks of all lower chunks):
// the first hole of the chunk that takes the request once the zones of the side buffer are
// cleared.  Returns true and the address if there is one.  This is what a wave could not
// publish when its chunk held more holes than it has slots.
template <typename Addr, int kThreads, typename List>
__device__ __forceinline__ bool chunk_lowest_fit(const List& list, uint32_t count, int w, Addr below, Addr s,
                                                 uint32_t ta, uint32_t tf, const Zones<Addr>& zones, Addr& x)
{
    const int lane = lane_id();
    const uint32_t sub = (count + kThreads - 1) / kThreads;     // 64-entry steps per wave, as in the scan
    const uint32_t chunk0 = (uint32_t)w * kWave * sub;
    Addr run = below;
    typename List::Entry ahead = List::none();
    if (chunk0 + lane < count) ahead = list.load(chunk0 + lane);
    for (uint32_t j = 0; j < sub; ++j) {
        const uint32_t k0 = chunk0 + j * kWave;
        if (k0 >= count) break;                                  // (uniform)
        const typename List::Entry en = ahead;
        const bool valid = k0 + lane < count;
        if (j + 1 < sub && k0 + kWave + lane < count) ahead = list.load(k0 + kWave + lane);
        const Addr e_lo = en.lo();
        const bool conflict = valid && en.ta() < tf && ta < en.tf();
        const Addr incl = wave_scan_max(conflict ? (Addr)en.hi() : (Addr)0);
        const Addr before = umax(run, wave_shift_up(incl, (Addr)0));
        const bool opens = conflict && e_lo >= (Addr)(before + s);            // a hole [before, e_lo) large enough as such
        if (__builtin_amdgcn_ballot_w64(opens)) {
            const Addr cleared = clear_zones(before, s, zones);
            const uint64_t fits = __builtin_amdgcn_ballot_w64(opens && e_lo >= (Addr)(cleared + s));
            if (fits) { x = read_lane(cleared, __builtin_ctzll(fits)); return true; }
        }
        run = umax(run, read_lane(incl, kWave - 1));
    }
    return false;
}

// Wave 0 settles the requests of the batch in order.  Returns how many were settled (all).
template <typename Addr, int kPend, int kThreads, typename List, typename Lds>
__device__ __forceinline__ uint32_t resolve_batch(const List& list, uint32_t count, uint32_t b0, uint32_t nb,
                                                  uint32_t shift, Addr& peak, Lds& sh)
{
    const int lane = lane_id();
    // lane r holds request r of the batch
    Addr rq_s = 0, topv = 0;
    uint32_t rq_ta = 0, rq_tf = 0, listedv = 0;
    if (lane < (int)nb) {
        rq_s = (Addr)(sh.rq_size[b0 + lane] >> shift);
        rq_ta = sh.rq_ta[b0 + lane];
        rq_tf = sh.rq_tf[b0 + lane];
        listedv = sh.listed[lane];
        topv = sh.top_of[lane];
    }
    Pending<Addr> pd = {0, 0, 0, 0};
    // lane i < kSurveyed holds surveyed hole i of the current request; fetched one request ahead
    Span<Addr> holes_next = sh.surveyed[0][lane < kSurveyed ? lane : 0];
    uint32_t r = 0;
    for (; r < nb; ++r) {
        const Addr s = read_lane(rq_s, (int)r);
        const uint32_t ta = read_lane(rq_ta, (int)r), tf = read_lane(rq_tf, (int)r);
        const uint32_t listed = read_lane(listedv, (int)r);
        const Span<Addr> holes = holes_next;
        if (r + 1 < nb) holes_next = sh.surveyed[r + 1][lane < kSurveyed ? lane : 0];
        // blocks settled earlier in this batch whose lifetime conflicts with the request
        const uint64_t rivals = __builtin_amdgcn_ballot_w64(lane < (int)r && pd.ta < tf && ta < pd.tf);
        Addr x = 0;
        bool placed = false;
        for (uint32_t i = 0; i < (listed & 0xffu) && !placed; ++i) {
            const Addr c = clear_rivals(read_lane(holes.hi, (int)i), s, rivals, pd);
            if (c + s <= read_lane(holes.lo, (int)i)) { x = c; placed = true; }
        }
        if (!placed) {
            if (!(listed & 0x100u)) {
                x = clear_rivals(read_lane(topv, (int)r), s, rivals, pd);       // on top of everything
            } else {
                const HoleView<Addr> v = view_holes<Addr>(sh, r);
                const Zones<Addr> zones = make_zones(pd, r, s, ta, tf);
                const Addr cleared = clear_zones(v.covered, s, zones);
                const uint64_t fits = v.published & lanes_ge(v.end, (Addr)(cleared + s));
                const int h = fits ? __builtin_ctzll(fits) : -1;
                // chunks with more holes than their wave could publish, lowest first, as long as
                // they lie below the chunk of hole h: the lowest fit may be one of those
                bool lower = false;
                for (uint64_t crowded = v.crowded; unpublished_below<Lds>(crowded, h);) {
                    const int first = __builtin_ctzll(crowded);
                    const int w = first / Lds::kSlots;
                    lower = chunk_lowest_fit<Addr, kThreads>(list, count, w, read_lane(v.below, first), s, ta, tf, zones, x);
                    if (lower) break;
                    for (int c = 0; c < Lds::kSlots; ++c) crowded &= ~(1ull << (w * Lds::kSlots + c));
                }
                if (!lower) x = fits ? read_lane(cleared, h) : read_lane(clear_zones(v.top, s, zones), 0);
            }
        }
        peak = umax(peak, (Addr)(x + s));
        if (lane == 0) sh.rq_addr[b0 + r] = (uint64_t)x << shift;
        pending_insert(pd, r, x, s, ta, tf);
    }
    if (lane < (int)r) {
        sh.pend_span[lane] = Span<Addr>{pd.lo, pd.hi};
        sh.pend_life[lane] = make_uint2(pd.ta, pd.tf);
    }
    if (lane == 0) sh.settled = r;
    return r;
}

template <typename Addr, bool kLds, bool kCompact, int kPend, int kThreads>
__global__ void __launch_bounds__(kThreads, 4) plan_kernel(PlanParams prm)   // <= 128 VGPRs: 16 waves per CU
{
    using Lds = PlanLds<Addr, kPend, kThreads>;
    using List = BlockList<Addr, kCompact>;
    extern __shared__ __align__(16) unsigned char smem[];
    Lds& sh = *reinterpret_cast<Lds*>(smem);
    const uint32_t n = prm.n;

    if (*prm.status != STALLOC_OK) return;               // malformed trace: nothing to plan
    const uint64_t mode = prm.acc[kAccMode];
    if (bitmap_shape(mode, prm.acc[kAccGranules], prm.bitmap_pool_words) >= 0) return;   // the occupancy-bitmap kernel places this trace
    // the kernel that lists only long-lived blocks places it (and leaves the plans that outgrow
    // 32-bit counts to the 64-bit instantiation here)
    if (sizeof(Addr) == 4 && (prm.acc[kAccSplit] & 1)) return;
    const bool narrow = (mode & kModeNarrow) != 0;
    // Not narrow, but no request is large: the 32-bit instantiation takes every plan as far as
    // 32-bit granule counts certainly hold its addresses and marks the plans that outgrow them;
    // the 64-bit instantiation (enqueued behind it) places those from scratch.
    const bool try32 = (mode & kModeTry32) != 0;
    if (sizeof(Addr) == 4 ? !(narrow || try32) : narrow) return;     // another instantiation handles this trace
    // of the two 32-bit instantiations the compact one runs when it was enqueued and applies
    const bool compact = prm.compact_enqueued && (mode & kModeCompact) != 0;
    if (sizeof(Addr) == 4 && compact != kCompact) return;
    const uint32_t shift = sizeof(Addr) == 4 ? (uint32_t)(mode & 63) : 0;
    if (blockIdx.x == 0 && threadIdx.x == 0 && !(sizeof(Addr) == 8 && try32))
        const_cast<uint64_t*>(prm.acc)[kAccKernel] = (kLds ? STALLOC_KERNEL_LIST_LDS : STALLOC_KERNEL_LIST_MEMORY) |
                                                     ((kCompact ? 16u : 8u * (uint32_t)sizeof(Addr)) << 8);

    List list, spare;
    if constexpr (kLds) {
        list.bind(smem + sizeof(Lds), n);
        spare = list;
    } else {
        unsigned char* slab = prm.slabs + (size_t)blockIdx.x * 2 * (size_t)n * entry_bytes<uint64_t>();
        list.bind(slab, n);
        spare.bind(slab + (size_t)n * entry_bytes<uint64_t>(), n);
    }

    for (uint32_t p = blockIdx.x; p < prm.P; p += gridDim.x) {
        if (sizeof(Addr) == 8 && try32 && !prm.wide_plans[p]) continue;   // (uniform) placed with 32-bit counts already
        if (sizeof(Addr) == 8 && try32 && threadIdx.x == 0)
            atomicAdd((unsigned long long*)&const_cast<uint64_t*>(prm.acc)[kAccWidePlans], 1ull);
        const uint32_t* order = prm.orders + (size_t)p * n;
        uint64_t* out = prm.offsets ? prm.offsets + (size_t)p * n : nullptr;
        Addr peak = 0;                                        // tracked by wave 0
        uint32_t count = 0;
        bool outgrown = false;                                // (uniform) 32-bit counts may not hold the next batch
        __syncthreads();                                      // (every wave has taken its decisions about the plan before)
        if (threadIdx.x == 0) sh.extent_now = 0;

        for (uint32_t r0 = 0; r0 < n; r0 += kBatch) {
            const uint32_t staged = n - r0 < (uint32_t)kBatch ? n - r0 : (uint32_t)kBatch;
            __syncthreads();                                  // previous batch fully consumed
            if (threadIdx.x < staged) {
                uint32_t i = order[r0 + threadIdx.x];
                if (i >= n) { atomicMax(prm.status, (uint32_t)STALLOC_ERR_BAD_ORDER); i = 0; }
                sh.rq_id[threadIdx.x] = i;
                sh.rq_size[threadIdx.x] = prm.size[i];
                sh.rq_ta[threadIdx.x] = prm.ta[i];
                sh.rq_tf[threadIdx.x] = prm.tf[i];
            }
            __syncthreads();

            for (uint32_t b0 = 0; b0 < staged;) {
                const uint32_t nb = staged - b0 < (uint32_t)kPend ? staged - b0 : (uint32_t)kPend;
                if (sizeof(Addr) == 4 && try32) {
                    // no address of this batch exceeds the extent so far plus the sizes of the batch
                    const int lane = lane_id();
                    const uint64_t growth = wave_sum64(lane < (int)nb ? sh.rq_size[b0 + lane] >> shift : 0ull);
                    if ((uint64_t)sh.extent_now + growth > 0xffffffffull) { outgrown = true; break; }
                }
                if constexpr (kLds) scan_batch<Addr, kPend, kThreads>(list, count, b0, nb, shift, sh);
                else scan_batch_by_request<Addr, kPend, kThreads>(list, count, b0, nb, shift, sh);
                __syncthreads();
                survey_batch<Addr, kPend, kThreads>(b0, nb, shift, sh);
                __syncthreads();
                if (wave_id() == 0) {
                    resolve_batch<Addr, kPend, kThreads>(list, count, b0, nb, shift, peak, sh);
                    if (lane_id() == 0) sh.extent_now = peak;
                }
                __syncthreads();
                const uint32_t settled = sh.settled;
                const bool last_of_plan = r0 + b0 + settled >= n;
                if (settled && !last_of_plan) merge_pending<Addr, kLds, kThreads>(list, spare, count, settled, sh);
                count += settled;
                b0 += settled;
            }
            if (outgrown) break;
            // addresses of this batch -> offsets[p][request id]
            __syncthreads();
            if (out && threadIdx.x < staged) out[sh.rq_id[threadIdx.x]] = sh.rq_addr[threadIdx.x];
        }
        if (outgrown) {
            if (threadIdx.x == 0) prm.wide_plans[p] = 1;
            continue;
        }
        if (threadIdx.x == 0) prm.peaks[p] = (uint64_t)peak << shift;
    }
}

__global__ void plan_clear_marks(uint32_t* wide_plans, uint32_t P)
{
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < P; p += gridDim.x * blockDim.x) wide_plans[p] = 0;
}

// best_plan = index of the smallest extent (lowest index among equals); one workgroup.
__global__ void __launch_bounds__(256) plan_argmin(const uint64_t* __restrict__ peaks, uint32_t P, uint32_t* best_plan,
                                                   const uint32_t* status)
{
    __shared__ uint64_t w_peak[4];
    __shared__ uint64_t w_idx[4];
    if (*status != STALLOC_OK) { if (threadIdx.x == 0) *best_plan = 0; return; }
    uint64_t best = ~0ull, idx = ~0ull;
    for (uint32_t p = threadIdx.x; p < P; p += 256) {
        uint64_t v = peaks[p];
        if (v < best) { best = v; idx = p; }       // ascending p per thread: first of equals kept
    }
    uint64_t wbest = wave_min64(best);
    uint64_t widx = wave_min64(best == wbest ? idx : ~0ull);
    if (lane_id() == 0) { w_peak[wave_id()] = wbest; w_idx[wave_id()] = widx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t b = w_peak[0], i = w_idx[0];
        for (int k = 1; k < 4; ++k)
            if (w_peak[k] < b || (w_peak[k] == b && w_idx[k] < i)) { b = w_peak[k]; i = w_idx[k]; }
        *best_plan = (uint32_t)i;
    }
}

__global__ void __launch_bounds__(256) plan_copy_best(const uint64_t* __restrict__ offsets, const uint32_t* best_plan,
                                                      uint32_t n, uint64_t* best_offsets, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    const uint64_t* src = offsets + (size_t)(*best_plan) * n;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) best_offsets[i] = src[i];
}

// Tuning knobs (overridable at build time with -D).
#ifndef STALLOC_PEND_LDS
#define STALLOC_PEND_LDS 16
#endif
#ifndef STALLOC_PEND_MEM
#define STALLOC_PEND_MEM 64
#endif
#ifndef STALLOC_THREADS_LDS
#define STALLOC_THREADS_LDS 1024
#endif
#ifndef STALLOC_THREADS_MEM
#define STALLOC_THREADS_MEM 1024
#endif
constexpr int kPendLds = STALLOC_PEND_LDS;        // requests per batch when the list is in LDS
constexpr int kPendMem = STALLOC_PEND_MEM;        // ... and when it is in the workspace (every batch costs passes over memory)
constexpr int kThreadsLds = STALLOC_THREADS_LDS;
constexpr int kThreadsMem = STALLOC_THREADS_MEM;

#ifndef STALLOC_THREADS_COMPACT
#define STALLOC_THREADS_COMPACT 512
#endif
constexpr int kThreadsCompact = STALLOC_THREADS_COMPACT;   // two such workgroups share one CU

// Entries the LDS-resident list may hold, for a given entry size and LDS budget.
template <typename Addr, int kThreads>
inline uint32_t lds_capacity_entries(size_t lds_budget, size_t bytes_per_entry)
{
    const size_t fixed = sizeof(PlanLds<Addr, kPendLds, kThreads>);
    if (lds_budget <= fixed) return 0;
    return (uint32_t)((lds_budget - fixed) / bytes_per_entry);
}

template <typename Addr, bool kLds, bool kCompact, int kPend, int kThreads>
inline bool launch_plan(const PlanParams& prm, uint32_t grid, const DeviceInfo& di, hipStream_t stream)
{
    auto kernel = &plan_kernel<Addr, kLds, kCompact, kPend, kThreads>;
    size_t lds = sizeof(PlanLds<Addr, kPend, kThreads>) +
                 (kLds ? (size_t)prm.n * BlockList<Addr, kCompact>::kEntryBytes : 0);
    static std::atomic<bool> attr_set[64] = {};        // (set twice at worst when threads race)
    if (!attr_set[di.device]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)di.lds_per_block) != hipSuccess)
            return false;
        attr_set[di.device] = true;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kThreads), lds, stream, prm);
    return true;
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_plan_report(const void* workspace, stalloc_plan_info* info, void* hip_stream)
{
    if (!workspace || !info) return STALLOC_ERR_INVALID_ARG;
    uint64_t acc[kAccWords];
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(acc, workspace, sizeof(acc), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return STALLOC_ERR_DEVICE;
    info->kernel = (uint32_t)(acc[kAccKernel] & 0xffu);
    info->address_bits = (uint32_t)((acc[kAccKernel] >> 8) & 0xffu);
    info->granule_log2 = (uint32_t)(acc[kAccMode] & 63);
    info->granules = acc[kAccGranules];
    info->plans_64bit = (uint32_t)acc[kAccWidePlans];
    info->lifetime_threshold = (acc[kAccSplit] & 1) ? (uint32_t)((acc[kAccSplit] >> 8) & 0xffffffu) : 0u;
    info->long_requests = (acc[kAccSplit] & 1) ? (uint32_t)(acc[kAccSplit] >> 32) : 0u;
    const bool large = (acc[kAccSplit] & 1) && (uint32_t)acc[kAccLargeShort] != 0xffffffffu;
    info->large_size = large ? (acc[kAccLargeShort] & 0xffffffffull) << (acc[kAccMode] & 63) : 0ull;
    info->large_requests = large ? (uint32_t)(acc[kAccLargeShort] >> 32) : 0u;
    info->list_entry_bytes = (uint32_t)((acc[kAccKernel] >> 16) & 0xffu);
    return STALLOC_OK;
}

extern "C" uint32_t stalloc_plan_lds_capacity(void)
{
    DeviceInfo di;
    if (!device_info(&di)) return 0;
    return lds_capacity_entries<uint32_t, kThreadsLds>(di.lds_per_block, entry_bytes<uint32_t>());
}

// allow_bitmap: false when the caller has said that its sizes cannot suit the occupancy-bitmap kernel; that
// kernel and its index of lifetime-overlapping pairs are then left out of the call and of the workspace.
static int plan_call(const stalloc_trace* tr, const uint32_t* orders, uint32_t P, uint64_t* offsets, uint64_t* peaks,
                     uint64_t* best_offsets, uint32_t* best_plan, uint32_t* device_status, bool allow_bitmap,
                     void* workspace, size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || P == 0 || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    DeviceInfo di;
    if (!device_info(&di)) return STALLOC_ERR_DEVICE;
    const uint32_t n = tr->n;
    const bool lds32 = n <= lds_capacity_entries<uint32_t, kThreadsLds>(di.lds_per_block, entry_bytes<uint32_t>());
    const bool lds64 = n <= lds_capacity_entries<uint64_t, kThreadsLds>(di.lds_per_block, entry_bytes<uint64_t>());
    // compact list: 8-byte entries, two workgroups per CU (half the LDS each)
    const bool compact = tr->t_end < 0x10000u &&
                         n <= lds_capacity_entries<uint32_t, kThreadsCompact>(di.lds_per_block / 2, sizeof(uint2));
    uint32_t grid_lds = (uint32_t)di.cus, grid_mem = (uint32_t)di.cus * 2, grid_compact = (uint32_t)di.cus * 2;
    if (grid_lds > P) grid_lds = P;
    if (grid_mem > P) grid_mem = P;
    if (grid_compact > P) grid_compact = P;

    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    uint64_t* own_offsets = (!offsets && best_offsets) ? cv.take<uint64_t>((size_t)P * n) : nullptr;
    unsigned char* slabs = lds64 ? nullptr : cv.take<unsigned char>((size_t)grid_mem * 2 * n * entry_bytes<uint64_t>());
    uint32_t* wide_plans = cv.take<uint32_t>(P);
    // occupancy-bitmap variant: lifetime-conflict index of the trace
    uint32_t pool_words[kBitmapShapes];
    const bool bitmap = bitmap_plan_shapes(n, di, pool_words) && allow_bitmap;
    uint32_t* nbr_begin = bitmap ? cv.take<uint32_t>((size_t)n + 2) : nullptr;
    uint16_t* nbr = bitmap ? cv.take<uint16_t>(bitmap_index_entries(n)) : nullptr;
    // variant for long traces with few long-lived requests: tables in allocation-time order
    const bool split = !lds32;
    SplitWorkspace sw;
    if (split) split_workspace(n, tr->t_end, di, cv, &sw);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!orders || !peaks || !best_plan || !device_status || *workspace_bytes < cv.used ||
        (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);

    PlanParams prm;
    prm.size = tr->size; prm.ta = tr->t_alloc; prm.tf = tr->t_free; prm.orders = orders;
    prm.offsets = offsets ? offsets : own_offsets;
    prm.peaks = peaks; prm.status = device_status; prm.acc = acc; prm.slabs = slabs; prm.n = n; prm.P = P;
    prm.compact_enqueued = compact ? 1u : 0u;
    prm.nbr_begin = nbr_begin; prm.nbr = nbr; prm.wide_plans = wide_plans;
    {
        uint32_t pb = (P + 255) / 256;
        if (pb > 256) pb = 256;
        hipLaunchKernelGGL(plan_clear_marks, dim3(pb), dim3(256), 0, stream, wide_plans, P);
    }
    for (int shape = 0; shape < kBitmapShapes; ++shape) prm.bitmap_pool_words[shape] = bitmap ? pool_words[shape] : 0u;
    bool ok = true;
    if (split) ok = ok && launch_plan_split(prm, tr->t_end, sw, di, stream);
    if (bitmap) ok = ok && launch_plan_bitmap(prm, di, stream);
    // exactly one of the launches does the work; the trace decides which (see the mode word)
    if (compact) ok = ok && launch_plan<uint32_t, true, true, kPendLds, kThreadsCompact>(prm, grid_compact, di, stream);
    if (lds32) ok = ok && launch_plan<uint32_t, true, false, kPendLds, kThreadsLds>(prm, grid_lds, di, stream);
    else       ok = ok && launch_plan<uint32_t, false, false, kPendMem, kThreadsMem>(prm, grid_mem, di, stream);
    if (lds64) ok = ok && launch_plan<uint64_t, true, false, kPendLds, kThreadsLds>(prm, grid_lds, di, stream);
    else       ok = ok && launch_plan<uint64_t, false, false, kPendMem, kThreadsMem>(prm, grid_mem, di, stream);
    if (!ok) return STALLOC_ERR_DEVICE;

    hipLaunchKernelGGL(plan_argmin, dim3(1), dim3(256), 0, stream, peaks, P, best_plan, device_status);
    if (best_offsets) {
        uint32_t blocks = (n + 255) / 256;
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(plan_copy_best, dim3(blocks), dim3(256), 0, stream, prm.offsets, best_plan, n, best_offsets,
                           device_status);
    }
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}

extern "C" int stalloc_plan(const stalloc_trace* tr, const uint32_t* orders, uint32_t P, uint64_t* offsets,
                            uint64_t* peaks, uint64_t* best_offsets, uint32_t* best_plan, uint32_t* device_status,
                            void* workspace, size_t* workspace_bytes, void* hip_stream)
{
    return plan_call(tr, orders, P, offsets, peaks, best_offsets, best_plan, device_status, true, workspace, workspace_bytes,
                     hip_stream);
}

extern "C" int stalloc_plan_sized(const stalloc_trace* tr, const uint32_t* orders, uint32_t P, uint64_t* offsets,
                                  uint64_t* peaks, uint64_t* best_offsets, uint32_t* best_plan, uint32_t* device_status,
                                  uint64_t largest_size, uint64_t granule, void* workspace, size_t* workspace_bytes,
                                  void* hip_stream)
{
    if (granule == 0 || (granule & (granule - 1)) != 0 || largest_size == 0) return STALLOC_ERR_INVALID_ARG;
    const bool allow_bitmap = largest_size / granule <= kBitmapMaxSize;
    return plan_call(tr, orders, P, offsets, peaks, best_offsets, best_plan, device_status, allow_bitmap, workspace,
                     workspace_bytes, hip_stream);
}
