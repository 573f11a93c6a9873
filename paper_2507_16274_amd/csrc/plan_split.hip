// stalloc_plan, placement kernel for long traces in which few requests live long: one
// workgroup per candidate placement order, the rule of Sec. 5.1 (every request gets the lowest
// address at which it conflicts with no earlier request of the plan in lifespan and address
// range at once).
//
// Training traces hold a few thousand long-lived tensors (activations kept from a forward to
// its backward pass) among hundreds of thousands that live for a handful of events (Sec. 2.3,
// Fig. 4).  A request's lifetime-conflicting blocks are then (a) long-lived blocks, of which
// there are few in all, and (b) short-lived blocks that started shortly before it or during
// its own lifetime, which in the order of allocation times form one contiguous range.  The
// kernel keeps the two kinds apart:
//
//   long blocks   (lifetime > theta) in a list sorted by address, in LDS, as the sorted-list
//                 kernel keeps all blocks.  Any request walks this list once, 64 blocks a step:
//                 two compares keep the blocks whose lifetime conflicts, a running maximum of
//                 their end addresses is "covered so far", a conflicting block that starts at
//                 least `size` above it closes a hole the request could take.
//   short blocks  (lifetime <= theta) in a per-plan table of addresses indexed by the request's
//                 rank in allocation-time order.  The short blocks that can conflict with a
//                 request are the placed entries of a window of that table, fixed per request
//                 and independent of the order: allocation times in (t_alloc - theta, t_free).
//                 A short-lived request reads its window (a few dozen entries) into the lanes
//                 of the wave.  A long-lived request, whose window spans thousands of entries,
//                 consults per-64-entry summaries (lowest start, highest end address of the
//                 placed blocks) and opens only the groups that can meet the range it tries.
//
// A hole of the long-block list takes the request if, after moving up past every other
// conflicting block that reaches into it (those of the window and those settled earlier in the
// same batch), the request still ends below the hole's end; the first such hole, else the top.
// Moving up: all addresses from c to the highest end of the blocks meeting [c, c + size) are
// blocked, so c jumps there, until nothing meets the range.
//
// Requests are settled in batches of 64 of the order.  Inside a batch a request waits only for
// the earlier requests of the batch whose lifetime conflicts with its own; everything that is
// ready is settled at once, dealt out to the waves (a wave with several short-lived requests
// settles up to four side by side, a row of 16 lanes each; the whole workgroup takes a
// long-lived one together), so that a batch takes as many rounds as its longest chain of
// conflicts (mostly two to four).  The long blocks of a batch are merged into the sorted list
// when the batch is done.
//
// The list comes in two forms (RankedList below): 16 bytes a block with its two times, two
// workgroups per CU, or 8 bytes a block with ranks in place of the times, three per CU.
//
// theta = 2^c - 1 is chosen so that the long requests fit the LDS list and are at most an eighth
// of all requests while the windows of the short ones stay narrow (sp_decide); traces for which
// no such theta exists, or in which many short requests have wide windows all the same (dense or
// tied timestamps), are left to the sorted-list kernel.  Addresses are 32-bit granule counts, with the same plan-by-plan
// hand-over to the 64-bit sorted-list kernel as there.
#include <type_traits>

#include "host_util.h"
#include "plan_list.h"
#include "plan_params.h"
#include "sort_keys.h"
#include "wave.h"

namespace stalloc {

constexpr int kSpThreads = 512;                  // two workgroups share a CU
constexpr int kSpBatch = 64;                     // requests between two merges; dependency masks have 64 bits
constexpr int kSpRefill = 128;                   // requests fetched per refill
constexpr int kSpPool = 640;                     // short blocks the windows of one batch may hold in LDS
constexpr int kSpWideHoles = 6;                  // holes of its part of the list that a wave writes down for a request the workgroup settles together
constexpr int kSpMaxWaves = 8;
constexpr uint32_t kSpRefetch = 0xffffffffu;     // (a window whose blocks did not fit the pool is read when its request is settled)
constexpr uint32_t kSpUnplaced = 0xffffffffu;
constexpr uint32_t kSpLongFlag = 0x80000000u;      // in a request's rank word: lives longer than theta
constexpr uint32_t kSpLargeFlag = 0x40000000u;     // short-lived, and at least sigma granules large
constexpr uint32_t kSpRankMask = 0x3fffffffu;
constexpr int kSpMaxThetaBits = 12;              // theta < 2^12 events
using SpList = BlockList<uint32_t, false>;

// The same list in 8 bytes per block, which lets a third workgroup share the LDS of a CU: the start
// address, and in the second word, instead of the two times, the block's ranks among the long-lived
// requests' allocation times (13 bits) and release times (13 bits, plus one), and the class of its
// size (6 bits; the sizes of the classes sit in an LDS table).  With, per request, the number A of
// long-lived requests allocated before its release and the number B released by its allocation, a
// block's lifetime conflicts with the request's if rank_alloc < A and B < rank_release + 1: the
// same two compares as on times.  Usable with at most 8190 long-lived requests of at most 64 sizes.
constexpr uint32_t kSpRankBits = 13;
constexpr uint32_t kSpRankedMost = (1u << kSpRankBits) - 2;
constexpr int kSpSizeClasses = 64;
struct RankedList {
    typedef uint32_t addr_type;
    static constexpr size_t kEntryBytes = sizeof(uint2);
    struct Entry {
        uint2 c;
        uint32_t end;
        __device__ __forceinline__ uint32_t lo() const { return c.x; }
        __device__ __forceinline__ uint32_t hi() const { return end; }
        __device__ __forceinline__ uint32_t ta() const { return c.y & ((1u << kSpRankBits) - 1); }
        __device__ __forceinline__ uint32_t tf() const { return (c.y >> kSpRankBits) & ((1u << kSpRankBits) - 1); }
    };
    uint2* cell;
    const uint32_t* class_size;      // [64] in LDS
    __device__ __forceinline__ void bind(unsigned char* base, uint32_t) { cell = reinterpret_cast<uint2*>(base); }
    __device__ __forceinline__ Entry load(uint32_t k) const
    {
        const uint2 c = cell[k];
        return Entry{c, c.x + class_size[c.y >> (2 * kSpRankBits)]};
    }
    __device__ __forceinline__ void store(uint32_t k, const Entry& e) const { cell[k] = e.c; }
    // (second word as made by sp_windows; hi is implied by the class)
    static __device__ __forceinline__ Entry make(uint32_t lo, uint32_t hi, uint32_t ranks_and_class, uint32_t)
    {
        return Entry{make_uint2(lo, ranks_and_class), hi};
    }
    static __device__ __forceinline__ Entry none() { return Entry{make_uint2(0u, 0u), 0u}; }
};
template <typename List> struct ListTraits { static constexpr bool kRanked = false; };
template <> struct ListTraits<RankedList> { static constexpr bool kRanked = true; };

struct SplitLds {
    uint32_t rq_id[kSpRefill];
    uint32_t rq_size[kSpRefill];                 // granules
    uint32_t rq_ta[kSpRefill];
    uint32_t rq_tf[kSpRefill];
    uint32_t rq_rank[kSpRefill];                 // rank in allocation-time order | kSpLongFlag
    uint32_t rq_wlo[kSpRefill];                  // window of that order holding the short requests that can conflict
    uint32_t rq_whi[kSpRefill];
    uint32_t rq_addr[kSpRefill];                 // granules
    uint32_t rq_counts[kSpRefill];               // ranked list: A | B << 16 (long-lived requests allocated before its release, released by its allocation)
    uint32_t rq_extra[kSpRefill];                // a large short block's place in the table of those; a long block's second list word (ranked list)
    uint32_t class_size[kSpSizeClasses];         // ranked list: sizes (granules) of the long-lived requests' size classes
    uint64_t dep[kSpBatch];                      // earlier requests of the batch with a conflicting lifetime
    Span<uint32_t> pend_span[kSpBatch];          // long blocks of the batch, sorted by address, for the merge
    uint2 pend_life[kSpBatch];
    Span<uint32_t> pool[kSpPool];                // conflicting short blocks of the windows of the batch's requests
    uint32_t pool_used;
    uint32_t pool_first[kSpBatch];               // where a request's part of the pool begins,
    uint32_t pool_count[kSpBatch];               // how many blocks it holds (kSpRefetch: they did not fit)
    uint32_t region_min[kWave];                  // lowest start / highest end address of the placed small short blocks of a
    uint32_t region_max[kWave];                  // region of ranks (64 regions cover the table)
    uint32_t large_min, large_max;               // the same over all placed large short blocks
    uint32_t reach[3];                           // window_reach: what the waves found, three calls in rotation
    // request with a wide window: every wave walks one part of the list.  Two sets, used in turn: the
    // waves still reading one request's set are a barrier away from those already writing the next but one's.
    Span<uint32_t> wide_hole[2][kSpMaxWaves][kSpWideHoles];   // candidate holes of that part {end, covered within the part}, in address order
    uint32_t wide_holes[2][kSpMaxWaves];         // how many there are (may exceed what is stored)
    uint32_t wide_part_top[2][kSpMaxWaves];      // highest end of the conflicting long blocks of that part
    uint32_t next_plan;                          // the plan this workgroup takes next
    uint32_t extent_now;                         // extent after the last finished batch
    uint32_t peak;                               // running extent
};

__host__ __device__ inline uint32_t split_list_capacity(size_t lds_per_workgroup, size_t entry_bytes = SpList::kEntryBytes)
{
    return lds_per_workgroup > sizeof(SplitLds) + 1024 ? (uint32_t)((lds_per_workgroup - sizeof(SplitLds)) / entry_bytes) : 0u;
}

// LDS of a workgroup when three share a CU (the allocation is rounded up, hence the slack).
inline size_t ranked_lds(const DeviceInfo& di) { return di.lds_per_block / 3 - 2048; }
// The ranked list needs two words per timestamp of the trace; traces whose timestamps are far apart do without it.
inline bool ranked_possible(uint32_t n, uint32_t t_end) { return (uint64_t)t_end <= 4ull * n + 4096; }

// ------------------------------------------------------------------------------------------
// Once per call: lifetime classes, allocation-time order, windows.

// hist[c] = requests whose lifetime lies in [2^c, 2^(c+1)).
__global__ void __launch_bounds__(256)
sp_histogram(const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf, uint32_t n, uint32_t* hist,
             const uint32_t* status)
{
    __shared__ uint32_t local[32];
    if (*status != STALLOC_OK) return;
    if (threadIdx.x < 32) local[threadIdx.x] = 0;
    __syncthreads();
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint32_t life = tf[i] - ta[i];                       // >= 1 in a sound trace
        atomicAdd(&local[life ? 31 - __builtin_clz(life) : 0], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 32 && local[threadIdx.x]) atomicAdd(&hist[threadIdx.x], local[threadIdx.x]);
}

constexpr int kSpHistWords = 80;                 // 32 lifetime classes, then [32]: requests with a wide window
constexpr int kSpHistWide = 32;
constexpr int kSpHistNextPlan = 33;              // (the counter that hands out plans lives behind the histogram)
constexpr int kSpHistSigma = 34;                 // sizes of at least this many granules count as large among the short-lived
constexpr int kSpHistTooManySizes = 35;          // ranked list: the long-lived requests have more than 64 sizes
constexpr int kSpHistSizes = 40;                 // 32 size classes of the short-lived requests

__global__ void sp_clear_histogram(uint32_t* hist, uint32_t* gate)
{
    for (int k = threadIdx.x; k < kSpHistWords; k += blockDim.x) hist[k] = 0;
    if (threadIdx.x == 0) *gate = 1;                                // closed until sp_decide opens it
}

// Decides whether this kernel places the trace, and with which theta; acc[kAccSplit] = 1 |
// theta << 8 | long requests << 32 (0: another kernel does), gate[0] = 0 when it does (the
// kernels that prepare its tables read the gate like a status word).
//
// theta = 2^c - 1.  Fewer long-lived requests mean a shorter list, but a larger theta widens the
// windows of the short-lived ones, which should fit the 64 lanes of a wave: with n allocations on
// t_end timestamps a window of up to 2 theta timestamps holds about 2 theta n / t_end ranks, and c
// is admissible while that stays below 48.  Among the admissible c that leave at most
// min(list_cap, n / 8) long requests, the one with the fewest long requests is taken, and of
// several such the smallest.
__global__ void sp_decide(uint64_t* acc, const uint32_t* hist, uint32_t n, uint32_t t_end, uint32_t list_cap,
                          PlanParams prm, uint32_t* gate, const uint32_t* status)
{
    if (threadIdx.x != 0) return;
    acc[kAccSplit] = 0;
    if (*status != STALLOC_OK) return;
    const uint64_t mode = acc[kAccMode];
    if (!(mode & (kModeNarrow | kModeTry32))) return;
    if (n > kSpRankMask) return;                                    // (a rank word keeps two bits for flags)
    if (bitmap_shape(mode, acc[kAccGranules], prm.bitmap_pool_words) >= 0) return;
    if ((mode & kModeCompact) && prm.compact_enqueued) return;
    uint32_t at_least[33];                                          // requests with lifetime >= 2^c
    at_least[32] = 0;
    for (int c = 31; c >= 0; --c) at_least[c] = at_least[c + 1] + hist[c];
    const uint32_t most = list_cap < n / 8 ? list_cap : n / 8;
    int c_min = 1;
    while (c_min <= kSpMaxThetaBits && at_least[c_min] > most) ++c_min;
    if (c_min > kSpMaxThetaBits) return;
    int c_best = c_min;
    for (int c = c_min + 1; c <= kSpMaxThetaBits; ++c)
        if (((1ull << c) - 1) * 2 * n <= 48ull * t_end) c_best = c;
    int c_sel = c_best;
    while (c_sel > c_min && at_least[c_sel - 1] == at_least[c_best]) --c_sel;
    const uint64_t theta = (1ull << c_sel) - 1;
    acc[kAccSplit] = 1ull | (theta << 8) | ((uint64_t)at_least[c_sel] << 32);
    *gate = 0;
}

// hist[kSpHistSizes + c] = short-lived requests whose size lies in [2^c, 2^(c+1)) granules.
__global__ void __launch_bounds__(256)
sp_size_histogram(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf,
                  uint32_t n, const uint64_t* acc, uint32_t* hist, const uint32_t* gate)
{
    __shared__ uint32_t local[32];
    if (*gate != 0) return;
    const uint32_t shift = (uint32_t)(acc[kAccMode] & 63);
    const uint32_t theta = (uint32_t)((acc[kAccSplit] >> 8) & 0xffffffu);
    if (threadIdx.x < 32) local[threadIdx.x] = 0;
    __syncthreads();
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint32_t s = (uint32_t)(size[i] >> shift);             // >= 1
        if (tf[i] - ta[i] <= theta) atomicAdd(&local[s ? 31 - __builtin_clz(s) : 0], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 32 && local[threadIdx.x]) atomicAdd(&hist[kSpHistSizes + threadIdx.x], local[threadIdx.x]);
}

// Short-lived blocks come in two kinds in a training trace: many small ones that settle low in
// the address space, and few large ones that end up anywhere (Sec. 2.3).  A long-lived request
// that looks for room high up is stopped by the large ones only, so those are also kept in a
// table of their own, which such a request reads whole.  sigma = 2^c with at most an eighth of the
// short-lived requests of at least that size (and at least one); of those c, the one with the
// most empty size classes right below it (the gap between the two kinds), the smallest of several
// such; none are large if even the largest occupied class holds more than an eighth.
__global__ void sp_sigma(uint32_t* hist, const uint32_t* gate)
{
    if (threadIdx.x != 0 || *gate != 0) return;
    uint32_t total = 0;
    for (int c = 0; c < 32; ++c) total += hist[kSpHistSizes + c];
    uint32_t above = 0, sigma = 0xffffffffu;
    int widest = -1;
    for (int c = 31; c >= 1; --c) {
        above += hist[kSpHistSizes + c];
        if (above > total / 8) break;
        if (above == 0) continue;
        int gap = 0;
        while (c - 1 - gap >= 0 && hist[kSpHistSizes + c - 1 - gap] == 0) ++gap;
        if (gap >= widest) { widest = gap; sigma = 1u << c; }
    }
    hist[kSpHistSigma] = sigma;
}

// For the list with ranks in place of times (RankedList): marks the allocation and release times of the
// long-lived requests (exclusive sums of the marks are the ranks and the counts A, B) and collects
// their sizes in a table of 64 classes.
__global__ void sp_clear_words(uint32_t* v, size_t m, const uint32_t* gate)
{
    if (*gate != 0) return;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < m; k += (size_t)gridDim.x * blockDim.x) v[k] = 0;
}

__global__ void __launch_bounds__(256)
sp_long_marks(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf, uint32_t n,
              const uint64_t* acc, uint32_t* allocated_at, uint32_t* released_at, uint32_t* class_size, uint32_t* hist,
              const uint32_t* gate)
{
    if (*gate != 0) return;
    const uint32_t shift = (uint32_t)(acc[kAccMode] & 63);
    const uint32_t theta = (uint32_t)((acc[kAccSplit] >> 8) & 0xffffffu);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        if (tf[i] - ta[i] <= theta) continue;
        atomicAdd(&allocated_at[ta[i]], 1u);
        atomicAdd(&released_at[tf[i]], 1u);
        const uint32_t s = (uint32_t)(size[i] >> shift);             // >= 1; 0 marks an empty class
        bool placed = false;
        for (int c = 0; c < kSpSizeClasses && !placed; ++c) {
            const uint32_t old = atomicCAS(&class_size[c], 0u, s);
            placed = old == 0u || old == s;
        }
        if (!placed) hist[kSpHistTooManySizes] = 1u;
    }
}

// acc[kAccSplit] bit 1: the list holds ranks in place of times (8-byte entries, three workgroups per CU).
// (sp_decide has admitted as many long-lived requests as the larger of the two lists holds: a trace
// that needs the ranked list for its length and cannot have it is left to the sorted-list kernel.)
__global__ void sp_ranked_decide(uint64_t* acc, const uint32_t* hist, uint32_t list_cap, uint32_t ranked_cap, uint32_t* gate)
{
    if (threadIdx.x != 0 || *gate != 0) return;
    const uint32_t longs = (uint32_t)(acc[kAccSplit] >> 32);
    if (hist[kSpHistTooManySizes] == 0 && longs <= kSpRankedMost && longs <= ranked_cap) acc[kAccSplit] |= 2ull;
    else if (longs > list_cap) { acc[kAccSplit] = 0; *gate = 1; }
}

// Keys (t_alloc, request) of one tile, sorted in LDS.
__global__ void __launch_bounds__(kSortTile)
sp_sort_tiles(const uint32_t* __restrict__ ta, uint32_t n, ulonglong2* keys, const uint32_t* gate)
{
    __shared__ ulonglong2 k[kSortTile];
    if (*gate != 0) return;
    const uint32_t e = blockIdx.x * kSortTile + threadIdx.x;
    k[threadIdx.x] = e < n ? make_ulonglong2((uint64_t)ta[e], (uint64_t)e) : filler_key(e);
    sort_tile(k);
    keys[e] = k[threadIdx.x];
}

// Per rank k of the allocation-time order: (size in granules, t_alloc, t_free, request); the
// slots past the end conflict with nothing.  Per request: its rank, flagged when it is long.
__global__ void __launch_bounds__(256)
sp_tables(const ulonglong2* __restrict__ sorted, const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta,
          const uint32_t* __restrict__ tf, uint32_t n, uint32_t slots, const uint64_t* acc, uint4* by_rank,
          uint32_t* size_by_rank, uint2* fit_by_rank, uint32_t* rank_of, uint32_t* is_large, const uint32_t* hist,
          const uint32_t* gate)
{
    if (*gate != 0) return;
    const uint32_t shift = (uint32_t)(acc[kAccMode] & 63);
    const uint32_t theta = (uint32_t)((acc[kAccSplit] >> 8) & 0xffffffu);
    const uint32_t sigma = hist[kSpHistSigma];
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < slots; k += gridDim.x * blockDim.x) {
        if (k >= n) {
            by_rank[k] = make_uint4(0u, 0xffffffffu, 0u, 0xffffffffu);
            size_by_rank[k] = 0u;
            fit_by_rank[k] = make_uint2(0u, 0u);
            is_large[k] = 0u;
            continue;
        }
        const uint32_t i = (uint32_t)sorted[k].y;
        const uint32_t a = ta[i], f = tf[i];
        const uint32_t s = (uint32_t)(size[i] >> shift);
        const bool lives_long = f - a > theta, large = !lives_long && s >= sigma;
        by_rank[k] = make_uint4(s, a, f, i);
        size_by_rank[k] = s;
        fit_by_rank[k] = make_uint2(s, f);
        is_large[k] = large ? 1u : 0u;
        rank_of[i] = k | (lives_long ? kSpLongFlag : 0u) | (large ? kSpLargeFlag : 0u);
    }
}

// First rank whose allocation time is >= t.
__device__ __forceinline__ uint32_t first_rank_at(const uint4* __restrict__ by_rank, uint32_t n, uint32_t t)
{
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (by_rank[mid].y < t) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Second word of a request's record: (window start, window end, for a large short block its place
// among the large short blocks in allocation-time order, -); with a ranked list: (.., .., for a
// long-lived request the second word of its list entry, A | B << 16).
// Window of request i: ranks of the requests allocated in (t_alloc - theta, t_free).  A short
// request j (lifetime <= theta) whose lifetime conflicts with i's has t_alloc_j < t_free_i and
// t_alloc_j >= t_free_j - theta > t_alloc_i - theta, so it lies in the window.
__global__ void __launch_bounds__(256)
sp_windows(const uint4* __restrict__ by_rank, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf, uint32_t n,
           const uint64_t* acc, const uint64_t* __restrict__ size, const uint32_t* __restrict__ rank_of,
           const uint32_t* __restrict__ large_before, const uint32_t* __restrict__ allocated_before,
           const uint32_t* __restrict__ released_before, const uint32_t* __restrict__ class_size, uint4* record,
           uint2* large_fit, uint32_t* hist, const uint32_t* gate)
{
    if (*gate != 0) return;
    const uint32_t theta = (uint32_t)((acc[kAccSplit] >> 8) & 0xffffffu);
    const bool ranked = (acc[kAccSplit] & 2) != 0;
    uint32_t wide = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint32_t a = ta[i];
        const uint32_t from = a + 1 > theta ? a + 1 - theta : 0u;
        const uint2 w = make_uint2(first_rank_at(by_rank, n, from), first_rank_at(by_rank, n, tf[i]));
        record[2 * i] = make_uint4((uint32_t)(size[i] >> (acc[kAccMode] & 63)), a, tf[i], rank_of[i]);
        // large_before[k] = large short blocks among the ranks below k: a large short block's place in
        // the table of those
        const bool large = (rank_of[i] & kSpLargeFlag) != 0;
        uint32_t extra = large ? large_before[rank_of[i] & kSpRankMask] : 0u, counts = 0u;
        const uint32_t place = extra;
        if (ranked) {
            // allocated_before[t] = long-lived requests allocated before t, released_before[t] = released before t
            counts = allocated_before[tf[i]] | (released_before[a + 1] << 16);
            if (rank_of[i] & kSpLongFlag) {
                const uint32_t s = (uint32_t)(size[i] >> (acc[kAccMode] & 63));
                uint32_t cls = 0;
                while (cls < (uint32_t)kSpSizeClasses - 1 && class_size[cls] != s) ++cls;
                extra = allocated_before[a] | ((released_before[tf[i]] + 1u) << kSpRankBits) | (cls << (2 * kSpRankBits));
            }
        }
        record[2 * i + 1] = make_uint4(w.x, w.y, extra, counts);
        if (large) large_fit[place] = make_uint2((uint32_t)(size[i] >> (acc[kAccMode] & 63)), tf[i]);
        wide += w.y - w.x > (uint32_t)kWave ? 1u : 0u;
    }
    wide = wave_sum32(wide);
    if (lane_id() == 0 && wide) atomicAdd(&hist[kSpHistWide], wide);
}

// A request whose window is wider than a wave is settled by the whole workgroup, with look-ups
// in the table for every step it moves up: affordable for the few long-lived requests this
// kernel is meant for, not when timestamps are so dense (or tied) that short-lived requests
// have such windows too.  Then the sorted-list kernel places the trace after all.
__global__ void sp_confirm(uint64_t* acc, const uint32_t* hist, uint32_t n, uint32_t* gate)
{
    if (threadIdx.x != 0 || *gate != 0) return;
    const uint32_t longs = (uint32_t)(acc[kAccSplit] >> 32);
    if ((uint64_t)hist[kSpHistWide] > 2ull * longs + 64 || (uint64_t)hist[kSpHistWide] * 8 > n) {
        acc[kAccSplit] = 0;
        *gate = 1;
    }
}

// ------------------------------------------------------------------------------------------
// The placement kernel.

struct SplitTables {
    const uint4* by_rank;        // [slots] (size, t_alloc, t_free, request) in allocation-time order
    const uint32_t* size_by_rank;// [slots] the sizes once more, on their own
    const uint2* fit_by_rank;    // [slots] (size, t_free): what a request needs to know of the short blocks of its window
    const uint4* record;         // [n] per request: (size, t_alloc, t_free, rank | long flag), then (window start, window end, -, -)
    const uint32_t* large_before;// [slots] large short blocks among the ranks below
    const uint2* large_fit;      // [large_slots] (size, t_free) of the large short blocks in allocation-time order
    uint32_t* addr;              // per resident workgroup: [slots] address of the short block at each rank
    uint2* group_span;           // per resident workgroup: [groups] lowest start, highest end address of the placed small short blocks of 64 ranks
    uint32_t* large_addr;        // per resident workgroup: [large_slots] addresses of the large short blocks
    uint32_t large_slots;        // a multiple of 64
    uint32_t slots;              // n rounded up to 64, plus 64
    uint32_t groups;             // slots / 64
    uint32_t list_cap;           // entries of the LDS list
    uint32_t region_shift;       // 2^region_shift ranks share one summary in LDS; at most 64 regions cover all slots
    uint32_t* next_plan;         // [1] plans handed out so far
    const uint32_t* sigma;       // [1] size from which a short-lived block counts as large
    const uint32_t* large_total; // [1] how many do
    const uint32_t* class_size;  // [64] ranked list: sizes of the long-lived requests' size classes
};

// What one wave knows about the request it settles.
struct SpRequest {
    uint32_t s, ta, tf;
    uint32_t list_a, list_b;         // a listed block conflicts in lifetime if block.ta() < list_a and list_b < block.tf():
                                     // (t_free, t_alloc) of the request, or its counts (A, B) with a ranked list
    uint32_t wlo, whi;
    uint32_t large_lo, large_hi;     // the window in the table of large short blocks (wide windows only)
    // blocks settled earlier in the batch (lane = position in the batch)
    uint64_t rivals_in;
    uint32_t in_lo, in_hi;
    // short blocks of the window (lane = rank - wlo), when it fits the wave
    uint64_t rivals_w;
    uint32_t w_lo, w_hi;
};

// The table of short blocks of the plan a workgroup is working on.
struct SpTable {
    uint32_t* addr;
    uint2* group_span;
    uint32_t* large_addr;
};

// (changed with atomic operations by one wave of the workgroup, read by all after a barrier)
__device__ __forceinline__ uint32_t load_coherent(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Highest end address of the placed short blocks of the window that conflict with the request
// in lifetime and meet [c, c + s); 0 if none does.  Called by ALL waves of the workgroup with the
// same arguments; every wave returns the same value.
//   small blocks: regions of ranks first (lowest start / highest end in LDS), then the groups of 64
//                 ranks of the regions that are left (lowest start / highest end), then the blocks
//                 of a group;
//   large blocks: all of the window, from the table of their own.
// Groups are dealt out to the waves in turn; `turn` counts the calls of the workgroup (the results
// of three consecutive calls use different LDS words, so that one barrier per call suffices).
template <int kWaves, typename Lds>
__device__ __forceinline__ uint32_t window_reach(const SpRequest& rq, uint32_t own_rank, uint32_t c, const SplitTables& tb,
                                                 const SpTable& pt, uint32_t& turn, Lds& sh)
{
    const int lane = lane_id(), wave = wave_id();
    const uint32_t cs = c + rq.s;
    const uint32_t g_begin = rq.wlo / kWave, g_end = (rq.whi + kWave - 1) / kWave;     // groups of the window
    const uint32_t region_of_group = tb.region_shift - 6;                               // 2^that groups per region
    const uint32_t r_begin = g_begin >> region_of_group, r_end = ((g_end - 1) >> region_of_group) + 1;   // <= 64
    const uint64_t regions = __builtin_amdgcn_ballot_w64((uint32_t)lane >= r_begin && (uint32_t)lane < r_end &&
                                                         sh.region_max[lane] > c && sh.region_min[lane] < cs);
    const bool large = rq.large_lo < rq.large_hi && sh.large_max > c && sh.large_min < cs;
    if (regions == 0 && !large) return 0;                                               // (the same in every wave)
    const uint32_t slot = turn % 3;
    ++turn;
    if (threadIdx.x == 0) sh.reach[(slot + 1) % 3] = 0;                                 // for the call after this one
    uint32_t reach = 0;
    constexpr int kFlight = 4;                                                          // groups whose reads are under way together
    if (large) {
        const uint32_t l_begin = rq.large_lo / kWave, l_end = (rq.large_hi + kWave - 1) / kWave;
        for (uint32_t g0 = l_begin + (uint32_t)wave; g0 < l_end; g0 += kFlight * kWaves) {
            uint32_t a[kFlight];
            uint2 fit[kFlight];
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const uint32_t k = umin(g0 + (uint32_t)u * kWaves, l_end - 1) * kWave + lane;      // < large_slots
                a[u] = pt.large_addr[k];
                fit[u] = tb.large_fit[k];
            }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                const uint32_t k = (g0 + (uint32_t)u * kWaves) * kWave + lane;
                // (a block of the window was allocated before the request is released: only its release counts)
                const bool live = k >= rq.large_lo && k < rq.large_hi && a[u] != kSpUnplaced && fit[u].y > rq.ta;
                reach = umax(reach, (live && a[u] < cs && a[u] + fit[u].x > c) ? a[u] + fit[u].x : 0u);
            }
        }
    }
    // wave w takes the groups g_begin + w, g_begin + w + kWaves, ...: neighbouring groups hold blocks of
    // the same phase of the trace and tend to be busy together
    for (uint32_t g0 = g_begin + (uint32_t)wave; regions != 0 && g0 < g_end; g0 += kWave * kWaves) {
        const uint32_t g = g0 + (uint32_t)lane * kWaves;
        const bool valid = g < g_end && ((regions >> umin(g >> region_of_group, 63u)) & 1);
        uint2 span = make_uint2(0xffffffffu, 0u);
        if (valid) {
            span.x = load_coherent(&pt.group_span[g].x);
            span.y = load_coherent(&pt.group_span[g].y);
        }
        // nothing of the group reaches into [c, c + s): not concerned
        bool look = span.y > c && span.x < cs;
        // every block of the group ends by c + s, so all of them start below it, and the highest end
        // is that of a block meeting [c, c + s): no need to read the blocks.  (Only for groups whose
        // ranks all lie in the window and above the request's own: those started during its lifetime.)
        if (look && span.y <= cs && g * kWave > own_rank && (g + 1) * kWave <= rq.whi) {
            reach = umax(reach, span.y);
            look = false;
        }
        uint64_t open = __builtin_amdgcn_ballot_w64(look);
        while (open) {
            uint32_t k[kFlight], a[kFlight], sz[kFlight];
            bool on[kFlight];
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                on[u] = open != 0;
                k[u] = on[u] ? (g0 + (uint32_t)__builtin_ctzll(open) * kWaves) * kWave + lane : k[0];      // < slots
                open &= open - 1;
            }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) { a[u] = pt.addr[k[u]]; sz[u] = tb.size_by_rank[k[u]]; }
#pragma unroll
            for (int u = 0; u < kFlight; ++u) {
                // ranks above the request's own started during its lifetime; the few below need a look at their release time
                bool live = on[u] && k[u] >= rq.wlo && k[u] < rq.whi && a[u] != kSpUnplaced;
                if (k[u] - lane <= own_rank) live = live && tb.by_rank[k[u]].z > rq.ta;
                reach = umax(reach, (live && a[u] < cs && a[u] + sz[u] > c) ? a[u] + sz[u] : 0u);
            }
        }
    }
    reach = read_lane(wave_scan_max(reach), kWave - 1);
    if (lane == 0 && reach) atomicMax(&sh.reach[slot], reach);
    __syncthreads();
    return sh.reach[slot];
}

// Lowest address >= c at which [c, c + s) meets no conflicting block other than the long blocks
// of the list; gives up (returns something > limit - s) once the request cannot end by `limit`.
// kWide: the request's window is looked up in the table itself, by the whole workgroup.
template <bool kWide, int kWaves, typename Lds>
__device__ __forceinline__ uint32_t clear_others(const SpRequest& rq, uint32_t own_rank, uint32_t c, uint32_t limit,
                                                 const SplitTables& tb, const SpTable& pt, uint32_t& turn, Lds& sh)
{
    for (;;) {
        if (c > limit || limit - c < rq.s) return c;                              // (uniform)
        const uint32_t cs = c + rq.s;
        const uint64_t hit_in = rq.rivals_in & lanes_lt(rq.in_lo, cs) & lanes_lt(c, rq.in_hi);
        const uint64_t hit_w = rq.rivals_w & lanes_lt(rq.w_lo, cs) & lanes_lt(c, rq.w_hi);
        if (hit_in | hit_w) {
            const uint32_t ends = umax(keep_lanes(hit_in, rq.in_hi), keep_lanes(hit_w, rq.w_hi));
            c = read_lane(wave_scan_max(ends), kWave - 1);
            continue;
        }
        if constexpr (!kWide) {
            return c;
        } else {
            const uint32_t reach = window_reach<kWaves>(rq, own_rank, c, tb, pt, turn, sh);
            if (reach == 0) return c;
            c = reach;
        }
    }
}

// The requests of the batch as the lanes of a wave hold them (lane = position in the batch).
struct SpBatch {
    uint32_t size, ta, tf, rank, wlo, whi, counts;
};

template <typename List>
__device__ __forceinline__ void list_operands(SpRequest& rq, uint32_t counts)
{
    if constexpr (ListTraits<List>::kRanked) { rq.list_a = counts & 0xffffu; rq.list_b = counts >> 16; }
    else { rq.list_a = rq.tf; rq.list_b = rq.ta; }
}

// Settles request q of the batch: the lowest address at which it conflicts with nothing placed
// before it.  A request whose window fits the lanes of a wave (kWide false) is settled by one
// wave; one with a wider window by all waves of the workgroup together, every wave taking the
// same steps (they read the same LDS) and sharing only the look-ups in the table.
template <bool kWide, int kWaves, typename List, typename Lds>
__device__ __forceinline__ uint32_t settle_request(const List& list, uint32_t count, uint32_t b0, uint32_t q,
                                                   uint64_t dep_q, const SpBatch& bt, uint32_t pool_first, uint32_t in_pool,
                                                   const SplitTables& tb, const SpTable& pt, uint32_t& turn, Lds& sh)
{
    const int lane = lane_id();
    SpRequest rq;
    rq.s = read_lane(bt.size, (int)q); rq.ta = read_lane(bt.ta, (int)q); rq.tf = read_lane(bt.tf, (int)q);
    rq.wlo = read_lane(bt.wlo, (int)q); rq.whi = read_lane(bt.whi, (int)q);
    list_operands<List>(rq, read_lane(bt.counts, (int)q));
    const uint32_t own_rank = read_lane(bt.rank, (int)q) & kSpRankMask;
    // What the first step needs from LDS is asked for in one go: the addresses of the batch, the
    // request's part of the pool, the lowest 64 blocks of the list.
    const uint32_t batch_addr = sh.rq_addr[b0 + lane];
    Span<uint32_t> pooled = {0u, 0u};
    if constexpr (!kWide) pooled = sh.pool[umin(pool_first + (uint32_t)lane, (uint32_t)kSpPool - 1)];
    typename List::Entry en = list.load(umin((uint32_t)lane, count ? count - 1 : 0u));
    // earlier requests of the batch with a conflicting lifetime: all settled by now (the mask says which lanes count)
    rq.rivals_in = dep_q;
    rq.in_lo = batch_addr;
    rq.in_hi = batch_addr + bt.size;
    rq.rivals_w = 0; rq.w_lo = 0; rq.w_hi = 0;
    rq.large_lo = 0; rq.large_hi = 0;
    if constexpr (kWide) {
        rq.large_lo = tb.large_before[rq.wlo];
        rq.large_hi = tb.large_before[rq.whi];
    }
    if constexpr (!kWide) {
        // conflicting short blocks of its window, as gathered when the batch began
        if (in_pool != kSpRefetch) {
            rq.rivals_w = in_pool >= (uint32_t)kWave ? ~0ull : (1ull << in_pool) - 1;
            rq.w_lo = pooled.lo;
            rq.w_hi = pooled.hi;
        } else {
            const uint32_t k = rq.wlo + lane;                       // < slots
            const uint32_t a = pt.addr[k];
            const uint4 rec = tb.by_rank[k];
            rq.rivals_w = __builtin_amdgcn_ballot_w64(k < rq.whi && a != kSpUnplaced && rec.z > rq.ta && rec.y < rq.tf);
            rq.w_lo = a;
            rq.w_hi = a + rec.x;
        }
    }
    // walk over the long blocks, in address order
    uint32_t run = 0;
    for (uint32_t k0 = 0; k0 < count; k0 += kWave) {
        const uint32_t k = k0 + lane;
        const bool valid = k < count;
        // (the blocks of the next step are asked for before this step's are looked at)
        typename List::Entry next = en;
        if (k0 + kWave < count) next = list.load(umin(k + kWave, count - 1));
        const bool conflict = valid && en.ta() < rq.list_a && rq.list_b < en.tf();
        const uint32_t incl = wave_scan_max(conflict ? en.hi() : 0u);
        const uint32_t before = umax(run, wave_shift_up(incl, 0u));
        // a hole [before, lo) in front of a conflicting block, large enough as such
        uint64_t opens = __builtin_amdgcn_ballot_w64(conflict && en.lo() >= before && en.lo() - before >= rq.s);
        while (opens) {
            const int f = __builtin_ctzll(opens);
            opens &= opens - 1;
            const uint32_t limit = read_lane(en.lo(), f);
            const uint32_t c = clear_others<kWide, kWaves>(rq, own_rank, read_lane(before, f), limit, tb, pt, turn, sh);
            if (c <= limit && limit - c >= rq.s) return c;
        }
        run = umax(run, read_lane(incl, kWave - 1));
        en = next;
    }
    return clear_others<kWide, kWaves>(rq, own_rank, run, 0xffffffffu, tb, pt, turn, sh);     // on top of every conflicting long block
}

// Up to four requests with narrow windows settled at once, each by one row of 16 lanes of the
// wave: the same steps as settle_request (walk over the long blocks, here 16 a step, holes in
// address order, moving up past the other conflicting blocks that reach into [c, c + size)), taken
// by the four rows side by side; a row that is done waits for the others.  `group` holds the
// requests (bits = places in the batch); each has at most 16 other conflicting blocks to look
// at -- its part of the pool and the requests of the batch settled before it.  The addresses go
// to sh.rq_addr, the extent to sh.peak.
template <typename List, typename Lds>
__device__ __forceinline__ void settle_rows(const List& list, uint32_t count, uint32_t b0, uint64_t group, uint64_t dep,
                                            const SpBatch& bt, uint32_t part_first, uint32_t part_count, Lds& sh)
{
    const int lane = lane_id();
    const uint32_t row = (uint32_t)lane >> 4, at = (uint32_t)lane & 15u, row_first = row * 16u;
    // the row's request: the row-th of the group
    const uint64_t g1 = group & (group - 1), g2 = g1 & (g1 - 1), g3 = g2 & (g2 - 1);
    const uint32_t q0 = (uint32_t)__builtin_ctzll(group), q1 = g1 ? (uint32_t)__builtin_ctzll(g1) : 0u,
                   q2 = g2 ? (uint32_t)__builtin_ctzll(g2) : 0u, q3 = g3 ? (uint32_t)__builtin_ctzll(g3) : 0u;
    const uint32_t q = row == 0 ? q0 : row == 1 ? q1 : row == 2 ? q2 : q3;
    const bool active = row < (uint32_t)__builtin_popcountll(group);
    const uint32_t s = lane_gather(bt.size, (int)q);
    uint32_t list_a, list_b;                                          // (see SpRequest)
    if constexpr (ListTraits<List>::kRanked) {
        const uint32_t counts = lane_gather(bt.counts, (int)q);
        list_a = counts & 0xffffu; list_b = counts >> 16;
    } else {
        list_a = lane_gather(bt.tf, (int)q); list_b = lane_gather(bt.ta, (int)q);
    }
    const uint32_t in_pool = lane_gather(part_count, (int)q), pool_at = lane_gather(part_first, (int)q);
    uint64_t before_it = lane_gather(dep, (int)q);                    // earlier requests of the batch with a conflicting lifetime
    // the other blocks the request has to keep clear of, one per lane of the row
    uint32_t r_lo = 0xffffffffu, r_hi = 0u;
    if (active) {
        if (at < in_pool) {
            const Span<uint32_t> sp = sh.pool[pool_at + at];
            r_lo = sp.lo; r_hi = sp.hi;
        } else if (at - in_pool < (uint32_t)__builtin_popcountll(before_it)) {
            for (uint32_t t = at - in_pool; t > 0; --t) before_it &= before_it - 1;
            const uint32_t e = (uint32_t)__builtin_ctzll(before_it);
            r_lo = sh.rq_addr[b0 + e];
            r_hi = r_lo + sh.rq_size[b0 + e];
        }
    }
    // Lowest address >= c at which [c, c + s) meets none of them; stops once the request cannot end by `limit`.
    auto clear_others_in_rows = [&](uint32_t c, uint32_t limit, bool trying) -> uint32_t {
        for (;;) {
            const bool fits = trying && c <= limit && limit - c >= s;
            const bool hit = fits && r_lo < c + s && c < r_hi;
            const uint64_t hits = __builtin_amdgcn_ballot_w64(hit);
            if (hits == 0) return c;                                  // (uniform)
            const uint32_t reach = row_max(hit ? r_hi : 0u);
            c = umax(c, reach);                                       // (reach > c in a row with a hit, 0 in the others)
        }
    };
    uint32_t run = 0, x = 0;
    bool settled = !active;
    for (uint32_t k0 = 0; k0 < count; k0 += 16) {
        if (__builtin_amdgcn_ballot_w64(!settled) == 0) break;        // (uniform)
        const uint32_t k = k0 + at;
        const bool valid = k < count;
        const typename List::Entry en = list.load(valid ? k : count - 1);
        const bool conflict = valid && en.ta() < list_a && list_b < en.tf();
        const uint32_t incl = row_scan_max(conflict ? en.hi() : 0u);
        const uint32_t before = umax(run, row_shift_up(incl, 0u));
        // a hole [before, lo) in front of a conflicting block, large enough as such
        const uint64_t opens = __builtin_amdgcn_ballot_w64(!settled && conflict && en.lo() >= before && en.lo() - before >= s);
        uint32_t holes = (uint32_t)(opens >> row_first) & 0xffffu;
        for (;;) {
            const bool trying = holes != 0 && !settled;
            if (__builtin_amdgcn_ballot_w64(trying) == 0) break;      // (uniform)
            const int from = (int)(row_first + (trying ? (uint32_t)__builtin_ctz(holes) : 0u));
            const uint32_t limit = lane_gather(en.lo(), from);
            const uint32_t c = clear_others_in_rows(lane_gather(before, from), limit, trying);
            if (trying && c <= limit && limit - c >= s) { settled = true; x = c; }
            holes &= holes - 1;
        }
        run = umax(run, lane_gather(incl, (int)row_first + 15));
    }
    if (__builtin_amdgcn_ballot_w64(!settled)) {                      // on top of every conflicting long block
        const uint32_t c = clear_others_in_rows(run, 0xffffffffu, !settled);
        if (!settled) x = c;
    }
    if (active && at == 0) {
        sh.rq_addr[b0 + q] = x;
        atomicMax(&sh.peak, x + s);
    }
}

// A request with a wide window, settled by the whole workgroup: the waves walk one part of the
// list of long blocks each and write down the holes that are large enough as such; then all
// waves try them in address order, sharing the look-ups in the table of short blocks.  Called by
// all waves.
template <int kWaves, typename List, typename Lds>
__device__ __forceinline__ uint32_t settle_wide(const List& list, uint32_t count, uint32_t b0, uint32_t q, uint64_t dep_q,
                                                const SpBatch& bt, const SplitTables& tb, const SpTable& pt, uint32_t& turn,
                                                uint32_t& wide_turn, Lds& sh)
{
    const int lane = lane_id();
    SpRequest rq;
    rq.s = read_lane(bt.size, (int)q); rq.ta = read_lane(bt.ta, (int)q); rq.tf = read_lane(bt.tf, (int)q);
    rq.wlo = read_lane(bt.wlo, (int)q); rq.whi = read_lane(bt.whi, (int)q);
    list_operands<List>(rq, read_lane(bt.counts, (int)q));
    const uint32_t own_rank = read_lane(bt.rank, (int)q) & kSpRankMask;
    rq.rivals_in = dep_q;
    rq.in_lo = sh.rq_addr[b0 + lane];
    rq.in_hi = rq.in_lo + bt.size;
    rq.rivals_w = 0; rq.w_lo = 0; rq.w_hi = 0;
    rq.large_lo = tb.large_before[rq.wlo];                        // (looked at after the walk over the list)
    rq.large_hi = tb.large_before[rq.whi];
    const uint32_t set = wide_turn & 1u;                          // (the set before the last one's: a barrier has passed since it was read)
    ++wide_turn;
    // Every wave takes one part of the list and writes down what may be a hole large enough as such,
    // as seen from the part's start, and the highest end of the part's conflicting blocks; what the
    // parts below cover is known once all waves are done, and decides which of them are holes.
    const int wave = wave_id();
    const uint32_t steps = (count + kWave - 1) / kWave, per_wave = (steps + kWaves - 1) / kWaves;
    const uint32_t k_begin = umin(count, (uint32_t)wave * per_wave * kWave), k_end = umin(count, k_begin + per_wave * kWave);
    {
        uint32_t run = 0, found = 0;
        for (uint32_t k0 = k_begin; k0 < k_end; k0 += kWave) {
            const uint32_t k = k0 + lane;
            const bool valid = k < k_end;
            const typename List::Entry en = list.load(valid ? k : k_end - 1);
            const bool conflict = valid && en.ta() < rq.list_a && rq.list_b < en.tf();
            const uint32_t incl = wave_scan_max(conflict ? en.hi() : 0u);
            const uint32_t before = umax(run, wave_shift_up(incl, 0u));
            const uint64_t opens = __builtin_amdgcn_ballot_w64(conflict && en.lo() >= before && en.lo() - before >= rq.s);
            const uint32_t at = found + lanes_below(opens);
            if (((opens >> lane) & 1) && at < (uint32_t)kSpWideHoles) sh.wide_hole[set][wave][at] = Span<uint32_t>{en.lo(), before};
            found += (uint32_t)__builtin_popcountll(opens);
            run = umax(run, read_lane(incl, kWave - 1));
        }
        if (lane == 0) { sh.wide_holes[set][wave] = found; sh.wide_part_top[set][wave] = run; }
    }
    __syncthreads();
    not_before_here(rq.large_lo);                                     // (the two reads had the walk's time to arrive)
    not_before_here(rq.large_hi);
    // All candidates at once, lane 8 w + i holding candidate i of part w (address order = lane order):
    // what the parts below a part cover is a running maximum over the parts' highest ends, and a
    // candidate is a hole if the request fits between that (or what its own part covers in front of
    // it) and the block behind it.
    static_assert(kSpWideHoles <= 7 && kWaves * 8 <= kWave, "eight lanes per part, the last one for the part's highest end");
    const uint32_t part = (uint32_t)lane >> 3, slot = (uint32_t)lane & 7u;
    uint32_t found = 0, part_top = 0;
    Span<uint32_t> hole = {0u, 0u};                                   // {end, covered within the part}
    if (part < (uint32_t)kWaves) {
        found = sh.wide_holes[set][part];
        part_top = sh.wide_part_top[set][part];
        if (slot < (uint32_t)kSpWideHoles) hole = sh.wide_hole[set][part][slot];
    }
    const uint32_t tops = wave_scan_max(slot == 7u ? part_top : 0u);  // in a part's first seven lanes: the parts below
    const uint32_t covered = umax(hole.hi, tops);
    uint64_t holes = __builtin_amdgcn_ballot_w64(slot < umin(found, (uint32_t)kSpWideHoles) && hole.lo >= covered &&
                                                 hole.lo - covered >= rq.s);
    // parts with more candidates than were written down (bit 8 w): if none of the holes up to the end
    // of such a part takes the request, every wave walks the list
    const uint64_t more = __builtin_amdgcn_ballot_w64(slot == 0u && found > (uint32_t)kSpWideHoles);
    while (holes) {
        const int at = __builtin_ctzll(holes);
        holes &= holes - 1;
        if (more & ((1ull << (at & ~7)) - 1)) break;                  // (a part below this one has more)
        const uint32_t end = read_lane(hole.lo, at);
        const uint32_t c = clear_others<true, kWaves>(rq, own_rank, read_lane(covered, at), end, tb, pt, turn, sh);
        if (c <= end && end - c >= rq.s) return c;
    }
    if (more) return settle_request<true, kWaves>(list, count, b0, q, dep_q, bt, 0u, 0u, tb, pt, turn, sh);
    return clear_others<true, kWaves>(rq, own_rank, read_lane(tops, kWave - 1), 0xffffffffu, tb, pt, turn, sh);
}

// kRanked: the list holds ranks in place of times (RankedList, 8 bytes a block) and three workgroups
// share a CU (six waves per SIMD: 80 registers); else 16 bytes a block and two workgroups.  Both are
// enqueued; acc[kAccSplit] bit 1 says which one works.
template <int kThreads, bool kRanked>
__global__ void __launch_bounds__(kThreads, kRanked ? 6 : 4) plan_split_kernel(PlanParams prm, SplitTables tb)
{
    using List = typename std::conditional<kRanked, RankedList, SpList>::type;
    static_assert(kThreads / kWave <= kSpMaxWaves, "a wave's part of the list has its own LDS words");
    constexpr int kWaves = kThreads / kWave;
    extern __shared__ __align__(16) unsigned char smem[];
    SplitLds& sh = *reinterpret_cast<SplitLds*>(smem);
    const uint32_t n = prm.n;
    if (*prm.status != STALLOC_OK) return;
    if (!(prm.acc[kAccSplit] & 1)) return;                            // another kernel places this trace
    if (((prm.acc[kAccSplit] & 2) != 0) != kRanked) return;           // the other form of the list does
    const uint64_t mode = prm.acc[kAccMode];
    const bool try32 = (mode & kModeTry32) != 0;
    const uint32_t shift = (uint32_t)(mode & 63);
    const int lane = lane_id(), wave = wave_id();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const_cast<uint64_t*>(prm.acc)[kAccKernel] = STALLOC_KERNEL_LONG_LIST | (32u << 8) | ((uint64_t)List::kEntryBytes << 16);
        const_cast<uint64_t*>(prm.acc)[kAccLargeShort] = (uint64_t)*tb.sigma | ((uint64_t)*tb.large_total << 32);
    }
    List list, spare;
    list.bind(smem + sizeof(SplitLds), tb.list_cap);
    if constexpr (kRanked) {
        list.class_size = sh.class_size;
        if (threadIdx.x < kSpSizeClasses) sh.class_size[threadIdx.x] = tb.class_size[threadIdx.x];   // (barriers follow)
    }
    spare = list;
    SpTable pt;
    pt.addr = tb.addr + (size_t)blockIdx.x * tb.slots;
    pt.group_span = tb.group_span + (size_t)blockIdx.x * tb.groups;
    pt.large_addr = tb.large_addr + (size_t)blockIdx.x * tb.large_slots;
    uint32_t* addr = pt.addr;

    // Plans are handed out one by one (a counter in the workspace): some orders take several times
    // longer than others (long chains of requests that wait for each other), and the first rows are such.
    for (;;) {
        __syncthreads();                                              // every wave is done with the previous plan
        if (threadIdx.x == 0) sh.next_plan = atomicAdd(tb.next_plan, 1u);
        __syncthreads();
        const uint32_t p = sh.next_plan;
        if (p >= prm.P) break;                                        // (uniform)
        const uint32_t* order = prm.orders + (size_t)p * n;
        uint64_t* out = prm.offsets ? prm.offsets + (size_t)p * n : nullptr;
        uint32_t count = 0;
        bool outgrown = false;                                        // (uniform) 32-bit counts may not hold the next batch
        for (uint32_t k = threadIdx.x; k < tb.slots; k += kThreads) addr[k] = kSpUnplaced;
        for (uint32_t k = threadIdx.x; k < tb.large_slots; k += kThreads) pt.large_addr[k] = kSpUnplaced;
        for (uint32_t g = threadIdx.x; g < tb.groups; g += kThreads) pt.group_span[g] = make_uint2(0xffffffffu, 0u);
        if (threadIdx.x < kWave) { sh.region_min[threadIdx.x] = 0xffffffffu; sh.region_max[threadIdx.x] = 0u; }
        if (threadIdx.x == 0) { sh.extent_now = 0; sh.peak = 0; sh.pool_used = 0; sh.reach[0] = 0; sh.large_min = 0xffffffffu; sh.large_max = 0u; }
        uint32_t turn = 0;                                            // calls of window_reach: slot 0 is clear
        uint32_t wide_turn = 0;                                       // requests settled by the whole workgroup
        uint32_t round = 0;                                           // rounds so far: which wave takes the first ready request

        for (uint32_t r0 = 0; r0 < n; r0 += kSpRefill) {
            const uint32_t staged = n - r0 < (uint32_t)kSpRefill ? n - r0 : (uint32_t)kSpRefill;
            __syncthreads();                                          // previous refill fully consumed
            if (threadIdx.x < staged) {
                uint32_t i = order[r0 + threadIdx.x];
                if (i >= n) { atomicMax(prm.status, (uint32_t)STALLOC_ERR_BAD_ORDER); i = 0; }
                const uint4 r0 = tb.record[2 * (size_t)i], r1 = tb.record[2 * (size_t)i + 1];    // one 32-byte read
                sh.rq_id[threadIdx.x] = i;
                sh.rq_size[threadIdx.x] = r0.x;
                sh.rq_ta[threadIdx.x] = r0.y;
                sh.rq_tf[threadIdx.x] = r0.z;
                sh.rq_rank[threadIdx.x] = r0.w;
                sh.rq_wlo[threadIdx.x] = r1.x;
                sh.rq_whi[threadIdx.x] = r1.y;
                sh.rq_extra[threadIdx.x] = r1.z;
                sh.rq_counts[threadIdx.x] = r1.w;
            }
            if (threadIdx.x < kSpBatch) sh.dep[threadIdx.x] = 0;
            __syncthreads();

            for (uint32_t b0 = 0; b0 < staged; b0 += kSpBatch) {
                vector_memory_done();     // (the previous batch's accesses: the window reads below go out as one run)
                const uint32_t nb = staged - b0 < (uint32_t)kSpBatch ? staged - b0 : (uint32_t)kSpBatch;
                const bool mine = lane < (int)nb;
                const uint32_t my_size = mine ? sh.rq_size[b0 + lane] : 0u;
                const uint32_t my_ta = mine ? sh.rq_ta[b0 + lane] : 0xffffffffu;      // an empty lifetime otherwise
                const uint32_t my_tf = mine ? sh.rq_tf[b0 + lane] : 0u;
                const uint32_t my_rank = mine ? sh.rq_rank[b0 + lane] : 0u;
                const uint32_t my_wlo = mine ? sh.rq_wlo[b0 + lane] : 0u;
                const uint32_t my_whi = mine ? sh.rq_whi[b0 + lane] : 0u;
                const uint32_t my_counts = mine ? sh.rq_counts[b0 + lane] : 0u;
                const SpBatch bt = {my_size, my_ta, my_tf, my_rank, my_wlo, my_whi, my_counts};
                if (try32) {
                    // no address of this batch exceeds the extent so far plus the sizes of the batch
                    const uint64_t growth = wave_sum64((uint64_t)my_size);
                    if ((uint64_t)sh.extent_now + growth > 0xffffffffull) { outgrown = true; break; }
                }
                // The windows of the requests this wave settles (positions wave, wave + kWaves, ... of
                // the batch): the reads go out now and are looked at after the next step.  What the
                // batch itself adds to the table concerns them through `dep` instead.
                constexpr int kMine = kSpBatch / kWaves;
                uint32_t f_addr[kMine];
                uint2 f_fit[kMine];
#pragma unroll
                for (int j = 0; j < kMine; ++j) {
                    const uint32_t k = read_lane(my_wlo, wave + j * kWaves) + lane;     // < slots
                    const bool inside = k < read_lane(my_whi, wave + j * kWaves);       // (nothing is read past the window)
                    f_addr[j] = inside ? addr[k] : kSpUnplaced;
                    f_fit[j] = inside ? tb.fit_by_rank[k] : make_uint2(0u, 0u);
                }
                // which earlier requests of the batch each request has to wait for: wave w looks at
                // the requests 64 / kWaves * w .. of the batch, for all 64 lanes
                {
                    uint64_t part = 0;
                    for (int j = 0; j < kSpBatch / kWaves; ++j) {
                        const int e = wave * (kSpBatch / kWaves) + j;
                        const uint32_t e_ta = read_lane(my_ta, e), e_tf = read_lane(my_tf, e);
                        if (e < lane && e_ta < my_tf && my_ta < e_tf) part |= 1ull << e;
                    }
                    if (part) atomicOr((unsigned long long*)&sh.dep[lane], (unsigned long long)part);
                }
                // the placed short blocks of each window that conflict in lifetime, packed into the pool; this
                // wave settles these very requests, so it keeps their parts of the pool to itself (lane j:
                // request wave + j * kWaves)
                uint64_t rivals[kMine];
                uint32_t found[kMine], total = 0;
#pragma unroll
                for (int j = 0; j < kMine; ++j) {
                    const int q = wave + j * kWaves;
                    const uint32_t wlo = read_lane(my_wlo, q), whi = read_lane(my_whi, q);
                    // (a block of the window was allocated before the request is released: only its release counts)
                    const uint32_t q_ta = read_lane(my_ta, q);
                    const bool rival = whi - wlo <= (uint32_t)kWave && wlo + lane < whi && f_addr[j] != kSpUnplaced &&
                                       f_fit[j].y > q_ta;
                    rivals[j] = __builtin_amdgcn_ballot_w64(rival);
                    found[j] = (uint32_t)__builtin_popcountll(rivals[j]);
                    total += found[j];
                }
                // (room in the pool for all of them at once)
                uint32_t first = 0;
                if (total) {                                                   // (uniform)
                    if (lane == 0) first = atomicAdd(&sh.pool_used, total);
                    first = read_lane(first, 0);
                }
#pragma unroll
                for (int j = 0; j < kMine; ++j) {
                    const bool fits = first + found[j] <= (uint32_t)kSpPool;
                    if (((rivals[j] >> lane) & 1) && fits)
                        sh.pool[first + lanes_below(rivals[j])] = Span<uint32_t>{f_addr[j], f_addr[j] + f_fit[j].x};
                    if (lane == 0) {
                        sh.pool_first[wave + j * kWaves] = first;
                        sh.pool_count[wave + j * kWaves] = fits ? found[j] : kSpRefetch;
                    }
                    first += fits ? found[j] : 0u;
                }
                __syncthreads();
                const uint64_t dep = sh.dep[lane];
                const uint32_t part_first = sh.pool_first[lane], part_count = sh.pool_count[lane];
                const uint64_t all = nb == (uint32_t)kSpBatch ? ~0ull : (1ull << nb) - 1;
                uint64_t done = 0;
                const uint64_t wide = __builtin_amdgcn_ballot_w64(mine && my_whi - my_wlo > (uint32_t)kWave);
                // requests whose other conflicting blocks (their part of the pool, earlier requests of the batch) fit 16 lanes
                const uint64_t fits_row = __builtin_amdgcn_ballot_w64(part_count != kSpRefetch &&
                                                                      part_count + (uint32_t)__builtin_popcountll(dep) <= 16u);
                while (done != all) {
                    // settled: bit set in `done`; ready: everything it waits for is settled.  (What is ready
                    // together does not conflict with each other, so the order inside a round is free.)
                    const uint64_t ready = __builtin_amdgcn_ballot_w64(mine && !((done >> lane) & 1) && (dep & ~done) == 0);
                    // the ready requests with narrow windows go round the waves, a request each ...
                    const uint64_t narrow = ready & ~wide;
                    const bool take = ((narrow >> lane) & 1) && (lanes_below(narrow) + round) % kWaves == (uint32_t)wave;
                    ++round;
                    // (four at a time, a row of 16 lanes each, when what each has to keep clear of fits a row)
                    const uint64_t mine_now = __builtin_amdgcn_ballot_w64(take);
                    // (a lone request has the whole wave to itself: 64 list blocks a step instead of 16, and none
                    // of the gathering that gives each of four requests a row)
                    const uint64_t in_rows = (mine_now & (mine_now - 1)) ? mine_now & fits_row : 0ull;
                    for (uint64_t todo = mine_now & ~in_rows; todo; todo &= todo - 1) {
                        const int q = __builtin_ctzll(todo);
                        const uint32_t x = settle_request<false, kWaves>(list, count, b0, (uint32_t)q, readlane64(dep, q), bt,
                                                                         read_lane(part_first, q), read_lane(part_count, q), tb, pt,
                                                                         turn, sh);
                        if (lane == 0) {
                            sh.rq_addr[b0 + q] = x;
                            atomicMax(&sh.peak, x + read_lane(my_size, q));
                        }
                    }
                    for (uint64_t todo = in_rows; todo;) {
                        uint64_t rest = todo & (todo - 1);
                        rest &= rest - 1;
                        rest &= rest - 1;
                        rest &= rest - 1;                                         // (todo without its four lowest bits)
                        settle_rows(list, count, b0, todo & ~rest, dep, bt, part_first, part_count, sh);
                        todo = rest;
                    }
                    // ... and the workgroup as a whole takes the requests with wide windows one by one
                    for (uint64_t todo = ready & wide; todo; todo &= todo - 1) {
                        const int q = __builtin_ctzll(todo);
                        const uint32_t x = settle_wide<kWaves>(list, count, b0, (uint32_t)q, readlane64(dep, q), bt, tb, pt, turn, wide_turn, sh);
                        if (threadIdx.x == 0) {
                            sh.rq_addr[b0 + q] = x;
                            atomicMax(&sh.peak, x + read_lane(my_size, q));
                        }
                    }
                    __syncthreads();
                    done |= ready;
                }
                // the short blocks of the batch enter the table and its summaries
                if (wave == 1 % kWaves && mine && !(my_rank & kSpLongFlag)) {
                    const uint32_t x = sh.rq_addr[b0 + lane];
                    const uint32_t rank = my_rank & kSpRankMask;
                    addr[rank] = x;
                    if (my_rank & kSpLargeFlag) {
                        pt.large_addr[sh.rq_extra[b0 + lane]] = x;
                        atomicMin(&sh.large_min, x);
                        atomicMax(&sh.large_max, x + my_size);
                    } else {
                        atomicMin(&pt.group_span[rank / kWave].x, x);
                        atomicMax(&pt.group_span[rank / kWave].y, x + my_size);
                        atomicMin(&sh.region_min[rank >> tb.region_shift], x);
                        atomicMax(&sh.region_max[rank >> tb.region_shift], x + my_size);
                    }
                }
                // the long blocks of the batch, sorted by address, go into the list
                const uint64_t longs = __builtin_amdgcn_ballot_w64(mine && (my_rank & kSpLongFlag));
                uint32_t pending = (uint32_t)__builtin_popcountll(longs);
                if (count + pending > tb.list_cap) pending = 0;          // (an order that repeats requests; result unspecified)
                if (wave == 0) {
                    const uint32_t x = mine ? sh.rq_addr[b0 + lane] : 0u;
                    uint32_t place = 0;
                    for (uint64_t m = longs; m; m &= m - 1) {
                        const int e = __builtin_ctzll(m);
                        const uint32_t e_x = read_lane(x, e);
                        place += (e_x < x || (e_x == x && e < lane)) ? 1u : 0u;
                    }
                    if (pending && ((longs >> lane) & 1)) {
                        sh.pend_span[place] = Span<uint32_t>{x, x + my_size};
                        sh.pend_life[place] = kRanked ? make_uint2(sh.rq_extra[b0 + lane], 0u) : make_uint2(my_ta, my_tf);
                    }
                    if (lane == 0) { sh.extent_now = sh.peak; sh.pool_used = 0; }
                    if (lane < kSpBatch) sh.dep[lane] = 0;
                }
                __syncthreads();
                if (pending) {
                    // (short segments: the few long blocks of a batch mostly leave the lower part of the list as it is)
                    merge_pending<uint32_t, true, kThreads, 1>(list, spare, count, pending, sh);
                    count += pending;
                }
            }
            if (outgrown) break;
            // addresses of this refill -> offsets[p][request]
            __syncthreads();
            if (out && threadIdx.x < staged) out[sh.rq_id[threadIdx.x]] = (uint64_t)sh.rq_addr[threadIdx.x] << shift;
        }
        __syncthreads();
        if (outgrown) {
            if (threadIdx.x == 0) prm.wide_plans[p] = 1;
            continue;
        }
        if (threadIdx.x == 0) prm.peaks[p] = (uint64_t)sh.peak << shift;
    }
}

size_t split_workspace(uint32_t n, uint32_t t_end, const DeviceInfo& di, Carver& cv, SplitWorkspace* ws)
{
    const uint32_t n_pad = (n + kSortTile - 1) / kSortTile * kSortTile;
    const uint32_t slots = (n + kWave - 1) / kWave * kWave + kWave;
    const bool ranked = ranked_possible(n, t_end);
    uint32_t grid = (uint32_t)di.cus * (ranked ? 3 : 2);              // resident workgroups: tables for each
    ws->hist = cv.take<uint32_t>(kSpHistWords);
    ws->gate = cv.take<uint32_t>(1);
    ws->keys = cv.take<ulonglong2>(n_pad);
    ws->spare = cv.take<ulonglong2>(n_pad);
    ws->by_rank = cv.take<uint4>(slots);
    ws->size_by_rank = cv.take<uint32_t>(slots);
    ws->rank_of = cv.take<uint32_t>(n);
    ws->record = cv.take<uint4>(2 * (size_t)n);
    ws->fit_by_rank = cv.take<uint2>(slots);
    ws->addr = cv.take<uint32_t>((size_t)grid * slots);
    // at most an eighth of the short-lived requests count as large (sp_sigma)
    const uint32_t large_slots = (n / 8 + kWave - 1) / kWave * kWave + kWave;
    ws->group_span = cv.take<uint2>((size_t)grid * (slots / kWave));
    ws->is_large = cv.take<uint32_t>(slots);
    ws->large_before = cv.take<uint32_t>(slots);
    const size_t times = ranked ? (size_t)t_end + 2 : 0;
    ws->scan_chunks = cv.take<uint32_t>(((times > slots ? times : slots) + 1023) / 1024);
    // ranked list: marks at the long-lived requests' allocation and release times (one block: cleared together), their sums
    ws->allocated_at = cv.take<uint32_t>(2 * times + kSpSizeClasses);
    ws->released_at = ws->allocated_at + times;
    ws->class_size = ws->released_at + times;
    ws->allocated_before = cv.take<uint32_t>(times);
    ws->released_before = cv.take<uint32_t>(times);
    ws->times = (uint32_t)times;
    ws->scan_total = cv.take<uint32_t>(1);
    ws->large_fit = cv.take<uint2>(large_slots);
    ws->large_addr = cv.take<uint32_t>((size_t)grid * large_slots);
    ws->slots = slots;
    ws->large_slots = large_slots;
    ws->n_pad = n_pad;
    ws->grid = grid;
    return cv.used;
}

bool launch_plan_split(const PlanParams& prm, uint32_t t_end, const SplitWorkspace& ws, const DeviceInfo& di, hipStream_t stream)
{
    const uint32_t n = prm.n;
    const size_t lds = di.lds_per_block / 2;                          // two workgroups per CU
    const uint32_t list_cap = split_list_capacity(lds);
    const bool ranked = ws.times != 0;
    const uint32_t ranked_cap = ranked ? split_list_capacity(ranked_lds(di), RankedList::kEntryBytes) : 0u;
    uint32_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    uint64_t* acc = const_cast<uint64_t*>(prm.acc);

    hipLaunchKernelGGL(sp_clear_histogram, dim3(1), dim3(64), 0, stream, ws.hist, ws.gate);
    hipLaunchKernelGGL(sp_histogram, dim3(blocks > 256 ? 256 : blocks), dim3(256), 0, stream, prm.ta, prm.tf, n, ws.hist,
                       prm.status);
    hipLaunchKernelGGL(sp_decide, dim3(1), dim3(64), 0, stream, acc, ws.hist, n, t_end, list_cap > ranked_cap ? list_cap : ranked_cap,
                       prm, ws.gate, prm.status);
    hipLaunchKernelGGL(sp_size_histogram, dim3(blocks > 256 ? 256 : blocks), dim3(256), 0, stream, prm.size, prm.ta, prm.tf, n,
                       prm.acc, ws.hist, ws.gate);
    hipLaunchKernelGGL(sp_sigma, dim3(1), dim3(64), 0, stream, ws.hist, ws.gate);
    hipLaunchKernelGGL(sp_sort_tiles, dim3(ws.n_pad / kSortTile), dim3(kSortTile), 0, stream, prm.ta, n, ws.keys, ws.gate);
    const ulonglong2* sorted = launch_merge_tiles(ws.keys, ws.spare, ws.n_pad, 1, ws.gate, stream);
    hipLaunchKernelGGL(sp_tables, dim3(blocks), dim3(256), 0, stream, sorted, prm.size, prm.ta, prm.tf, n, ws.slots, prm.acc,
                       ws.by_rank, ws.size_by_rank, ws.fit_by_rank, ws.rank_of, ws.is_large, ws.hist, ws.gate);
    if (ranked) {
        hipLaunchKernelGGL(sp_clear_words, dim3(256), dim3(256), 0, stream, ws.allocated_at, 2 * (size_t)ws.times + kSpSizeClasses,
                           ws.gate);
        hipLaunchKernelGGL(sp_long_marks, dim3(blocks > 256 ? 256 : blocks), dim3(256), 0, stream, prm.size, prm.ta, prm.tf, n,
                           prm.acc, ws.allocated_at, ws.released_at, ws.class_size, ws.hist, ws.gate);
        launch_scan(ws.allocated_at, ws.times, ws.allocated_before, ws.scan_chunks, ws.scan_total, ws.gate, stream);
        launch_scan(ws.released_at, ws.times, ws.released_before, ws.scan_chunks, ws.scan_total, ws.gate, stream);
        hipLaunchKernelGGL(sp_ranked_decide, dim3(1), dim3(64), 0, stream, acc, ws.hist, list_cap, ranked_cap, ws.gate);
    }
    launch_scan(ws.is_large, ws.slots, ws.large_before, ws.scan_chunks, ws.scan_total, ws.gate, stream);
    hipLaunchKernelGGL(sp_windows, dim3(blocks), dim3(256), 0, stream, ws.by_rank, prm.ta, prm.tf, n, prm.acc, prm.size,
                       ws.rank_of, ws.large_before, ws.allocated_before, ws.released_before, ws.class_size, ws.record,
                       ws.large_fit, ws.hist, ws.gate);
    hipLaunchKernelGGL(sp_confirm, dim3(1), dim3(64), 0, stream, acc, ws.hist, n, ws.gate);

    SplitTables tb;
    tb.by_rank = ws.by_rank; tb.size_by_rank = ws.size_by_rank; tb.fit_by_rank = ws.fit_by_rank; tb.record = ws.record;
    tb.addr = ws.addr; tb.group_span = ws.group_span; tb.large_before = ws.large_before; tb.large_fit = ws.large_fit;
    tb.large_addr = ws.large_addr; tb.large_slots = ws.large_slots;
    tb.slots = ws.slots; tb.groups = ws.slots / kWave; tb.list_cap = list_cap;
    tb.next_plan = ws.hist + kSpHistNextPlan;
    tb.sigma = ws.hist + kSpHistSigma;
    tb.large_total = ws.scan_total;
    tb.region_shift = 6;
    while (((uint64_t)ws.slots + (1ull << tb.region_shift) - 1) >> tb.region_shift > (uint64_t)kWave) ++tb.region_shift;
    tb.class_size = ws.class_size;
    auto kernel = &plan_split_kernel<kSpThreads, false>;
    auto kernel_ranked = &plan_split_kernel<kSpThreads, true>;
    static std::atomic<bool> attr_set[64] = {};        // (set twice at worst when threads race)
    if (!attr_set[di.device]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)di.lds_per_block) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(kernel_ranked), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)di.lds_per_block) != hipSuccess)
            return false;
        attr_set[di.device] = true;
    }
    // exactly one of the two does the work (acc[kAccSplit] bit 1)
    uint32_t grid = (uint32_t)di.cus * 2;
    if (grid > prm.P) grid = prm.P;
    const size_t lds_bytes = sizeof(SplitLds) + (size_t)list_cap * SpList::kEntryBytes;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kSpThreads), lds_bytes, stream, prm, tb);
    if (ranked) {
        grid = ws.grid;                                               // three per CU
        if (grid > prm.P) grid = prm.P;
        tb.list_cap = ranked_cap;
        hipLaunchKernelGGL(kernel_ranked, dim3(grid), dim3(kSpThreads), sizeof(SplitLds) + (size_t)ranked_cap * RankedList::kEntryBytes,
                           stream, prm, tb);
    }
    return true;
}

}  // namespace stalloc
