// stalloc_reusable_space: the dynamic reusable space of a plan (Sec. 5.2).
//
// For a time window T the occupied addresses A_o are the union of the address ranges R_s(d) of
// the decisions d whose lifespan R_t(d) meets T; the pool A runs from the lowest start address to
// the highest end address of the whole plan; the reusable space is A_i = A \ A_o.  It is returned
// as its maximal intervals in ascending address order.  Windows are half-open like lifespans.
//
//   sort     The decisions are sorted by (start address, request number) once per call: tiles of
//            256 keys are sorted in LDS (bitonic network) and merged in log2(n / 256) passes,
//            an element's place being its place in its own run plus the number of elements
//            of the partner run that sort before it (binary search); nothing depends on how
//            the addresses are distributed.
//   gather   (start, end, lifespan) of the decisions in that order; the unit of the pool's
//            addresses (largest power of two dividing every start and end relative to the
//            pool's start): when 32-bit counts of it cover the pool, the sweep below runs on
//            such counts.
//   sweep    One workgroup per window over the address-sorted decisions, each wave a contiguous
//            part, 64 decisions a step.  A decision counts if its lifespan meets the window; a
//            wave64 running maximum (DPP) of the ends of those before it is "covered so far", and a
//            counting decision that starts above it closes an idle interval [covered, start).  Three
//            walks, a barrier between them: (1) the maximum end per wave, which gives every wave the
//            "covered" it starts from; (2) the number of intervals per wave, which gives every wave
//            its place in the output; (3) the intervals themselves.  What lies between the last
//            covered address and the end of the pool is the final interval.
//            With thousands of windows the roles are exchanged: a wave takes 64 windows, one
//            per lane, and a contiguous part of the sorted decisions, which
//            are taken one at a time as wave-uniform values -- two compares per decision tell
//            for all 64 windows whether it counts (most decisions count for none and are done
//            with), and "covered so far" is a per-lane maximum without any cross-lane step.  The
//            same three walks (one launch each, a wave per group of windows and part of the
//            plan), at a fraction of the instructions per decision and window.
#include "host_util.h"
#include "sort_keys.h"
#include "wave.h"

namespace stalloc {

constexpr int kRsTile = kSortTile;
constexpr int kRsThreads = 256;
constexpr int kRsWaves = kRsThreads / kWave;

// A = [lo, hi).  Every start and end address, taken relative to lo, is a multiple of 2^shift
// (the largest such power); `narrow` says that the pool counted in those units fits 32 bits.
struct RsPool { uint64_t lo, hi, bits; uint32_t shift, narrow; };

__global__ void rs_init(RsPool* pool)
{
    if (threadIdx.x == 0) { pool->lo = ~0ull; pool->hi = 0; pool->bits = 0; pool->shift = 0; pool->narrow = 0; }
}

// One tile of 256 decisions per workgroup, sorted in LDS; slot e past the end holds a key behind
// every real one, (~0, ~0 << 32 | e).  Also the pool's bounds.
__global__ void __launch_bounds__(kRsTile)
rs_sort_tiles(const uint64_t* __restrict__ size, const uint64_t* __restrict__ offsets, uint32_t n, ulonglong2* keys,
              RsPool* pool, const uint32_t* status)
{
    __shared__ ulonglong2 k[kRsTile];
    if (*status != STALLOC_OK) return;
    const uint32_t t = threadIdx.x, i = blockIdx.x * kRsTile + t;
    const bool ok = i < n;
    const uint64_t a = ok ? offsets[i] : ~0ull;
    k[t] = ok ? make_ulonglong2(a, i) : filler_key(i);          // keys (address, request number)
    {
        const uint64_t lo = wave_min64(a);                                       // (slots past n hold ~0)
        const uint64_t hi = wave_max64(ok ? a + size[i] : 0ull);
        if (lane_id() == 0) {
            atomicMin((unsigned long long*)&pool->lo, (unsigned long long)lo);
            atomicMax((unsigned long long*)&pool->hi, (unsigned long long)hi);
        }
    }
    sort_tile(k);
    keys[blockIdx.x * kRsTile + t] = k[t];
}

// (start, end, lifespan) of the decisions in address order; the bits set in any start or end
// address relative to the pool's start.
__global__ void __launch_bounds__(256)
rs_gather(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf,
          const uint64_t* __restrict__ offsets, const ulonglong2* __restrict__ sorted, uint32_t n,
          uint64_t* s_lo, uint64_t* s_hi, uint2* s_life, RsPool* pool, const uint32_t* status)
{
    __shared__ uint64_t part[4];
    if (*status != STALLOC_OK) return;
    const uint64_t pool_lo = pool->lo;
    uint64_t bits = 0;
    for (uint32_t r = blockIdx.x * blockDim.x + threadIdx.x; r < n; r += gridDim.x * blockDim.x) {
        uint32_t i = (uint32_t)sorted[r].y;
        if (i >= n) i = 0;                                   // (cannot happen: the first n sorted keys are the real ones)
        const uint64_t lo = offsets[i], hi = lo + size[i];
        s_lo[r] = lo;
        s_hi[r] = hi;
        s_life[r] = make_uint2(ta[i], tf[i]);
        bits |= (lo - pool_lo) | (hi - pool_lo);
    }
    bits = wave_or64(bits);
    if (lane_id() == 0) part[wave_id()] = bits;
    __syncthreads();
    if (threadIdx.x == 0) {
        bits = part[0] | part[1] | part[2] | part[3];
        if (bits) atomicOr((unsigned long long*)&pool->bits, (unsigned long long)bits);
    }
}

// The unit of the pool's addresses and whether 32-bit counts of it cover the pool.
__global__ void rs_units(RsPool* pool, const uint32_t* status)
{
    if (*status != STALLOC_OK || threadIdx.x != 0) return;
    const uint64_t span = pool->hi - pool->lo;                  // > 0: sizes are
    const uint32_t shift = (uint32_t)__builtin_ctzll(pool->bits | span);
    pool->shift = shift;
    pool->narrow = (span >> shift) <= 0xffffffffull ? 1u : 0u;
}

// Start and end of every sorted decision in units of the pool, relative to its start.
__global__ void __launch_bounds__(256)
rs_compress(const uint64_t* __restrict__ s_lo, const uint64_t* __restrict__ s_hi, uint32_t n, const RsPool* pool,
            uint32_t* c_lo, uint32_t* c_hi, const uint32_t* status)
{
    if (*status != STALLOC_OK || !pool->narrow) return;
    const uint64_t pool_lo = pool->lo;
    const uint32_t shift = pool->shift;
    for (uint32_t r = blockIdx.x * blockDim.x + threadIdx.x; r < n; r += gridDim.x * blockDim.x) {
        c_lo[r] = (uint32_t)((s_lo[r] - pool_lo) >> shift);
        c_hi[r] = (uint32_t)((s_hi[r] - pool_lo) >> shift);
    }
}

struct RsArgs {
    const uint32_t* c_lo;        // sorted decisions in 32-bit units of the pool (valid when the pool is narrow)
    const uint32_t* c_hi;
    const uint64_t* s_lo;
    const uint64_t* s_hi;
    const uint2* s_life;
    const RsPool* pool;
    const uint32_t* windows;     // [k][2]
    uint64_t* ranges;            // [k][max_ranges][2] or nullptr
    uint32_t* counts;            // [k]
    uint64_t* idle_bytes;        // [k] or nullptr
    uint32_t* status;
    uint32_t n, k, max_ranges;
};

__global__ void __launch_bounds__(kRsThreads) rs_sweep(RsArgs g)
{
    __shared__ uint64_t wave_reach[kRsWaves];
    __shared__ uint32_t wave_found[kRsWaves];
    __shared__ uint64_t wave_idle[kRsWaves];
    if (*g.status != STALLOC_OK) return;
    const int lane = lane_id(), wave = wave_id();
    const uint64_t pool_lo = g.pool->lo, pool_hi = g.pool->hi;
    const uint32_t steps = (g.n + kRsThreads - 1) / kRsThreads;           // 64-decision steps per wave
    const uint32_t first = (uint32_t)wave * steps * kWave;

    for (uint32_t w = blockIdx.x; w < g.k; w += gridDim.x) {
        const uint32_t w_lo = g.windows[2 * w], w_hi = g.windows[2 * w + 1];
        if (w_lo >= w_hi) {                                               // (uniform) not a window
            if (threadIdx.x == 0) atomicMax(g.status, (uint32_t)STALLOC_ERR_BAD_WINDOW);
            continue;
        }
        // per step: `ends` = end address where the decision counts, else 0
        auto ends_of = [&](uint32_t s, uint64_t& lo) -> uint64_t {
            const uint32_t at = first + s * kWave + lane;
            lo = 0;
            if (at >= g.n) return 0;
            const uint2 life = g.s_life[at];
            if (!(life.x < w_hi && w_lo < life.y)) return 0;
            lo = g.s_lo[at];
            return g.s_hi[at];
        };

        // walk 1: how far the decisions of each wave reach
        uint64_t reach = 0, lo;
        for (uint32_t s = 0; s < steps; ++s) reach = umax64(reach, ends_of(s, lo));
        reach = wave_max64(reach);
        __syncthreads();                                                  // (previous window's reads done)
        if (lane == 0) wave_reach[wave] = reach;
        __syncthreads();
        uint64_t covered0 = pool_lo, covered_all = pool_lo;               // covered before this wave's part / at the end
        for (int v = 0; v < kRsWaves; ++v) {
            if (v < wave) covered0 = umax64(covered0, wave_reach[v]);
            covered_all = umax64(covered_all, wave_reach[v]);
        }

        // walk 2: idle intervals closed inside each wave's part
        uint32_t found = 0;
        uint64_t run = covered0;
        for (uint32_t s = 0; s < steps; ++s) {
            const uint64_t end = ends_of(s, lo);
            const uint64_t incl = wave_scan_max64(end);
            const uint64_t covered = umax64(run, wave_shift_up64(incl, 0));
            found += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(end != 0 && lo > covered));
            run = umax64(run, readlane64(incl, kWave - 1));
        }
        if (lane == 0) wave_found[wave] = found;
        __syncthreads();
        uint32_t place = 0, total = 0;
        for (int v = 0; v < kRsWaves; ++v) {
            if (v < wave) place += wave_found[v];
            total += wave_found[v];
        }

        // walk 3: write them
        uint64_t* out = g.ranges ? g.ranges + (size_t)w * g.max_ranges * 2 : nullptr;
        uint64_t idle = 0;
        run = covered0;
        for (uint32_t s = 0; s < steps; ++s) {
            const uint64_t end = ends_of(s, lo);
            const uint64_t incl = wave_scan_max64(end);
            const uint64_t covered = umax64(run, wave_shift_up64(incl, 0));
            const bool closes = end != 0 && lo > covered;
            const uint64_t closers = __builtin_amdgcn_ballot_w64(closes);
            if (closes) {
                const uint32_t at = place + lanes_below(closers);
                if (out && at < g.max_ranges) { out[2 * at] = covered; out[2 * at + 1] = lo; }
                idle += lo - covered;
            }
            place += (uint32_t)__builtin_popcountll(closers);
            run = umax64(run, readlane64(incl, kWave - 1));
        }
        idle = wave_sum64(idle);
        if (lane == 0) wave_idle[wave] = idle;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint64_t sum = 0;
            for (int v = 0; v < kRsWaves; ++v) sum += wave_idle[v];
            if (covered_all < pool_hi) {                                  // from the last covered address to the end of the pool
                if (out && total < g.max_ranges) { out[2 * total] = covered_all; out[2 * total + 1] = pool_hi; }
                sum += pool_hi - covered_all;
                ++total;
            }
            g.counts[w] = total;
            if (g.idle_bytes) g.idle_bytes[w] = sum;
        }
    }
}

#ifndef STALLOC_RS_WIDE_FROM
#define STALLOC_RS_WIDE_FROM (1ull << 23)
#endif
// A lane takes a window from this many decisions x windows on (three launches and per-part
// prefixes cost more than they save below it), given at least half a wave of windows.
constexpr uint64_t kRsWideFrom = STALLOC_RS_WIDE_FROM;
__host__ inline bool rs_window_per_lane(uint32_t n, uint32_t k) { return k >= 32 && (uint64_t)n * k >= kRsWideFrom; }
constexpr uint32_t kRsMaxParts = 256;                    // parts the sorted plan is cut into, at most

// Scratch of the window-per-lane sweep, [group of 64 windows][part][lane].
struct RsParts {
    uint64_t* reach;        // walk 1: maximum end of the counting decisions of the part
    uint64_t* idle;         // walk 2: bytes of the idle intervals closed inside the part
    uint32_t* found;        //         and their number
    uint32_t parts;         // parts per group; one wave each
    uint32_t steps;         // 64-decision steps per part
};

// One wave = 64 windows (one per lane) x one part of the sorted plan.  kWalk = 1, 2, 3: the
// three walks, one launch each (a part needs the results of all lower parts of the walk before).
__device__ __forceinline__ uint32_t read_lane_addr(uint32_t v, int q) { return __builtin_amdgcn_readlane(v, q); }
__device__ __forceinline__ uint64_t read_lane_addr(uint64_t v, int q) { return readlane64(v, q); }

// Addr = uint32_t: addresses in units of the pool relative to its start (a narrow pool: half the
// registers, single-instruction compares and maxima); Addr = uint64_t: byte addresses.
template <int kWalk, typename Addr>
__device__ __forceinline__ void sweep_by_window(const RsArgs& g, const RsParts& sc)
{
    constexpr bool kNarrow = sizeof(Addr) == 4;
    const int lane = lane_id();
    const uint64_t pool_lo = g.pool->lo;
    const uint32_t shift = kNarrow ? g.pool->shift : 0u;
    auto bytes = [&](Addr v) -> uint64_t { return kNarrow ? pool_lo + ((uint64_t)v << shift) : (uint64_t)v; };
    const uint32_t groups = (g.k + kWave - 1) / kWave;
    const uint32_t waves = groups * sc.parts;
    for (uint32_t unit = blockIdx.x * kRsWaves + (uint32_t)wave_id(); unit < waves; unit += gridDim.x * kRsWaves) {
        const uint32_t grp = unit / sc.parts, part = unit % sc.parts;
        const uint32_t w = grp * kWave + lane;
        // lanes without a window, and malformed windows, get bounds that no lifespan meets
        uint32_t w_lo = 1, w_hi = 0;
        bool live = false;
        if (w < g.k) {
            const uint32_t lo = g.windows[2 * w], hi = g.windows[2 * w + 1];
            if (lo < hi) { w_lo = lo; w_hi = hi; live = true; }
            else if (kWalk == 1 && part == 0) atomicMax(g.status, (uint32_t)STALLOC_ERR_BAD_WINDOW);
        }
        const size_t row = ((size_t)grp * sc.parts) * kWave + lane;        // [grp][0][lane]; next part: + kWave
        const uint32_t first = part * sc.steps * kWave;
        // body(start, end, counts): called for every decision of this part that counts for at
        // least one window, in address order, with wave-uniform start and end
        auto walk = [&](auto&& body) {
            for (uint32_t s = 0; s < sc.steps; ++s) {
                const uint32_t k0 = first + s * kWave;
                if (k0 >= g.n) break;                                     // (uniform)
                const uint32_t at = k0 + lane;
                const bool valid = at < g.n;
                const uint2 life = valid ? g.s_life[at] : make_uint2(0xffffffffu, 0u);   // past the end: meets no window
                Addr lo = 0, hi = 0;
                if (valid) {
                    if constexpr (kNarrow) { lo = g.c_lo[at]; hi = g.c_hi[at]; }
                    else { lo = g.s_lo[at]; hi = g.s_hi[at]; }
                }
#pragma unroll 8
                for (int q = 0; q < kWave; ++q) {
                    const uint32_t ts_q = __builtin_amdgcn_readlane(life.x, q), te_q = __builtin_amdgcn_readlane(life.y, q);
                    const bool counts = ts_q < w_hi && w_lo < te_q;
                    if (__builtin_amdgcn_ballot_w64(counts) == 0) continue;           // (uniform)
                    body(read_lane_addr(lo, q), read_lane_addr(hi, q), counts);
                }
            }
        };

        if constexpr (kWalk == 1) {          // how far the decisions of each part reach
            Addr covered = 0;
            walk([&](Addr, Addr end, bool counts) { covered = counts ? umax(covered, end) : covered; });
            sc.reach[row + (size_t)part * kWave] = covered;
        } else {
            Addr covered = kNarrow ? (Addr)0 : (Addr)pool_lo;       // covered before this part
            for (uint32_t v = 0; v < part; ++v) covered = umax(covered, (Addr)sc.reach[row + (size_t)v * kWave]);
            if constexpr (kWalk == 2) {      // idle intervals closed inside each part
                uint32_t count = 0;
                Addr idle = 0;               // (disjoint intervals of the pool: fits the address type)
                walk([&](Addr start, Addr end, bool counts) {
                    if (counts && start > covered) { ++count; idle += start - covered; }
                    covered = counts ? umax(covered, end) : covered;
                });
                sc.found[row + (size_t)part * kWave] = count;
                sc.idle[row + (size_t)part * kWave] = idle;
            } else {                         // write them; the last part adds the tail of the pool and the totals
                uint32_t place = 0;
                for (uint32_t v = 0; v < part; ++v) place += sc.found[row + (size_t)v * kWave];
                uint64_t* out = (g.ranges && live) ? g.ranges + (size_t)w * g.max_ranges * 2 : nullptr;
                const Addr covered0 = covered;
                if (g.ranges) {                                           // (uniform; lanes without a window count nothing)
                    walk([&](Addr start, Addr end, bool counts) {
                        if (counts && start > covered) {
                            if (place < g.max_ranges) { out[2 * place] = bytes(covered); out[2 * place + 1] = bytes(start); }
                            ++place;
                        }
                        covered = counts ? umax(covered, end) : covered;
                    });
                }
                if (part + 1 == sc.parts && live) {
                    const size_t mine = row + (size_t)part * kWave;
                    const uint64_t covered_all = bytes(umax(covered0, (Addr)sc.reach[mine]));
                    uint32_t total = sc.found[mine];
                    uint64_t idle_total = sc.idle[mine];
                    for (uint32_t v = 0; v < part; ++v) { total += sc.found[row + (size_t)v * kWave]; idle_total += sc.idle[row + (size_t)v * kWave]; }
                    idle_total <<= shift;                                 // units of the pool -> bytes
                    const uint64_t pool_hi = g.pool->hi;
                    if (covered_all < pool_hi) {                          // from the last covered address to the end of the pool
                        if (out && total < g.max_ranges) { out[2 * total] = covered_all; out[2 * total + 1] = pool_hi; }
                        idle_total += pool_hi - covered_all;
                        ++total;
                    }
                    g.counts[w] = total;
                    if (g.idle_bytes) g.idle_bytes[w] = idle_total;
                }
            }
        }
    }
}

template <int kWalk>
__global__ void __launch_bounds__(kRsThreads) rs_sweep_by_window(RsArgs g, RsParts sc)
{
    if (*g.status != STALLOC_OK) return;
    if (g.pool->narrow) sweep_by_window<kWalk, uint32_t>(g, sc);       // (uniform)
    else sweep_by_window<kWalk, uint64_t>(g, sc);
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_reusable_space(const stalloc_trace* tr, const uint64_t* offsets, const uint32_t* windows,
                                      uint32_t k, uint32_t max_ranges, uint64_t* ranges, uint32_t* counts,
                                      uint64_t* idle_bytes, uint32_t* device_status, void* workspace,
                                      size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || k == 0 || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    DeviceInfo di;
    if (!device_info(&di)) return STALLOC_ERR_DEVICE;
    const uint32_t n = tr->n;

    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    RsPool* pool = cv.take<RsPool>(1);
    const uint32_t tiles = (n + kRsTile - 1) / kRsTile;
    ulonglong2* keys = cv.take<ulonglong2>((size_t)tiles * kRsTile);
    ulonglong2* spare = cv.take<ulonglong2>((size_t)tiles * kRsTile);
    uint64_t* s_lo = cv.take<uint64_t>(n);
    uint64_t* s_hi = cv.take<uint64_t>(n);
    uint2* s_life = cv.take<uint2>(n);
    uint32_t* c_lo = cv.take<uint32_t>(n);
    uint32_t* c_hi = cv.take<uint32_t>(n);
    // window-per-lane sweep: enough (group of 64 windows) x (part of the plan) waves to fill the chip
    RsParts sc = {nullptr, nullptr, nullptr, 0, 0};
    const uint32_t groups = (k + kWave - 1) / kWave;
    if (rs_window_per_lane(n, k)) {
        const uint32_t all_steps = (n + kWave - 1) / kWave;
        uint32_t parts = ((uint32_t)di.cus * 16 + groups - 1) / groups;
        if (parts > kRsMaxParts) parts = kRsMaxParts;
        if (parts > (all_steps + 1) / 2) parts = (all_steps + 1) / 2;     // at least two steps to a part
        sc.steps = (all_steps + parts - 1) / parts;
        sc.parts = (all_steps + sc.steps - 1) / sc.steps;
        const size_t cells = (size_t)groups * sc.parts * kWave;
        sc.reach = cv.take<uint64_t>(cells);
        sc.idle = cv.take<uint64_t>(cells);
        sc.found = cv.take<uint32_t>(cells);
    }
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!offsets || !windows || !counts || !device_status || (max_ranges != 0 && !ranges) ||
        *workspace_bytes < cv.used || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);

    uint32_t blocks = (n + 255) / 256;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(rs_init, dim3(1), dim3(64), 0, stream, pool);
    hipLaunchKernelGGL(rs_sort_tiles, dim3(tiles), dim3(kRsTile), 0, stream, tr->size, offsets, n, keys, pool, device_status);
    const ulonglong2* sorted = launch_merge_tiles(keys, spare, tiles * kRsTile, 1, device_status, stream);
    hipLaunchKernelGGL(rs_gather, dim3(blocks), dim3(256), 0, stream, tr->size, tr->t_alloc, tr->t_free, offsets, sorted, n,
                       s_lo, s_hi, s_life, pool, device_status);
    RsArgs g;
    g.c_lo = c_lo; g.c_hi = c_hi;
    g.s_lo = s_lo; g.s_hi = s_hi; g.s_life = s_life; g.pool = pool; g.windows = windows;
    g.ranges = max_ranges ? ranges : nullptr; g.counts = counts; g.idle_bytes = idle_bytes; g.status = device_status;
    g.n = n; g.k = k; g.max_ranges = max_ranges;
    if (rs_window_per_lane(n, k)) {
        hipLaunchKernelGGL(rs_units, dim3(1), dim3(64), 0, stream, pool, device_status);
        hipLaunchKernelGGL(rs_compress, dim3(blocks), dim3(256), 0, stream, s_lo, s_hi, n, pool, c_lo,
                           c_hi, device_status);
        const uint64_t waves = (uint64_t)groups * sc.parts;
        uint32_t grid = (uint32_t)di.cus * 8;
        if (grid > (waves + kRsWaves - 1) / kRsWaves) grid = (uint32_t)((waves + kRsWaves - 1) / kRsWaves);
        hipLaunchKernelGGL(rs_sweep_by_window<1>, dim3(grid), dim3(kRsThreads), 0, stream, g, sc);
        hipLaunchKernelGGL(rs_sweep_by_window<2>, dim3(grid), dim3(kRsThreads), 0, stream, g, sc);
        hipLaunchKernelGGL(rs_sweep_by_window<3>, dim3(grid), dim3(kRsThreads), 0, stream, g, sc);
    } else {
        uint32_t grid = (uint32_t)di.cus * 8;
        if (grid > k) grid = k;
        hipLaunchKernelGGL(rs_sweep, dim3(grid), dim3(kRsThreads), 0, stream, g);
    }
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
