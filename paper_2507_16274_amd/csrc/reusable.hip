// stalloc_reusable_space: the dynamic reusable space of a plan (Sec. 5.2).
//
// For a time window T the occupied addresses A_o are the union of the address ranges R_s(d) of
// the decisions d whose lifespan R_t(d) meets T; the pool A runs from the lowest start address to
// the highest end address of the whole plan; the reusable space is A_i = A \ A_o.  It is returned
// as its maximal intervals in ascending address order.  Windows are half-open like lifespans.
//
//   rank     The decisions are sorted by (start address, request number) once per call: tiles of
//            256 are sorted in LDS (bitonic network); the rank of a decision is then its position
//            in its own tile plus, for every other tile, the number of that tile's decisions
//            that sort before it -- a binary search in the tile, staged in LDS.  n^2 / 32 steps
//            in all, no scratch passes, nothing to tune, no dependence on how the addresses are
//            distributed.
//   scatter  (start, end, lifespan) of every decision go to their rank.
//   sweep    One workgroup per window over the address-sorted decisions, each wave a contiguous
//            part, 64 decisions a step.  A decision counts if its lifespan meets the window; a
//            wave64 running maximum (DPP) of the ends of those before it is "covered so far", and a
//            counting decision that starts above it closes an idle interval [covered, start).  Three
//            walks, a barrier between them: (1) the maximum end per wave, which gives every wave the
//            "covered" it starts from; (2) the number of intervals per wave, which gives every wave
//            its place in the output; (3) the intervals themselves.  What lies between the last
//            covered address and the end of the pool is the final interval.
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kRsTile = 256;
constexpr int kRsThreads = 256;
constexpr int kRsWaves = kRsThreads / kWave;

struct RsPool { uint64_t lo, hi; };      // A = [lo, hi)

__global__ void rs_init(uint32_t* rank, uint32_t n, RsPool* pool)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) rank[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) { pool->lo = ~0ull; pool->hi = 0; }
}

// (address, request number), ordered lexicographically
struct RsKey { uint64_t a; uint32_t id; };
__device__ __forceinline__ bool before(const RsKey& x, const RsKey& y) { return x.a < y.a || (x.a == y.a && x.id < y.id); }

// One tile of 256 decisions per workgroup: sorted in LDS, written to t_a / t_id; past-the-end
// slots hold (~0, ~0) and sort last.  Also the pool's bounds.
__global__ void __launch_bounds__(kRsTile)
rs_sort_tiles(const uint64_t* __restrict__ size, const uint64_t* __restrict__ offsets, uint32_t n, uint64_t* t_a,
              uint32_t* t_id, RsPool* pool, const uint32_t* status)
{
    __shared__ uint64_t k_a[kRsTile];
    __shared__ uint32_t k_id[kRsTile];
    if (*status != STALLOC_OK) return;
    const uint32_t t = threadIdx.x, i = blockIdx.x * kRsTile + t;
    const bool ok = i < n;
    const uint64_t a = ok ? offsets[i] : ~0ull;
    k_a[t] = a;
    k_id[t] = ok ? i : ~0u;
    {
        const uint64_t lo = wave_min64(a);                                       // (slots past n hold ~0)
        const uint64_t hi = wave_max64(ok ? a + size[i] : 0ull);
        if (lane_id() == 0) {
            atomicMin((unsigned long long*)&pool->lo, (unsigned long long)lo);
            atomicMax((unsigned long long*)&pool->hi, (unsigned long long)hi);
        }
    }
    for (uint32_t span = 2; span <= (uint32_t)kRsTile; span <<= 1) {
        for (uint32_t gap = span >> 1; gap > 0; gap >>= 1) {
            __syncthreads();
            const uint32_t other = t ^ gap;
            if (other > t) {
                const RsKey x = {k_a[t], k_id[t]}, y = {k_a[other], k_id[other]};
                const bool ascending = (t & span) == 0;
                if (before(y, x) == ascending) {
                    k_a[t] = y.a; k_id[t] = y.id;
                    k_a[other] = x.a; k_id[other] = x.id;
                }
            }
        }
    }
    __syncthreads();
    t_a[blockIdx.x * kRsTile + t] = k_a[t];
    t_id[blockIdx.x * kRsTile + t] = k_id[t];
}

// grid (tiles, slices of the tile range): thread p of workgroup b holds the decision at position p
// of sorted tile b and adds, to its rank, how many decisions of the slice's tiles sort before it.
__global__ void __launch_bounds__(kRsTile)
rs_rank(const uint64_t* __restrict__ t_a, const uint32_t* __restrict__ t_id, uint32_t n, uint32_t tiles,
        uint32_t tiles_per_slice, uint32_t* rank, const uint32_t* status)
{
    __shared__ uint64_t k_a[kRsTile];
    __shared__ uint32_t k_id[kRsTile];
    if (*status != STALLOC_OK) return;
    const uint32_t p = threadIdx.x, own = blockIdx.x;
    const RsKey me = {t_a[own * kRsTile + p], t_id[own * kRsTile + p]};
    uint32_t count = 0;
    const uint32_t tile0 = blockIdx.y * tiles_per_slice;
    for (uint32_t t = tile0; t < tile0 + tiles_per_slice && t < tiles; ++t) {
        if (t == own) { count += p; continue; }                                  // (uniform)
        __syncthreads();
        k_a[p] = t_a[t * kRsTile + p];
        k_id[p] = t_id[t * kRsTile + p];
        __syncthreads();
        uint32_t lo = 0;                                                          // first position not before `me`
        for (uint32_t half = kRsTile / 2; half > 0; half >>= 1) {
            const RsKey probe = {k_a[lo + half - 1], k_id[lo + half - 1]};
            if (before(probe, me)) lo += half;
        }
        const RsKey last = {k_a[lo], k_id[lo]};                                   // lo <= 255 here
        count += lo + (before(last, me) ? 1u : 0u);
    }
    if (me.id < n && count) atomicAdd(&rank[me.id], count);
}

__global__ void __launch_bounds__(256)
rs_scatter(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf,
           const uint64_t* __restrict__ offsets, const uint32_t* __restrict__ rank, uint32_t n,
           uint64_t* s_lo, uint64_t* s_hi, uint2* s_life, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint32_t r = rank[i];
        s_lo[r] = offsets[i];
        s_hi[r] = offsets[i] + size[i];
        s_life[r] = make_uint2(ta[i], tf[i]);
    }
}

struct RsArgs {
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
    uint32_t* rank = cv.take<uint32_t>(n);
    const uint32_t tiles = (n + kRsTile - 1) / kRsTile;
    uint64_t* t_a = cv.take<uint64_t>((size_t)tiles * kRsTile);
    uint32_t* t_id = cv.take<uint32_t>((size_t)tiles * kRsTile);
    uint64_t* s_lo = cv.take<uint64_t>(n);
    uint64_t* s_hi = cv.take<uint64_t>(n);
    uint2* s_life = cv.take<uint2>(n);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!offsets || !windows || !counts || !device_status || (max_ranges != 0 && !ranges) ||
        *workspace_bytes < cv.used || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);

    uint32_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(rs_init, dim3(blocks > 1024 ? 1024 : blocks), dim3(256), 0, stream, rank, n, pool);
    hipLaunchKernelGGL(rs_sort_tiles, dim3(tiles), dim3(kRsTile), 0, stream, tr->size, offsets, n, t_a, t_id, pool,
                       device_status);
    // enough slices of the tile range to fill the chip, at least 8 tiles each
    uint32_t slices = (uint32_t)di.cus * 8 / tiles;
    if (slices < 1) slices = 1;
    if (slices > (tiles + 7) / 8) slices = (tiles + 7) / 8;
    const uint32_t tiles_per_slice = (tiles + slices - 1) / slices;
    slices = (tiles + tiles_per_slice - 1) / tiles_per_slice;
    hipLaunchKernelGGL(rs_rank, dim3(tiles, slices), dim3(kRsTile), 0, stream, t_a, t_id, n, tiles, tiles_per_slice, rank,
                       device_status);
    hipLaunchKernelGGL(rs_scatter, dim3(blocks > 1024 ? 1024 : blocks), dim3(256), 0, stream, tr->size, tr->t_alloc,
                       tr->t_free, offsets, rank, n, s_lo, s_hi, s_life, device_status);
    RsArgs g;
    g.s_lo = s_lo; g.s_hi = s_hi; g.s_life = s_life; g.pool = pool; g.windows = windows;
    g.ranges = max_ranges ? ranges : nullptr; g.counts = counts; g.idle_bytes = idle_bytes; g.status = device_status;
    g.n = n; g.k = k; g.max_ranges = max_ranges;
    uint32_t grid = (uint32_t)di.cus * 8;
    if (grid > k) grid = k;
    hipLaunchKernelGGL(rs_sweep, dim3(grid), dim3(kRsThreads), 0, stream, g);
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
