// stalloc_plan: batched greedy placement, one workgroup per candidate placement order.
//
// Rule (Sec. 5.1): requests are taken in the given order; each gets the lowest address at
// which it conflicts with no earlier request of the same plan in lifespan and address
// range at once.  Extent of a plan = max(a + s) (Eq. 2).
//
// Per plan the workgroup keeps the list of placed blocks SORTED BY ADDRESS, so that no
// sorting is needed when a request is placed:
//   scan    the sorted list is walked in address order, 64 blocks per wave; a ballot-free
//           compare keeps the blocks whose lifetime conflicts with the request, a wave64
//           running maximum of their end addresses gives "first address not covered so
//           far", and the walk stops at the first block that starts at least `size` bytes
//           above it (lowest fitting hole) or at the end of the list;
//   pending freshly placed blocks go to a small side buffer, sorted by address and held in
//           registers by every wave (one block per lane), instead of being inserted at once.
//           Let f(c) be the lowest address >= c at which the request clears the pending
//           blocks that conflict with its lifetime (a short walk over those blocks).  f is
//           monotone and idempotent, so f(max(a, b)) = max(f(a), f(b)): replacing every
//           listed block's end address e by f(e) before the running maximum, and starting
//           from f(0), makes the scan honour the side buffer without a second pass.  When
//           the side buffer is full it is merged into the sorted list in one pass (each
//           listed block moves up by the number of pending blocks at or below it).
// The sorted list lives in LDS when it fits (small traces) and in the workspace otherwise.
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kBatch = 256;          // requests fetched per refill
constexpr int kPending = 16;         // side-buffer entries (at most one wave)
constexpr int kEntryBytes = 24;      // start address, end address, (t_alloc, t_free)
constexpr uint64_t kNoHit = ~0ull;

// LDS that does not depend on the list capacity
struct PlanFixedLds {
    uint64_t rq_size[kBatch];
    uint64_t rq_addr[kBatch];
    uint32_t rq_ta[kBatch];
    uint32_t rq_tf[kBatch];
    uint32_t rq_id[kBatch];
    uint64_t wave_top[kPlanWaves];
    uint64_t wave_hit[kPlanWaves];
    uint64_t sorted_lo[kPending];
    uint64_t sorted_hi[kPending];
    uint2 sorted_tt[kPending];
};

struct PlanParams {
    const uint64_t* size;
    const uint32_t* ta;
    const uint32_t* tf;
    const uint32_t* orders;
    uint64_t* offsets;       // [P][n] or nullptr
    uint64_t* peaks;         // [P]
    uint32_t* status;
    unsigned char* slabs;    // global variant: gridDim.x slabs of 2 * n * kEntryBytes
    uint32_t n;
    uint32_t P;
    uint32_t cap;            // LDS variant: list capacity in entries
};

struct BlockList {
    uint64_t* lo;
    uint64_t* hi;
    uint2* tt;
};

// The side buffer: pending block q lives in lane q of every wave, ascending start address.
struct Pending {
    uint64_t lo, hi;
    uint32_t ta, tf;
};

// f(c): lowest address >= c at which [c, c + s) clears the pending blocks selected by `mask`
// (the ones whose lifetime conflicts with the request), walked in ascending start address.
__device__ __forceinline__ uint64_t clear_pending(uint64_t c, uint64_t s, uint64_t mask, const Pending& pd)
{
    while (mask) {
        const int q = __builtin_ctzll(mask);
        mask &= mask - 1;
        const uint64_t lo = readlane64(pd.lo, q), hi = readlane64(pd.hi, q);
        if (lo < c + s && hi > c) c = hi;
    }
    return c;
}

// Sorted insertion of a block into the register-held side buffer (every wave does the same).
__device__ __forceinline__ void pending_insert(Pending& pd, uint32_t pending, uint64_t x, uint64_t s,
                                               uint32_t ta, uint32_t tf)
{
    const int lane = lane_id();
    const uint64_t keep = __builtin_amdgcn_ballot_w64(lane < (int)pending && pd.lo <= x);
    const int pos = __builtin_popcountll(keep);
    const uint64_t up_lo = wave_shift_up64(pd.lo, 0), up_hi = wave_shift_up64(pd.hi, 0);
    const uint32_t up_ta = __builtin_amdgcn_update_dpp(0u, pd.ta, kDppWaveShr1, 0xf, 0xf, false);
    const uint32_t up_tf = __builtin_amdgcn_update_dpp(0u, pd.tf, kDppWaveShr1, 0xf, 0xf, false);
    if (lane > pos) { pd.lo = up_lo; pd.hi = up_hi; pd.ta = up_ta; pd.tf = up_tf; }
    if (lane == pos) { pd.lo = x; pd.hi = x + s; pd.ta = ta; pd.tf = tf; }
}

// Lowest address x such that [x, x + s) meets neither a listed block nor a pending block whose
// lifetime conflicts with [ta, tf).  The list is sorted by start address.  All threads of the
// workgroup must call this together; the result is uniform.
__device__ __forceinline__ uint64_t
lowest_fit(const BlockList& list, uint32_t count, uint64_t s, uint32_t ta, uint32_t tf,
           const Pending& pd, uint32_t pending, PlanFixedLds& sh)
{
    const int lane = lane_id(), wave = wave_id();
    const uint64_t pmask = __builtin_amdgcn_ballot_w64(lane < (int)pending && pd.ta < tf && ta < pd.tf);
    uint64_t covered = clear_pending(0, s, pmask, pd);      // first address not known to be blocked
    for (uint32_t base = 0;; base += kPlanThreads) {
        const uint32_t k = base + threadIdx.x;
        const bool valid = k < count;
        uint64_t lo = 0, hi = 0;
        uint2 tt = make_uint2(0, 0);
        if (valid) { lo = list.lo[k]; hi = list.hi[k]; tt = list.tt[k]; }
        const bool conflict = valid && tt.x < tf && ta < tt.y;
        uint64_t reach = conflict ? hi : 0;
        if (pmask) reach = clear_pending(reach, s, pmask, pd);
        const uint64_t incl = wave_scan_max64(reach);
        const uint64_t excl = wave_shift_up64(incl, 0);
        if (lane == kWave - 1) sh.wave_top[wave] = incl;
        __syncthreads();
        uint64_t below = covered, all = covered;
#pragma unroll
        for (int w = 0; w < kPlanWaves; ++w) {
            uint64_t t = sh.wave_top[w];
            all = umax64(all, t);
            if (w < wave) below = umax64(below, t);
        }
        const uint64_t before = umax64(below, excl);      // covered up to here when block k is reached
        const bool stop = valid && lo >= before + s;       // hole [before, lo) is large enough
        const uint64_t stops = __builtin_amdgcn_ballot_w64(stop);
        if (lane == 0) sh.wave_hit[wave] = stops ? readlane64(before, __builtin_ctzll(stops)) : kNoHit;
        __syncthreads();
        uint64_t answer = kNoHit;
#pragma unroll
        for (int w = kPlanWaves - 1; w >= 0; --w) {
            uint64_t h = sh.wave_hit[w];
            if (h != kNoHit) answer = h;
        }
        if (answer != kNoHit) return answer;
        covered = all;
        if (base + kPlanThreads >= count) return covered;
    }
}

// Number of sorted pending blocks with start address <= lo.
__device__ __forceinline__ uint32_t pending_at_or_below(const PlanFixedLds& sh, uint32_t pending, uint64_t lo)
{
    uint32_t a = 0, b = pending;
    while (a < b) {
        uint32_t m = (a + b) >> 1;
        if (sh.sorted_lo[m] <= lo) a = m + 1; else b = m;
    }
    return a;
}

// Number of listed blocks with start address < lo.
__device__ __forceinline__ uint32_t listed_below(const uint64_t* list_lo, uint32_t count, uint64_t lo)
{
    uint32_t a = 0, b = count;
    while (a < b) {
        uint32_t m = (a + b) >> 1;
        if (list_lo[m] < lo) a = m + 1; else b = m;
    }
    return a;
}

template <bool kLds>
__global__ void __launch_bounds__(kPlanThreads) plan_kernel(PlanParams prm)
{
    extern __shared__ __align__(16) unsigned char smem[];
    PlanFixedLds& sh = *reinterpret_cast<PlanFixedLds*>(smem);
    const uint32_t n = prm.n;

    if (*prm.status != STALLOC_OK) return;   // malformed trace: nothing to plan (uniform exit)

    BlockList list, spare;
    if constexpr (kLds) {
        unsigned char* dyn = smem + sizeof(PlanFixedLds);
        list.lo = reinterpret_cast<uint64_t*>(dyn);
        list.hi = list.lo + prm.cap;
        list.tt = reinterpret_cast<uint2*>(list.hi + prm.cap);
        spare = list;
    } else {
        unsigned char* slab = prm.slabs + (size_t)blockIdx.x * 2 * (size_t)n * kEntryBytes;
        list.lo = reinterpret_cast<uint64_t*>(slab);
        list.hi = list.lo + n;
        list.tt = reinterpret_cast<uint2*>(list.hi + n);
        spare.lo = reinterpret_cast<uint64_t*>(slab + (size_t)n * kEntryBytes);
        spare.hi = spare.lo + n;
        spare.tt = reinterpret_cast<uint2*>(spare.hi + n);
    }

    for (uint32_t p = blockIdx.x; p < prm.P; p += gridDim.x) {
        const uint32_t* order = prm.orders + (size_t)p * n;
        uint64_t* out = prm.offsets ? prm.offsets + (size_t)p * n : nullptr;
        uint64_t peak = 0;
        uint32_t count = 0, pending = 0;
        Pending pd = {0, 0, 0, 0};

        for (uint32_t r0 = 0; r0 < n; r0 += kBatch) {
            const uint32_t nb = n - r0 < (uint32_t)kBatch ? n - r0 : (uint32_t)kBatch;
            __syncthreads();                                  // previous batch fully consumed
            if (threadIdx.x < nb) {
                uint32_t i = order[r0 + threadIdx.x];
                if (i >= n) { atomicMax(prm.status, (uint32_t)STALLOC_ERR_BAD_ORDER); i = 0; }
                sh.rq_id[threadIdx.x] = i;
                sh.rq_size[threadIdx.x] = prm.size[i];
                sh.rq_ta[threadIdx.x] = prm.ta[i];
                sh.rq_tf[threadIdx.x] = prm.tf[i];
            }
            __syncthreads();

            for (uint32_t b = 0; b < nb; ++b) {
                const uint64_t s = sh.rq_size[b];
                const uint32_t ta = sh.rq_ta[b], tf = sh.rq_tf[b];

                const uint64_t x = lowest_fit(list, count, s, ta, tf, pd, pending, sh);
                peak = umax64(peak, x + s);
                if (threadIdx.x == 0) sh.rq_addr[b] = x;
                pending_insert(pd, pending, x, s, ta, tf);
                ++pending;

                if (pending == kPending && r0 + b + 1 < n) {
                    // merge the side buffer into the sorted list
                    if (threadIdx.x < pending) {             // wave 0 publishes the (sorted) side buffer
                        sh.sorted_lo[threadIdx.x] = pd.lo;
                        sh.sorted_hi[threadIdx.x] = pd.hi;
                        sh.sorted_tt[threadIdx.x] = make_uint2(pd.ta, pd.tf);
                    }
                    __syncthreads();
                    if constexpr (kLds) {
                        constexpr int kMaxPer = 7;           // capacity <= 7 * kPlanThreads entries
                        uint64_t m_lo[kMaxPer], m_hi[kMaxPer];
                        uint2 m_tt[kMaxPer];
                        uint32_t m_to[kMaxPer];
#pragma unroll
                        for (int j = 0; j < kMaxPer; ++j) {
                            const uint32_t k = threadIdx.x + j * kPlanThreads;
                            m_to[j] = 0xffffffffu;
                            if (k < count) {
                                m_lo[j] = list.lo[k];
                                const uint32_t up = pending_at_or_below(sh, pending, m_lo[j]);
                                if (up) { m_hi[j] = list.hi[k]; m_tt[j] = list.tt[k]; m_to[j] = k + up; }
                            }
                        }
                        uint32_t p_to = 0xffffffffu;
                        if (threadIdx.x < pending) p_to = threadIdx.x + listed_below(list.lo, count, sh.sorted_lo[threadIdx.x]);
                        __syncthreads();
#pragma unroll
                        for (int j = 0; j < kMaxPer; ++j)
                            if (m_to[j] != 0xffffffffu) { list.lo[m_to[j]] = m_lo[j]; list.hi[m_to[j]] = m_hi[j]; list.tt[m_to[j]] = m_tt[j]; }
                        if (p_to != 0xffffffffu) {
                            list.lo[p_to] = sh.sorted_lo[threadIdx.x];
                            list.hi[p_to] = sh.sorted_hi[threadIdx.x];
                            list.tt[p_to] = sh.sorted_tt[threadIdx.x];
                        }
                    } else {
                        for (uint32_t k = threadIdx.x; k < count; k += kPlanThreads) {
                            const uint64_t lo = list.lo[k];
                            const uint32_t to = k + pending_at_or_below(sh, pending, lo);
                            spare.lo[to] = lo; spare.hi[to] = list.hi[k]; spare.tt[to] = list.tt[k];
                        }
                        if (threadIdx.x < pending) {
                            const uint32_t to = threadIdx.x + listed_below(list.lo, count, sh.sorted_lo[threadIdx.x]);
                            spare.lo[to] = sh.sorted_lo[threadIdx.x];
                            spare.hi[to] = sh.sorted_hi[threadIdx.x];
                            spare.tt[to] = sh.sorted_tt[threadIdx.x];
                        }
                        BlockList t = list; list = spare; spare = t;
                    }
                    count += pending;
                    pending = 0;
                    __syncthreads();
                }
            }
            // addresses of this batch -> offsets[p][request id]
            __syncthreads();
            if (out && threadIdx.x < nb) out[sh.rq_id[threadIdx.x]] = sh.rq_addr[threadIdx.x];
        }
        if (threadIdx.x == 0) prm.peaks[p] = peak;
    }
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

inline uint32_t lds_capacity_entries(const DeviceInfo& di)
{
    if (di.lds_per_block <= sizeof(PlanFixedLds)) return 0;
    size_t cap = (di.lds_per_block - sizeof(PlanFixedLds)) / kEntryBytes;
    if (cap > 7u * kPlanThreads) cap = 7u * kPlanThreads;
    return (uint32_t)cap;
}

}  // namespace stalloc

using namespace stalloc;

extern "C" uint32_t stalloc_plan_lds_capacity(void)
{
    DeviceInfo di;
    if (!device_info(&di)) return 0;
    return lds_capacity_entries(di);
}

extern "C" int stalloc_plan(const stalloc_trace* tr, const uint32_t* orders, uint32_t P, uint64_t* offsets,
                            uint64_t* peaks, uint64_t* best_offsets, uint32_t* best_plan, uint32_t* device_status,
                            void* workspace, size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || P == 0 || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    DeviceInfo di;
    if (!device_info(&di)) return STALLOC_ERR_DEVICE;
    const uint32_t n = tr->n;
    const uint32_t lds_cap = lds_capacity_entries(di);
    const bool use_lds = n <= lds_cap;
    uint32_t grid = use_lds ? (uint32_t)di.cus : (uint32_t)di.cus * 2;
    if (grid > P) grid = P;

    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(4);
    uint64_t* own_offsets = (!offsets && best_offsets) ? cv.take<uint64_t>((size_t)P * n) : nullptr;
    unsigned char* slabs = use_lds ? nullptr : cv.take<unsigned char>((size_t)grid * 2 * n * kEntryBytes);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!orders || !peaks || !best_plan || !device_status || *workspace_bytes < cv.used ||
        (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);

    PlanParams prm;
    prm.size = tr->size; prm.ta = tr->t_alloc; prm.tf = tr->t_free; prm.orders = orders;
    prm.offsets = offsets ? offsets : own_offsets;
    prm.peaks = peaks; prm.status = device_status; prm.slabs = slabs; prm.n = n; prm.P = P;
    prm.cap = n;
    if (use_lds) {
        const size_t lds_bytes = sizeof(PlanFixedLds) + (size_t)n * kEntryBytes;
        static bool attr_set[64] = {};
        if (!attr_set[di.device]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&plan_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)di.lds_per_block) != hipSuccess)
                return STALLOC_ERR_DEVICE;
            attr_set[di.device] = true;
        }
        hipLaunchKernelGGL(plan_kernel<true>, dim3(grid), dim3(kPlanThreads), lds_bytes, stream, prm);
    } else {
        hipLaunchKernelGGL(plan_kernel<false>, dim3(grid), dim3(kPlanThreads), sizeof(PlanFixedLds), stream, prm);
    }
    hipLaunchKernelGGL(plan_argmin, dim3(1), dim3(256), 0, stream, peaks, P, best_plan, device_status);
    if (best_offsets) {
        uint32_t blocks = (n + 255) / 256;
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(plan_copy_best, dim3(blocks), dim3(256), 0, stream, prm.offsets, best_plan, n, best_offsets,
                           device_status);
    }
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
