// stalloc_fuse_groups: candidate fusions of HomoPhase groups (Sec. 5.1, HomoPhase Group Planning),
// many at once, one workgroup per candidate pair of groups.
//
// A HomoPhase group holds the requests allocated in one computation phase and released in one
// (other) phase; its local plan packs them contiguously.  Two plans are fused by inserting the
// smaller into the larger: the larger plan is packed from 0 in descending order of release time;
// an address pointer starts at its lowest start address; the requests of the smaller plan are
// tried in order of allocation time, the first that conflicts with nothing when put at the
// pointer is placed there and the pointer moves up by its size; if none fits the pointer moves to
// the next higher start address of the larger plan; what is left when those run out is packed on
// top.  The fusion is accepted if its time-memory product (Eq. 2) exceeds the average of the two
// plans' products weighted by the memory-time each reserves, i.e. if the fused plan reserves less
// memory-time (extent x span) than the two together.
//
// Per pair everything lives in LDS.  Sorting is by counting (an element's place is the number of
// elements that sort before it).  The insertion is a chain of steps; inside a step every thread
// tests candidates of the smaller plan against the blocks of the larger plan whose address range
// meets [pointer, pointer + size) -- the larger plan is contiguous and sorted by address, so those
// are the blocks from the one that holds the pointer upwards -- and the earliest fitting
// candidate is found with an LDS minimum.  (Requests of the smaller plan that are already placed
// lie below the pointer and cannot be met.)
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kFuThreads = 256;

struct FuseParams {
    const uint64_t* size;
    const uint32_t* ta;
    const uint32_t* tf;
    const uint32_t* members;
    const uint32_t* pair_begin;
    const uint32_t* count1;
    uint32_t* order;
    uint64_t* addr;
    uint64_t* extents;
    uint32_t* accepted;
    uint32_t* status;
    uint32_t n;
    uint32_t entries;        // length of members / order / addr
    uint32_t cap;            // requests of one pair that fit the LDS arrays
};

__device__ __forceinline__ uint64_t block_sum64(uint64_t v, uint64_t* scratch)
{
    const uint64_t w = wave_sum64(v);
    __syncthreads();
    if (lane_id() == 0) scratch[wave_id()] = w;
    __syncthreads();
    uint64_t tot = 0;
    for (int k = 0; k < kFuThreads / kWave; ++k) tot += scratch[k];
    return tot;
}

// a * b as a 96-bit number {high 32 bits, low 64 bits}
__device__ __forceinline__ void mul_64_32(uint64_t a, uint32_t b, uint64_t& hi, uint64_t& lo)
{
    lo = a * (uint64_t)b;
    hi = __umul64hi(a, (uint64_t)b);
}

__global__ void __launch_bounds__(kFuThreads) fuse_pairs(FuseParams prm)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint64_t scratch[kFuThreads / kWave];
    __shared__ uint32_t found_at;
    __shared__ uint32_t t_lo[2], t_hi[2];
    if (*prm.status != STALLOC_OK) return;
    const uint32_t p = blockIdx.x, tid = threadIdx.x;
    const uint32_t m0 = prm.pair_begin[p], m1 = prm.pair_begin[p + 1], m = m1 - m0, c1 = prm.count1[p];
    const bool outside = m1 < m0 || m1 > prm.entries;               // (nothing is read or written beyond the arrays)
    if (outside || m > prm.cap || c1 == 0 || c1 >= m) {             // (uniform) nothing sensible to do
        if (tid == 0) atomicMax(prm.status, (uint32_t)(!outside && m > prm.cap ? STALLOC_ERR_TOO_LARGE : STALLOC_ERR_INVALID_ARG));
        return;
    }
    uint32_t* id = reinterpret_cast<uint32_t*>(smem);                 // [cap] request numbers, as given
    uint32_t* srt = id + prm.cap;                                     // [cap] the fused plan's order
    uint64_t* sz = reinterpret_cast<uint64_t*>(srt + prm.cap);        // [cap] in the fused plan's order:
    uint64_t* at = sz + prm.cap;                                      //       size, address,
    uint32_t* ts = reinterpret_cast<uint32_t*>(at + prm.cap);         //       lifetime
    uint32_t* te = ts + prm.cap;
    if (tid < 2) { t_lo[tid] = 0xffffffffu; t_hi[tid] = 0u; }
    __syncthreads();
    // the two local plans: extent = sum of sizes, span = first allocation .. last release
    uint64_t sum1 = 0, sum2 = 0;
    for (uint32_t k = tid; k < m; k += kFuThreads) {
        uint32_t i = prm.members[m0 + k];
        if (i >= prm.n) { atomicMax(prm.status, (uint32_t)STALLOC_ERR_BAD_ORDER); i = 0; }
        id[k] = i;
        srt[k] = 0;                                                   // (a request listed twice leaves places empty)
        const int g = k < c1 ? 0 : 1;
        (g ? sum2 : sum1) += prm.size[i];
        const uint32_t a = prm.ta[i], f = prm.tf[i];
        ts[k] = a; te[k] = f;                                         // (as given, for the sort)
        atomicMin(&t_lo[g], a);
        atomicMax(&t_hi[g], f);
    }
    const uint64_t ext1 = block_sum64(sum1, scratch), ext2 = block_sum64(sum2, scratch);
    __syncthreads();
    const bool first_larger = ext1 >= ext2;
    const uint32_t nl = first_larger ? c1 : m - c1, ns = m - nl;
    const uint32_t l0 = first_larger ? 0 : c1, s0 = first_larger ? c1 : 0;     // where the two groups start in id[]
    // larger plan: by release time, latest first (request number among equals); smaller plan: by
    // allocation time (request number among equals).  Place = elements that sort before.
    for (uint32_t k = tid; k < m; k += kFuThreads) {
        const bool in_larger = k >= l0 && k < l0 + nl;
        const uint32_t i = id[k];
        const uint32_t* keys = in_larger ? te : ts;
        const uint32_t key = keys[k];
        const uint32_t g0 = in_larger ? l0 : s0, gn = in_larger ? nl : ns;
        uint32_t place = 0;
        for (uint32_t q = g0; q < g0 + gn; ++q) {
            const uint32_t j = id[q], other = keys[q];
            const bool before = other == key ? j < i : (other > key) == in_larger;
            place += before ? 1u : 0u;
        }
        srt[(in_larger ? 0 : nl) + place] = i;
    }
    __syncthreads();
    for (uint32_t k = tid; k < m; k += kFuThreads) {
        const uint32_t i = srt[k];
        sz[k] = prm.size[i]; ts[k] = prm.ta[i]; te[k] = prm.tf[i];
        at[k] = ~0ull;                                                // (smaller plan: not placed yet)
    }
    __syncthreads();
    if (tid == 0) {                                                   // the larger plan, packed from 0
        uint64_t top = 0;
        for (uint32_t k = 0; k < nl; ++k) { at[k] = top; top += sz[k]; }
    }
    __syncthreads();
    // insertion of the smaller plan
    uint64_t addr = 0;                                                // lowest start address of the larger plan
    uint32_t holder = 0;                                              // block of the larger plan with at[holder] <= addr < at[holder + 1]
    uint32_t left = ns;
    while (left) {
        while (holder + 1 < nl && at[holder + 1] <= addr) ++holder;
        if (tid == 0) found_at = 0xffffffffu;
        __syncthreads();
        for (uint32_t k = tid; k < ns; k += kFuThreads) {
            if (at[nl + k] != ~0ull) continue;                        // placed already
            if (k > found_at) break;                                  // (an earlier candidate fits; racy reads only skip work)
            const uint64_t end = addr + sz[nl + k];
            bool clash = false;
            for (uint32_t q = holder; q < nl && at[q] < end && !clash; ++q)
                clash = at[q] + sz[q] > addr && ts[q] < te[nl + k] && ts[nl + k] < te[q];
            if (!clash) atomicMin(&found_at, k);
        }
        __syncthreads();
        const uint32_t fit = found_at;
        __syncthreads();
        if (fit != 0xffffffffu) {
            if (tid == 0) at[nl + fit] = addr;
            addr += sz[nl + fit];
            --left;
            __syncthreads();
        } else {
            // on to the next higher start address of the larger plan, if there is one (start
            // addresses are distinct and at[0] = 0 <= addr, so that is the holder's successor)
            if (holder + 1 >= nl) break;
            addr = at[holder + 1];
        }
    }
    __syncthreads();
    // what is left goes on top of everything placed
    if (tid == 0) {
        uint64_t top = 0;
        for (uint32_t k = 0; k < m; ++k)
            if (at[k] != ~0ull && at[k] + sz[k] > top) top = at[k] + sz[k];
        for (uint32_t k = nl; k < m; ++k)
            if (at[k] == ~0ull) { at[k] = top; top += sz[k]; }
        const uint32_t lo_f = t_lo[0] < t_lo[1] ? t_lo[0] : t_lo[1], hi_f = t_hi[0] > t_hi[1] ? t_hi[0] : t_hi[1];
        uint64_t h1, l1, h2, l2, hf, lf;
        mul_64_32(ext1, t_hi[0] - t_lo[0], h1, l1);
        mul_64_32(ext2, t_hi[1] - t_lo[1], h2, l2);
        mul_64_32(top, hi_f - lo_f, hf, lf);
        const uint64_t ls = l1 + l2, hs = h1 + h2 + (ls < l1 ? 1 : 0);
        prm.extents[3 * (size_t)p] = ext1;
        prm.extents[3 * (size_t)p + 1] = ext2;
        prm.extents[3 * (size_t)p + 2] = top;
        prm.accepted[p] = (hf < hs || (hf == hs && lf < ls)) ? 1u : 0u;
    }
    __syncthreads();
    for (uint32_t k = tid; k < m; k += kFuThreads) {
        prm.order[m0 + k] = srt[k];
        prm.addr[m0 + k] = at[k];
    }
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_fuse_groups(const stalloc_trace* tr, const uint32_t* members, const uint32_t* pair_begin,
                                   const uint32_t* count1, uint32_t k, uint32_t m, uint32_t largest_pair, uint32_t* order,
                                   uint64_t* addr, uint64_t* extents, uint32_t* accepted, uint32_t* device_status,
                                   void* workspace, size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || k == 0 || largest_pair < 2 || m < 2 || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    DeviceInfo di;
    if (!device_info(&di)) return STALLOC_ERR_DEVICE;
    const size_t per_request = 2 * sizeof(uint32_t) + 2 * sizeof(uint64_t) + 2 * sizeof(uint32_t);
    const size_t lds_budget = di.lds_per_block - 1024;
    if ((size_t)largest_pair * per_request > lds_budget) return STALLOC_ERR_TOO_LARGE;
    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!members || !pair_begin || !count1 || !order || !addr || !extents || !accepted || !device_status ||
        *workspace_bytes < cv.used || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    launch_trace_check(*tr, acc, device_status, stream);
    static std::atomic<bool> attr_set[64] = {};        // (set twice at worst when threads race)
    if (!attr_set[di.device]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&fuse_pairs), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds_budget) != hipSuccess)     // (the kernel's static LDS takes the rest)
            return STALLOC_ERR_DEVICE;
        attr_set[di.device] = true;
    }
    FuseParams prm;
    prm.size = tr->size; prm.ta = tr->t_alloc; prm.tf = tr->t_free; prm.members = members; prm.pair_begin = pair_begin;
    prm.count1 = count1; prm.order = order; prm.addr = addr; prm.extents = extents; prm.accepted = accepted;
    prm.status = device_status; prm.n = tr->n; prm.entries = m;
    prm.cap = (largest_pair + 1) & ~1u;                               // (keeps the 64-bit arrays aligned)
    hipLaunchKernelGGL(fuse_pairs, dim3(k), dim3(kFuThreads), (size_t)prm.cap * per_request, stream, prm);
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
