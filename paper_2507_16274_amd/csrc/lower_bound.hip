// stalloc_lower_bound: M_a of Eq. 1 -- the maximum over time of live bytes.
//
// Every request adds +size at t_alloc and -size at t_free into a per-timestamp
// net-change array; an inclusive prefix sum of that array is the number of bytes
// alive at each timestamp (half-open lifetimes: a release at t is already gone at t);
// the answer is the maximum and the earliest timestamp reaching it.
//
// Three launches: lb_clear (net changes, accumulators, status) -> lb_scatter (64-bit atomics,
// integer adds commute so the result is exact; the sanity pass over the trace rides along) ->
// lb_tiles (per tile of timestamps: sum, and maximum of the running sum counted from the tile's
// start; the workgroup that finishes last adds the tiles up and writes the answer and the status).
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kLbThreads = 256;
constexpr int kLbPerThread = 16;
constexpr int kLbTile = kLbThreads * kLbPerThread;
constexpr int kLbAccDone = 10;                 // word of the accumulators that counts finished tiles

struct LbBest {
    int64_t live;
    uint32_t t;
    uint32_t pad;
};

__device__ __forceinline__ bool lb_better(int64_t live_a, uint32_t t_a, int64_t live_b, uint32_t t_b)
{
    return live_a > live_b || (live_a == live_b && t_a < t_b);
}

__global__ void __launch_bounds__(kLbThreads) lb_clear(int64_t* net, uint32_t len, uint64_t* acc, uint32_t* status)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < len; i += gridDim.x * blockDim.x) net[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x < kAccWords) acc[threadIdx.x] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) *status = STALLOC_OK;
}

// Net changes per timestamp, and the trace's sanity on the way: acc[0], acc[1] = sums of the high
// and low halves of the sizes, acc[2] = 1 if a request is malformed.
__global__ void __launch_bounds__(kLbThreads)
lb_scatter(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf,
           uint32_t n, uint32_t t_end, int64_t* net, uint64_t* acc)
{
    __shared__ uint64_t part[kLbThreads / kWave][3];
    uint64_t hi = 0, lo = 0;
    uint32_t bad = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        uint64_t s = size[i];
        uint32_t a = ta[i], f = tf[i];
        bad |= (s == 0) | (a >= f) | (f > t_end);
        hi += s >> 32;               // n < 2^31 terms below 2^32 each: cannot wrap
        lo += s & 0xffffffffull;
        if (a < f && f <= t_end) {   // malformed requests are reported; never index out of range
            atomicAdd((unsigned long long*)&net[a], (unsigned long long)s);
            atomicAdd((unsigned long long*)&net[f], (unsigned long long)(0 - s));
        }
    }
    hi = wave_sum64(hi);
    lo = wave_sum64(lo);
    uint64_t any_bad = __builtin_amdgcn_ballot_w64(bad != 0);
    if (lane_id() == 0) { part[wave_id()][0] = hi; part[wave_id()][1] = lo; part[wave_id()][2] = any_bad ? 1 : 0; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kLbThreads / kWave; ++w) { hi += part[w][0]; lo += part[w][1]; any_bad |= part[w][2]; }
        atomicAdd((unsigned long long*)&acc[0], (unsigned long long)hi);
        atomicAdd((unsigned long long*)&acc[1], (unsigned long long)lo);
        if (any_bad) atomicOr((unsigned long long*)&acc[2], 1ull);
    }
}

// Inclusive sums over the workgroup's threads, in place in lds[kLbThreads].
__device__ __forceinline__ void block_scan(int64_t* lds)
{
    __syncthreads();
    for (int d = 1; d < kLbThreads; d <<= 1) {
        int64_t add = threadIdx.x >= (uint32_t)d ? lds[threadIdx.x - d] : 0;
        __syncthreads();
        lds[threadIdx.x] += add;
        __syncthreads();
    }
}

// The best (live, t) over the workgroup (largest live, earliest t among equals), valid in thread 0.
__device__ __forceinline__ LbBest block_best(int64_t best, uint32_t best_t, LbBest* best_lds)
{
    const uint64_t key = (uint64_t)best ^ (1ull << 63);               // order of int64 as unsigned
    const uint64_t wmax = wave_max64(key);
    const uint64_t wt = wave_min64(key == wmax ? (uint64_t)best_t : ~0ull);
    if (lane_id() == 0) { best_lds[wave_id()].live = (int64_t)(wmax ^ (1ull << 63)); best_lds[wave_id()].t = (uint32_t)wt; }
    __syncthreads();
    LbBest b = best_lds[0];
    for (int k = 1; k < kLbThreads / kWave; ++k)
        if (lb_better(best_lds[k].live, best_lds[k].t, b.live, b.t)) b = best_lds[k];
    b.pad = 0;
    return b;
}

__device__ __forceinline__ int64_t load_coherent(const int64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void __launch_bounds__(kLbThreads)
lb_tiles(const int64_t* __restrict__ net, uint32_t t_end, int64_t* tile_sum, LbBest* tile_best, uint64_t* acc,
         uint64_t* lower_bound, uint32_t* t_at_max, uint32_t* status)
{
    __shared__ int64_t lds[kLbThreads];
    __shared__ LbBest best_lds[kLbThreads / kWave];
    __shared__ uint32_t finished_before;
    // thread owns kLbPerThread consecutive timestamps
    const uint32_t t0 = blockIdx.x * kLbTile + threadIdx.x * kLbPerThread;
    int64_t v[kLbPerThread];
    int64_t mine = 0;
#pragma unroll
    for (int j = 0; j < kLbPerThread; ++j) {
        const uint32_t t = t0 + j;
        v[j] = t < t_end ? net[t] : 0;
        mine += v[j];
    }
    lds[threadIdx.x] = mine;
    block_scan(lds);
    int64_t live = lds[threadIdx.x] - mine;                            // running sum from the tile's start, before t0
    const int64_t tile_total = lds[kLbThreads - 1];
    int64_t best = INT64_MIN;
    uint32_t best_t = 0xffffffffu;
#pragma unroll
    for (int j = 0; j < kLbPerThread; ++j) {
        const uint32_t t = t0 + j;
        live += v[j];
        if (t < t_end && lb_better(live, t, best, best_t)) { best = live; best_t = t; }
    }
    const LbBest b = block_best(best, best_t, best_lds);
    if (threadIdx.x == 0) {
        tile_sum[blockIdx.x] = tile_total;
        tile_best[blockIdx.x] = b;
        __threadfence();
        finished_before = (uint32_t)atomicAdd((unsigned long long*)&acc[kLbAccDone], 1ull);
    }
    __syncthreads();
    if (finished_before != gridDim.x - 1) return;
    // the last tile to finish: bytes alive at a tile's start = sum of the tiles before it
    __threadfence();
    int64_t carry = 0;
    best = INT64_MIN;
    best_t = 0xffffffffu;
    for (uint32_t base = 0; base < gridDim.x; base += kLbThreads) {
        const uint32_t k = base + threadIdx.x;
        const int64_t sum = k < gridDim.x ? load_coherent(&tile_sum[k]) : 0;
        __syncthreads();
        lds[threadIdx.x] = sum;
        block_scan(lds);
        if (k < gridDim.x) {
            const int64_t cand = carry + lds[threadIdx.x] - sum + load_coherent(&tile_best[k].live);
            const uint32_t cand_t = __hip_atomic_load(&tile_best[k].t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lb_better(cand, cand_t, best, best_t)) { best = cand; best_t = cand_t; }
        }
        carry += lds[kLbThreads - 1];
    }
    __syncthreads();
    LbBest all = block_best(best, best_t, best_lds);
    if (threadIdx.x == 0) {
        // a maximum of zero live bytes is reported at t = 0
        if (all.live <= 0) { all.live = 0; all.t = 0; }
        *lower_bound = (uint64_t)all.live;
        if (t_at_max) *t_at_max = all.t;
        // total = acc[0] * 2^32 + acc[1]  >= 2^63  <=>  acc[0] + (acc[1] >> 32) >= 2^31
        const uint64_t hi = acc[0], lo = acc[1];
        uint32_t code = STALLOC_OK;
        if (hi + (lo >> 32) >= (1ull << 31)) code = STALLOC_ERR_OVERFLOW;
        if (acc[2] & 1ull) code = STALLOC_ERR_BAD_TRACE;
        if (code != STALLOC_OK) atomicMax(status, code);
    }
}

// Pieces of the scratch memory one call needs, carved from `base` (nullptr: sizes only).
struct LbScratch {
    uint64_t* acc;
    int64_t* net;
    int64_t* tile_sum;
    LbBest* tile_best;
    uint32_t tiles;
    size_t bytes;
    LbScratch(void* base, uint32_t t_end)
    {
        tiles = (t_end + kLbTile - 1) / kLbTile;
        Carver cv(base);
        acc = cv.take<uint64_t>(kAccWords);
        net = cv.take<int64_t>((size_t)t_end + 1);
        tile_sum = cv.take<int64_t>(tiles);
        tile_best = cv.take<LbBest>(tiles);
        bytes = cv.used;
    }
};

static int enqueue_lower_bound(const stalloc_trace& tr, uint64_t* lower_bound, uint32_t* t_at_max,
                               uint32_t* device_status, const LbScratch& sc, hipStream_t stream)
{
    const uint32_t t_end = tr.t_end;
    uint32_t clear_blocks = (t_end + 1 + kLbThreads - 1) / kLbThreads;
    if (clear_blocks > 4096) clear_blocks = 4096;
    hipLaunchKernelGGL(lb_clear, dim3(clear_blocks), dim3(kLbThreads), 0, stream, sc.net, t_end + 1, sc.acc, device_status);
    uint32_t sc_blocks = (tr.n + kLbThreads - 1) / kLbThreads;
    if (sc_blocks > 4096) sc_blocks = 4096;
    hipLaunchKernelGGL(lb_scatter, dim3(sc_blocks), dim3(kLbThreads), 0, stream, tr.size, tr.t_alloc, tr.t_free,
                       tr.n, t_end, sc.net, sc.acc);
    hipLaunchKernelGGL(lb_tiles, dim3(sc.tiles), dim3(kLbThreads), 0, stream, sc.net, t_end, sc.tile_sum, sc.tile_best,
                       sc.acc, lower_bound, t_at_max, device_status);
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}

// Scratch memory of stalloc_lower_bound_static: one copy per GPU, resident from the moment the
// library is loaded on that GPU until the process ends.  Host code never uses this name as an
// address; it asks the runtime for the device address once per device (static_scratch()).
constexpr uint32_t kStaticMaxTEnd = STALLOC_STATIC_MAX_T_END;
constexpr size_t kStaticScratchBytes =
    kAlign * 4 + sizeof(uint64_t) * kAccWords + sizeof(int64_t) * ((size_t)kStaticMaxTEnd + 1) +
    (sizeof(int64_t) + sizeof(LbBest)) * ((kStaticMaxTEnd + kLbTile - 1) / kLbTile);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (nullptr if the runtime refuses).
static void* static_scratch()
{
    static void* ptr[64] = {};
    static std::mutex guard;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(guard);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        ptr[dev] = p;
    }
    return ptr[dev];
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_lower_bound(const stalloc_trace* tr, uint64_t* lower_bound, uint32_t* t_at_max,
                                   uint32_t* device_status, void* workspace, size_t* workspace_bytes,
                                   void* hip_stream)
{
    if (!trace_args_ok(tr) || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    const LbScratch sc(workspace, tr->t_end);
    if (!workspace) { *workspace_bytes = sc.bytes; return STALLOC_OK; }
    if (!lower_bound || !device_status || *workspace_bytes < sc.bytes ||
        (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    return enqueue_lower_bound(*tr, lower_bound, t_at_max, device_status, sc, static_cast<hipStream_t>(hip_stream));
}

extern "C" int stalloc_lower_bound_static(const stalloc_trace* tr, uint64_t* lower_bound, uint32_t* t_at_max,
                                          uint32_t* device_status, void* hip_stream)
{
    if (!trace_args_ok(tr) || !lower_bound || !device_status) return STALLOC_ERR_INVALID_ARG;
    if (tr->t_end > kStaticMaxTEnd) return STALLOC_ERR_TOO_LARGE;
    void* base = static_scratch();
    if (!base) return STALLOC_ERR_DEVICE;
    const LbScratch sc(base, tr->t_end);
    if (sc.bytes > kStaticScratchBytes) return STALLOC_ERR_TOO_LARGE;
    // every word of the scratch memory a call reads is written by that call first (lb_clear resets
    // the net changes and the accumulators), so what the last call left is harmless
    return enqueue_lower_bound(*tr, lower_bound, t_at_max, device_status, sc, static_cast<hipStream_t>(hip_stream));
}
