// stalloc_lower_bound: M_a of Eq. 1 -- the maximum over time of live bytes.
//
// Every request adds +size at t_alloc and -size at t_free into a per-timestamp
// net-change array; an inclusive prefix sum of that array is the number of bytes
// alive at each timestamp (half-open lifetimes: a release at t is already gone at t);
// the answer is the maximum and the earliest timestamp reaching it.
//
// Kernels: clear -> scatter (64-bit atomics, integer adds commute so the result is
// exact) -> per-tile sums -> scan of tile sums (one workgroup) -> per-tile running
// sum + maximum -> final reduction (one workgroup).
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kLbThreads = 256;
constexpr int kLbPerThread = 16;
constexpr int kLbTile = kLbThreads * kLbPerThread;

struct LbBest {
    int64_t live;
    uint32_t t;
    uint32_t pad;
};

__device__ __forceinline__ bool lb_better(int64_t live_a, uint32_t t_a, int64_t live_b, uint32_t t_b)
{
    return live_a > live_b || (live_a == live_b && t_a < t_b);
}

__global__ void __launch_bounds__(kLbThreads) lb_clear(int64_t* net, uint32_t len)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < len; i += gridDim.x * blockDim.x) net[i] = 0;
}

__global__ void __launch_bounds__(kLbThreads)
lb_scatter(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf,
           uint32_t n, uint32_t t_end, int64_t* net)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        uint64_t s = size[i];
        uint32_t a = ta[i], f = tf[i];
        if (a < f && f <= t_end) {   // malformed requests are reported by the trace check; never index out of range
            atomicAdd((unsigned long long*)&net[a], (unsigned long long)s);
            atomicAdd((unsigned long long*)&net[f], (unsigned long long)(0 - s));
        }
    }
}

// Block-wide sum of one int64 per thread; result valid in every thread.
__device__ __forceinline__ int64_t block_sum(int64_t v, int64_t* lds)
{
    int64_t w = (int64_t)wave_sum64((uint64_t)v);
    __syncthreads();
    if (lane_id() == 0) lds[wave_id()] = w;
    __syncthreads();
    int64_t tot = 0;
    for (int k = 0; k < kLbThreads / kWave; ++k) tot += lds[k];
    return tot;
}

__global__ void __launch_bounds__(kLbThreads)
lb_tile_sums(const int64_t* __restrict__ net, uint32_t t_end, int64_t* tile_sum)
{
    __shared__ int64_t lds[kLbThreads / kWave];
    uint32_t base = blockIdx.x * kLbTile;
    int64_t acc = 0;
    for (int j = 0; j < kLbPerThread; ++j) {
        uint32_t t = base + j * kLbThreads + threadIdx.x;
        if (t < t_end) acc += net[t];
    }
    int64_t tot = block_sum(acc, lds);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = tot;
}

// Exclusive scan of the tile sums, in place, by one workgroup.
__global__ void __launch_bounds__(kLbThreads) lb_scan_tiles(int64_t* tile_sum, uint32_t tiles)
{
    __shared__ int64_t lds[kLbThreads];
    int64_t carry = 0;
    for (uint32_t base = 0; base < tiles; base += kLbThreads) {
        uint32_t k = base + threadIdx.x;
        int64_t v = k < tiles ? tile_sum[k] : 0;
        lds[threadIdx.x] = v;
        __syncthreads();
        for (int d = 1; d < kLbThreads; d <<= 1) {
            int64_t add = threadIdx.x >= (uint32_t)d ? lds[threadIdx.x - d] : 0;
            __syncthreads();
            lds[threadIdx.x] += add;
            __syncthreads();
        }
        int64_t incl = lds[threadIdx.x];
        int64_t total = lds[kLbThreads - 1];
        if (k < tiles) tile_sum[k] = carry + incl - v;
        carry += total;
        __syncthreads();
    }
}

__global__ void __launch_bounds__(kLbThreads)
lb_tile_max(const int64_t* __restrict__ net, uint32_t t_end, const int64_t* __restrict__ tile_prefix, LbBest* tile_best)
{
    __shared__ int64_t lds[kLbThreads];
    __shared__ LbBest best_lds[kLbThreads / kWave];
    // thread owns kLbPerThread consecutive timestamps
    uint32_t t0 = blockIdx.x * kLbTile + threadIdx.x * kLbPerThread;
    int64_t v[kLbPerThread];
    int64_t mine = 0;
#pragma unroll
    for (int j = 0; j < kLbPerThread; ++j) {
        uint32_t t = t0 + j;
        v[j] = t < t_end ? net[t] : 0;
        mine += v[j];
    }
    lds[threadIdx.x] = mine;
    __syncthreads();
    for (int d = 1; d < kLbThreads; d <<= 1) {
        int64_t add = threadIdx.x >= (uint32_t)d ? lds[threadIdx.x - d] : 0;
        __syncthreads();
        lds[threadIdx.x] += add;
        __syncthreads();
    }
    int64_t live = tile_prefix[blockIdx.x] + lds[threadIdx.x] - mine;   // bytes alive just before t0
    int64_t best = -1;
    uint32_t best_t = 0xffffffffu;
#pragma unroll
    for (int j = 0; j < kLbPerThread; ++j) {
        uint32_t t = t0 + j;
        live += v[j];
        if (t < t_end && lb_better(live, t, best, best_t)) { best = live; best_t = t; }
    }
    // reduce (best, best_t) over the block: pack-free two-step (max live, then min t among holders)
    uint64_t wmax = wave_max64((uint64_t)(best + 1));                 // best >= -1, so best + 1 >= 0
    uint64_t cand_t = ((uint64_t)(best + 1) == wmax) ? (uint64_t)best_t : ~0ull;
    uint64_t wt = wave_min64(cand_t);
    if (lane_id() == 0) { best_lds[wave_id()].live = (int64_t)wmax - 1; best_lds[wave_id()].t = (uint32_t)wt; }
    __syncthreads();
    if (threadIdx.x == 0) {
        LbBest b = best_lds[0];
        for (int k = 1; k < kLbThreads / kWave; ++k)
            if (lb_better(best_lds[k].live, best_lds[k].t, b.live, b.t)) b = best_lds[k];
        b.pad = 0;
        tile_best[blockIdx.x] = b;
    }
}

__global__ void __launch_bounds__(kLbThreads)
lb_final(const LbBest* __restrict__ tile_best, uint32_t tiles, uint64_t* lower_bound, uint32_t* t_at_max)
{
    __shared__ LbBest best_lds[kLbThreads / kWave];
    int64_t best = -1;
    uint32_t best_t = 0xffffffffu;
    for (uint32_t k = threadIdx.x; k < tiles; k += kLbThreads) {
        LbBest b = tile_best[k];
        if (lb_better(b.live, b.t, best, best_t)) { best = b.live; best_t = b.t; }
    }
    uint64_t wmax = wave_max64((uint64_t)(best + 1));
    uint64_t cand_t = ((uint64_t)(best + 1) == wmax) ? (uint64_t)best_t : ~0ull;
    uint64_t wt = wave_min64(cand_t);
    if (lane_id() == 0) { best_lds[wave_id()].live = (int64_t)wmax - 1; best_lds[wave_id()].t = (uint32_t)wt; }
    __syncthreads();
    if (threadIdx.x == 0) {
        LbBest b = best_lds[0];
        for (int k = 1; k < kLbThreads / kWave; ++k)
            if (lb_better(best_lds[k].live, best_lds[k].t, b.live, b.t)) b = best_lds[k];
        // a maximum of zero live bytes is reported at t = 0
        if (b.live <= 0) { b.live = 0; b.t = 0; }
        *lower_bound = (uint64_t)b.live;
        if (t_at_max) *t_at_max = b.t;
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
    launch_trace_check(tr, sc.acc, device_status, stream);
    uint32_t clear_blocks = (t_end + 1 + kLbThreads - 1) / kLbThreads;
    if (clear_blocks > 4096) clear_blocks = 4096;
    hipLaunchKernelGGL(lb_clear, dim3(clear_blocks), dim3(kLbThreads), 0, stream, sc.net, t_end + 1);
    uint32_t sc_blocks = (tr.n + kLbThreads - 1) / kLbThreads;
    if (sc_blocks > 4096) sc_blocks = 4096;
    hipLaunchKernelGGL(lb_scatter, dim3(sc_blocks), dim3(kLbThreads), 0, stream, tr.size, tr.t_alloc, tr.t_free,
                       tr.n, t_end, sc.net);
    hipLaunchKernelGGL(lb_tile_sums, dim3(sc.tiles), dim3(kLbThreads), 0, stream, sc.net, t_end, sc.tile_sum);
    hipLaunchKernelGGL(lb_scan_tiles, dim3(1), dim3(kLbThreads), 0, stream, sc.tile_sum, sc.tiles);
    hipLaunchKernelGGL(lb_tile_max, dim3(sc.tiles), dim3(kLbThreads), 0, stream, sc.net, t_end, sc.tile_sum,
                       sc.tile_best);
    hipLaunchKernelGGL(lb_final, dim3(1), dim3(kLbThreads), 0, stream, sc.tile_best, sc.tiles, lower_bound, t_at_max);
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
    // every word of the scratch memory a call reads is written by that call first (the trace
    // check resets its accumulators, lb_clear the net changes), so what the last call left is harmless
    return enqueue_lower_bound(*tr, lower_bound, t_at_max, device_status, sc, static_cast<hipStream_t>(hip_stream));
}
