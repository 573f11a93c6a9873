// stalloc_make_orders: candidate placement orders, produced on the device.
//
// Row p is a permutation of the request numbers, the stable sort of the requests by a key:
//   p = 0          size descending, then allocation time  (large requests first, so that smaller
//                  ones fill the intervals they leave: Sec. 5.1, Global Planning)
//   p = 1          lifetime descending, then size descending
//   p = 2          allocation time  (the order Algorithm 1 takes a group's requests in)
//   p >= 3, odd    a 64-bit pseudo-random key k(p, i): a uniform random permutation
//   p >= 4, even   (c(i) + 1) * 2^32 + (k(p, i) >> 31), c(i) = number of distinct sizes larger than
//                  request i's: size descending with a random order inside each size and a shift
//                  of up to one size to either side
// k(p, i) = mix(i * 0xD1342543DE82EF95 + mix(seed + p)) modulo 2^64; mix(x) is the output of the
// SplitMix64 generator (Steele, Lea, Flood, OOPSLA 2014) whose state before the step is x.
//
// Every key is packed, with the request number in its lowest 32 bits, into two 64-bit words
// compared in turn; keys of a row are therefore distinct and no tie rule is needed.  A row is
// sorted as tiles of 256 keys in LDS (bitonic network) followed by passes that merge runs in
// pairs: an element's place in the merged run is its place in its own run plus the number of
// elements of the other run that sort before it, found by binary search.  log2(n / 256) passes,
// all rows of a batch side by side in every launch.
#include "host_util.h"
#include "sort_keys.h"
#include "wave.h"

namespace stalloc {

constexpr int kOrTile = kSortTile;

__device__ __forceinline__ uint64_t splitmix64_out(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct OrTrace {
    const uint64_t* size;
    const uint32_t* ta;
    const uint32_t* tf;
    const uint32_t* larger;      // [n] c(i); only read for even rows >= 4
    uint32_t n;
};

// The two key words of request i in row p; slot e past the end gets a key behind every real one.
__device__ __forceinline__ ulonglong2 order_key(const OrTrace& t, uint64_t p, uint64_t stream, uint32_t i, uint32_t e)
{
    ulonglong2 k;
    if (i >= t.n) return filler_key(e);
    if (p == 0) {
        k.x = ~t.size[i];
        k.y = ((uint64_t)t.ta[i] << 32) | i;
    } else if (p == 1) {
        const uint64_t inv_size = ~t.size[i];
        const uint32_t inv_life = ~(t.tf[i] - t.ta[i]);
        k.x = ((uint64_t)inv_life << 32) | (inv_size >> 32);
        k.y = (inv_size << 32) | i;
    } else if (p == 2) {
        k.x = t.ta[i];
        k.y = i;
    } else {
        const uint64_t r = splitmix64_out((uint64_t)i * 0xD1342543DE82EF95ull + stream);
        k.x = (p & 1) ? r : (((uint64_t)t.larger[i] + 1) << 32) + (r >> 31);
        k.y = i;
    }
    return k;
}

// grid (tiles, rows): the keys of one tile of one row, sorted in LDS.
__global__ void __launch_bounds__(kOrTile)
or_sort_tiles(OrTrace t, uint64_t first_plan, uint64_t seed, uint32_t n_pad, ulonglong2* keys, const uint32_t* status)
{
    __shared__ ulonglong2 k[kOrTile];
    if (*status != STALLOC_OK) return;
    const uint32_t th = threadIdx.x, e = blockIdx.x * kOrTile + th;
    const uint64_t p = first_plan + blockIdx.y;
    k[th] = order_key(t, p, splitmix64_out(seed + p), e, e);
    sort_tile(k);
    keys[(size_t)blockIdx.y * n_pad + e] = k[th];
}

// Element e of a row whose runs of `run` keys are merged in pairs: where it goes.
__device__ __forceinline__ uint32_t merged_place(const ulonglong2* row, uint32_t n_pad, uint32_t run, uint32_t e,
                                                 const ulonglong2& me)
{
    const uint32_t mine = e / run;                              // my run; its partner is the other one of the pair
    const uint32_t other0 = (mine ^ 1u) * run;
    uint32_t lo = 0, hi = other0 < n_pad ? (n_pad - other0 < run ? n_pad - other0 : run) : 0u;
    while (lo < hi) {                                           // keys of the partner that sort before mine
        const uint32_t mid = (lo + hi) >> 1;
        if (key_before(row[other0 + mid], me)) lo = mid + 1; else hi = mid;
    }
    return (mine & ~1u) * run + (e - mine * run) + lo;
}

// grid (tiles, rows): runs of `run` keys merged in pairs, src -> dst.
__global__ void __launch_bounds__(kOrTile)
or_merge(const ulonglong2* __restrict__ src, ulonglong2* dst, uint32_t n_pad, uint32_t run, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    const uint32_t e = blockIdx.x * kOrTile + threadIdx.x;
    const ulonglong2* row = src + (size_t)blockIdx.y * n_pad;
    const ulonglong2 me = row[e];
    dst[(size_t)blockIdx.y * n_pad + merged_place(row, n_pad, run, e, me)] = me;
}

// A few short rows in one launch (n^2 / 32 steps a row instead of n log n, but no launch per pass), grid (tiles, rows): thread p of workgroup b holds the key at position p
// of sorted tile b; its place in the row is p plus, for every other tile (staged in LDS), the
// number of that tile's keys that sort before it.
constexpr uint32_t kOrShortRow = 8192;
__global__ void __launch_bounds__(kOrTile)
or_place_short(const ulonglong2* __restrict__ src, ulonglong2* dst, uint32_t n_pad, const uint32_t* status)
{
    __shared__ ulonglong2 k[kOrTile];
    if (*status != STALLOC_OK) return;
    const uint32_t p = threadIdx.x, own = blockIdx.x, tiles = n_pad / kOrTile;
    const ulonglong2* row = src + (size_t)blockIdx.y * n_pad;
    const ulonglong2 me = row[own * kOrTile + p];
    uint32_t place = p;
    for (uint32_t t = 0; t < tiles; ++t) {
        if (t == own) continue;                                  // (uniform)
        __syncthreads();
        k[p] = row[t * kOrTile + p];
        __syncthreads();
        uint32_t lo = 0;                                         // first position of the tile not before `me`
        for (uint32_t half = kOrTile / 2; half > 0; half >>= 1)
            if (key_before(k[lo + half - 1], me)) lo += half;
        place += lo + (key_before(k[lo], me) ? 1u : 0u);         // lo <= 255 here
    }
    dst[(size_t)blockIdx.y * n_pad + place] = me;
}

__global__ void __launch_bounds__(256)
or_emit(const ulonglong2* __restrict__ keys, uint32_t n_pad, uint32_t n, uint32_t* orders, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    const ulonglong2* row = keys + (size_t)blockIdx.y * n_pad;
    uint32_t* out = orders + (size_t)blockIdx.y * n;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x) out[k] = (uint32_t)row[k].y;
}

// Sorted by size descending (row 0): flag[k] = 1 where a new size starts.
__global__ void __launch_bounds__(256)
or_size_flags(const ulonglong2* __restrict__ keys, uint32_t n, uint32_t* flag, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x)
        flag[k] = (k > 0 && keys[k].x != keys[k - 1].x) ? 1u : 0u;
}

// larger[request at sorted position k] = distinct sizes in front of position k.
__global__ void __launch_bounds__(256)
or_size_classes(const ulonglong2* __restrict__ keys, const uint32_t* __restrict__ flag,
                const uint32_t* __restrict__ flags_before, uint32_t n, uint32_t* larger, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x)
        larger[(uint32_t)keys[k].y] = flags_before[k] + flag[k];
}

ulonglong2* launch_merge_tiles(ulonglong2* keys, ulonglong2* spare, uint32_t n_pad, uint32_t rows, const uint32_t* status,
                               hipStream_t stream)
{
    const uint32_t tiles = n_pad / kOrTile;
    ulonglong2 *src = keys, *dst = spare;
    if (tiles == 1) return keys;
    if (n_pad <= kOrShortRow && (uint64_t)rows * tiles <= 2048) {       // few short rows: launches are what costs
        hipLaunchKernelGGL(or_place_short, dim3(tiles, rows), dim3(kOrTile), 0, stream, keys, spare, n_pad, status);
        return spare;
    }
    for (uint64_t run = kOrTile; run < n_pad; run <<= 1) {
        hipLaunchKernelGGL(or_merge, dim3(tiles, rows), dim3(kOrTile), 0, stream, src, dst, n_pad, (uint32_t)run, status);
        ulonglong2* s = src; src = dst; dst = s;
    }
    return src;
}

// Sorts `rows` rows starting at plan first_plan; returns the buffer that holds the result.
static ulonglong2* sort_rows(const OrTrace& t, uint64_t first_plan, uint32_t rows, uint64_t seed, uint32_t n_pad,
                             ulonglong2* buf_a, ulonglong2* buf_b, const uint32_t* status, hipStream_t stream)
{
    hipLaunchKernelGGL(or_sort_tiles, dim3(n_pad / kOrTile, rows), dim3(kOrTile), 0, stream, t, first_plan, seed, n_pad, buf_a,
                       status);
    return launch_merge_tiles(buf_a, buf_b, n_pad, rows, status, stream);
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_make_orders(const stalloc_trace* tr, uint32_t first_plan, uint32_t P, uint64_t seed,
                                   uint32_t* orders, uint32_t* device_status, void* workspace,
                                   size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || P == 0 || (uint64_t)first_plan + P > 0xffffffffull || !workspace_bytes)
        return STALLOC_ERR_INVALID_ARG;
    const uint32_t n = tr->n;
    const uint32_t tiles = (n + kOrTile - 1) / kOrTile;
    const uint32_t n_pad = tiles * kOrTile;
    // rows sorted side by side: as many as 1 GiB of key buffers hold, at most 32768 (grid.y)
    uint64_t batch = (1ull << 30) / (2ull * n_pad * sizeof(ulonglong2));
    if (batch < 1) batch = 1;
    if (batch > 32768) batch = 32768;
    if (batch > P) batch = P;
    const uint32_t chunks = (n + 1023) / 1024;

    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    ulonglong2* buf_a = cv.take<ulonglong2>((size_t)batch * n_pad);
    ulonglong2* buf_b = cv.take<ulonglong2>((size_t)batch * n_pad);
    uint32_t* larger = cv.take<uint32_t>(n);
    uint32_t* flag = cv.take<uint32_t>(n);
    uint32_t* flags_before = cv.take<uint32_t>(n);
    uint32_t* chunk_sum = cv.take<uint32_t>(chunks);
    uint32_t* total = cv.take<uint32_t>(1);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!orders || !device_status || *workspace_bytes < cv.used || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);

    OrTrace t;
    t.size = tr->size; t.ta = tr->t_alloc; t.tf = tr->t_free; t.larger = larger; t.n = n;
    uint32_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    // c(i) for the rows that sort by size with jitter: from the order of row 0
    const uint64_t last = (uint64_t)first_plan + P - 1;
    if (last >= 4) {
        const ulonglong2* by_size = sort_rows(t, 0, 1, seed, n_pad, buf_a, buf_b, device_status, stream);
        hipLaunchKernelGGL(or_size_flags, dim3(blocks), dim3(256), 0, stream, by_size, n, flag, device_status);
        launch_scan(flag, n, flags_before, chunk_sum, total, device_status, stream);
        hipLaunchKernelGGL(or_size_classes, dim3(blocks), dim3(256), 0, stream, by_size, flag, flags_before, n, larger,
                           device_status);
    }
    for (uint64_t p0 = 0; p0 < P; p0 += batch) {
        const uint32_t rows = (uint32_t)(P - p0 < batch ? P - p0 : batch);
        const ulonglong2* sorted = sort_rows(t, (uint64_t)first_plan + p0, rows, seed, n_pad, buf_a, buf_b, device_status, stream);
        uint32_t eb = blocks > 64 ? 64 : blocks;
        hipLaunchKernelGGL(or_emit, dim3(eb, rows), dim3(256), 0, stream, sorted, n_pad, n, orders + (size_t)p0 * n,
                           device_status);
    }
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
