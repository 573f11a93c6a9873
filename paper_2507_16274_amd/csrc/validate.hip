// stalloc_validate: pairwise check of the planning constraint of Sec. 5.1 -- no two
// allocation decisions may conflict in lifespan and in address range at once.
//
// All n(n-1)/2 unordered pairs of every plan are tested.  The pair space is cut into
// 256 x 256 tiles (upper triangle only); one workgroup owns one tile of one plan: each
// thread keeps its own request i in registers and walks the 256 requests j of the tile,
// which sit in LDS and are read as broadcasts.  Per plan the kernel accumulates the
// number of conflicting pairs and the smallest key (i << 32 | j), i < j, which is the
// lexicographically first conflicting pair.
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kValTile = 256;

__global__ void val_init(uint64_t* conflicts, uint64_t* first_key, uint32_t P)
{
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < P; p += gridDim.x * blockDim.x) {
        conflicts[p] = 0;
        first_key[p] = ~0ull;
    }
}

__global__ void __launch_bounds__(kValTile)
val_pairs(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf,
          const uint64_t* __restrict__ offsets, uint32_t n, uint32_t tiles, uint32_t plan0,
          uint64_t* conflicts, uint64_t* first_key, uint32_t* status)
{
    __shared__ uint64_t j_lo[kValTile];
    __shared__ uint64_t j_hi[kValTile];
    __shared__ uint32_t j_ta[kValTile];
    __shared__ uint32_t j_tf[kValTile];

    // linear tile index -> (ti, tj) with ti <= tj, row-major over the upper triangle
    const uint32_t lin = blockIdx.x;
    const double nt = (double)tiles;
    uint32_t ti = (uint32_t)((2.0 * nt + 1.0 - sqrt((2.0 * nt + 1.0) * (2.0 * nt + 1.0) - 8.0 * (double)lin)) * 0.5);
    if (ti >= tiles) ti = tiles - 1;
    // row ti starts at ti*tiles - ti*(ti-1)/2; fix rounding either way
    auto row_start = [&](uint32_t r) { return (uint64_t)r * tiles - (uint64_t)r * (r - 1) / 2; };
    while (ti > 0 && row_start(ti) > lin) --ti;
    while (ti + 1 < tiles && row_start(ti + 1) <= lin) ++ti;
    const uint32_t tj = ti + (uint32_t)(lin - row_start(ti));

    const uint32_t p = plan0 + blockIdx.y;
    const uint64_t* off = offsets + (size_t)p * n;

    const uint32_t j0 = tj * kValTile;
    {
        uint32_t j = j0 + threadIdx.x;
        bool ok = j < n;
        uint64_t o = ok ? off[j] : 0, s = ok ? size[j] : 0;
        // an address range that would run past 2^64 is reported, and kept from wrapping so that
        // what it covers still counts
        if (o + s < o) { atomicMax(status, (uint32_t)STALLOC_ERR_OVERFLOW); s = ~o; }
        j_lo[threadIdx.x] = o;
        j_hi[threadIdx.x] = o + s;
        j_ta[threadIdx.x] = ok ? ta[j] : 0;
        j_tf[threadIdx.x] = ok ? tf[j] : 0;     // empty lifetime [0,0): conflicts with nothing
    }
    const uint32_t i = ti * kValTile + threadIdx.x;
    const bool i_ok = i < n;
    const uint64_t i_lo = i_ok ? off[i] : 0;
    const uint64_t i_size = i_ok ? size[i] : 0;
    const uint64_t i_hi = i_lo + i_size < i_lo ? ~0ull : i_lo + i_size;
    const uint32_t i_ta = i_ok ? ta[i] : 0;
    const uint32_t i_tf = i_ok ? tf[i] : 0;
    __syncthreads();

    uint32_t count = 0;
    uint32_t min_j = 0xffffffffu;
    // on the diagonal tile only j > i counts
    const uint32_t first = (ti == tj) ? threadIdx.x + 1 : 0;
#pragma unroll 8
    for (uint32_t q = 0; q < kValTile; ++q) {
        bool hit = (q >= first) & (j_ta[q] < i_tf) & (i_ta < j_tf[q]) & (j_lo[q] < i_hi) & (i_lo < j_hi[q]);
        if (hit) {
            ++count;
            uint32_t j = j0 + q;
            min_j = j < min_j ? j : min_j;
        }
    }
    uint64_t key = count ? (((uint64_t)i << 32) | min_j) : ~0ull;
    uint32_t wave_count = wave_sum32(count);
    uint64_t wave_key = wave_min64(key);
    if (lane_id() == 0 && wave_count) {
        atomicAdd((unsigned long long*)&conflicts[p], (unsigned long long)wave_count);
        atomicMin((unsigned long long*)&first_key[p], (unsigned long long)wave_key);
    }
}

__global__ void val_finish(const uint64_t* first_key, uint32_t* first_pair, uint32_t P)
{
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < P; p += gridDim.x * blockDim.x) {
        uint64_t k = first_key[p];
        first_pair[2 * p] = (uint32_t)(k >> 32);
        first_pair[2 * p + 1] = (uint32_t)k;
    }
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_validate(const stalloc_trace* tr, const uint64_t* offsets, uint32_t P, uint64_t* conflicts,
                                uint32_t* first_pair, uint32_t* device_status, void* workspace,
                                size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || P == 0 || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    const uint64_t tiles = ((uint64_t)tr->n + kValTile - 1) / kValTile;
    const uint64_t tri = tiles * (tiles + 1) / 2;
    if (tri >= 0x7fffffffull) return STALLOC_ERR_INVALID_ARG;   // n beyond ~16.7 million requests
    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    uint64_t* first_key = cv.take<uint64_t>(P);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!offsets || !conflicts || !first_pair || !device_status || *workspace_bytes < cv.used ||
        (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);
    uint32_t pb = (P + 255) / 256;
    if (pb > 1024) pb = 1024;
    hipLaunchKernelGGL(val_init, dim3(pb), dim3(256), 0, stream, conflicts, first_key, P);
    for (uint32_t p0 = 0; p0 < P; p0 += 32768) {          // grid.y is limited to 65535
        uint32_t py = P - p0 < 32768 ? P - p0 : 32768;
        hipLaunchKernelGGL(val_pairs, dim3((uint32_t)tri, py), dim3(kValTile), 0, stream, tr->size, tr->t_alloc,
                           tr->t_free, offsets, tr->n, (uint32_t)tiles, p0, conflicts, first_key,
                           device_status);
    }
    hipLaunchKernelGGL(val_finish, dim3(pb), dim3(256), 0, stream, first_key, first_pair, P);
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
