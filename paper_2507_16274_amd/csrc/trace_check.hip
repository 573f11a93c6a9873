// Device-side sanity pass over a trace: sizes > 0, t_alloc < t_free <= t_end, and the
// sum of sizes below 2^63 so that no address can wrap (requests are the events
// m = (s, t_s, t_e) of Sec. 4).  The verdict lands in the caller's device status word.
// The pass also derives the address granule: every address a plan can produce is a sum of
// request sizes, hence a multiple of the largest power of two dividing all sizes; when the
// sum of sizes counted in granules stays below 2^31 the placement kernel may keep
// addresses as 32-bit granule counts without any loss.
#include "host_util.h"
#include "wave.h"

namespace stalloc {

__global__ void trace_check_init(uint64_t* acc, uint32_t* status)
{
    if (threadIdx.x < kAccWords) acc[threadIdx.x] = 0;
    if (threadIdx.x == 0) *status = STALLOC_OK;
}

__global__ void __launch_bounds__(256)
trace_check_scan(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta,
                 const uint32_t* __restrict__ tf, uint32_t n, uint32_t t_end, uint64_t* acc)
{
    __shared__ uint64_t part[4][5];                  // per wave: hi, lo, bad, bits, largest
    uint64_t hi = 0, lo = 0, bits = 0, largest = 0;
    uint32_t bad = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        uint64_t s = size[i];
        uint32_t a = ta[i], f = tf[i];
        bad |= (s == 0) | (a >= f) | (f > t_end);
        hi += s >> 32;               // n < 2^31 terms below 2^32 each: cannot wrap
        lo += s & 0xffffffffull;
        bits |= s;
        largest = umax64(largest, s);
    }
    hi = wave_sum64(hi);
    lo = wave_sum64(lo);
    bits = wave_or64(bits);
    largest = wave_max64(largest);
    uint64_t any_bad = __builtin_amdgcn_ballot_w64(bad != 0);
    // one set of atomics per workgroup: thousands of waves on five words would queue up
    if (lane_id() == 0) {
        uint64_t* mine = part[wave_id()];
        mine[0] = hi; mine[1] = lo; mine[2] = any_bad ? 1 : 0; mine[3] = bits; mine[4] = largest;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) {
            hi += part[w][0]; lo += part[w][1]; any_bad |= part[w][2]; bits |= part[w][3];
            largest = umax64(largest, part[w][4]);
        }
        atomicAdd((unsigned long long*)&acc[0], (unsigned long long)hi);
        atomicAdd((unsigned long long*)&acc[1], (unsigned long long)lo);
        if (any_bad) atomicOr((unsigned long long*)&acc[2], 1ull);
        atomicOr((unsigned long long*)&acc[3], (unsigned long long)bits);
        atomicMax((unsigned long long*)&acc[kAccMaxSize], (unsigned long long)largest);
    }
}

__global__ void trace_check_finish(uint64_t* acc, uint32_t* status)
{
    if (threadIdx.x != 0) return;
    uint32_t code = STALLOC_OK;
    acc[kAccMode] = 0;
    if (acc[0] + (acc[1] >> 32) < (1ull << 31) && acc[3] != 0) {
        const uint64_t total = (acc[0] << 32) + acc[1];              // below 2^63 here
        const uint32_t shift = (uint32_t)__builtin_ctzll(acc[3]);
        const uint64_t narrow = (total >> shift) < (1ull << 31) ? kModeNarrow : 0;
        const uint64_t compact = (total >> shift) < (1ull << 16) ? kModeCompact : 0;
        const uint64_t bitmap = (total >> shift) <= kBitmapGranules && (acc[kAccMaxSize] >> shift) <= kBitmapMaxSize
                                    ? kModeBitmap : 0;
        // The sum of sizes bounds every address, but plans worth having end far below it: when the
        // sum is too large for 32-bit granule counts and no single request is, the 32-bit placement
        // kernel takes each plan as far as its extent allows and hands the rest to the 64-bit one.
        const uint64_t try32 = (!narrow && (acc[kAccMaxSize] >> shift) < (1ull << 30)) ? kModeTry32 : 0;
        acc[kAccMode] = shift | narrow | compact | bitmap | try32;
        acc[kAccGranules] = total >> shift;
    }
    // total = acc[0] * 2^32 + acc[1]  >= 2^63  <=>  acc[0] + (acc[1] >> 32) >= 2^31
    if (acc[0] + (acc[1] >> 32) >= (1ull << 31)) code = STALLOC_ERR_OVERFLOW;
    if (acc[2] & 1ull) code = STALLOC_ERR_BAD_TRACE;
    if (code != STALLOC_OK) atomicMax(status, code);
}

void launch_trace_check(const stalloc_trace& tr, uint64_t* acc, uint32_t* device_status, hipStream_t stream)
{
    hipLaunchKernelGGL(trace_check_init, dim3(1), dim3(64), 0, stream, acc, device_status);
    uint32_t blocks = (tr.n + 255) / 256;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(trace_check_scan, dim3(blocks), dim3(256), 0, stream, tr.size, tr.t_alloc, tr.t_free,
                       tr.n, tr.t_end, acc);
    hipLaunchKernelGGL(trace_check_finish, dim3(1), dim3(64), 0, stream, acc, device_status);
}

}  // namespace stalloc

extern "C" const char* stalloc_status_string(int status)
{
    switch (status) {
        case STALLOC_OK: return "STALLOC_OK";
        case STALLOC_ERR_INVALID_ARG: return "STALLOC_ERR_INVALID_ARG";
        case STALLOC_ERR_BAD_TRACE: return "STALLOC_ERR_BAD_TRACE";
        case STALLOC_ERR_OVERFLOW: return "STALLOC_ERR_OVERFLOW";
        case STALLOC_ERR_NOMEM: return "STALLOC_ERR_NOMEM";
        case STALLOC_ERR_DEVICE: return "STALLOC_ERR_DEVICE";
        case STALLOC_ERR_BAD_ORDER: return "STALLOC_ERR_BAD_ORDER";
        case STALLOC_ERR_BAD_WINDOW: return "STALLOC_ERR_BAD_WINDOW";
        case STALLOC_ERR_BAD_LAYER: return "STALLOC_ERR_BAD_LAYER";
        case STALLOC_ERR_TOO_LARGE: return "STALLOC_ERR_TOO_LARGE";
        default: return "STALLOC_UNKNOWN_STATUS";
    }
}
