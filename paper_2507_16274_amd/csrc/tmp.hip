// stalloc_tmp: the time-memory product of Eq. 2 for P plans of one trace, with the whole
// plan as the group D_g:
//
//     TMP = sum_i s_i (t_e,i - t_s,i)  /  ( extent * (max t_e - min t_s) ),   extent = max(a + s).
//
// The numerator and the span belong to the trace; the extent is what differs between plans
// (stalloc_plan returns it per plan).  A higher value means fewer spatio-temporal bubbles.
//
// The numerator is summed exactly: every product s * (t_e - t_s) has up to 96 bits and is cut
// into three 32-bit limbs, each limb summed in a 64-bit word (fewer than 2^31 terms: no
// wrap).  The limbs are combined in double precision and divided once per plan: at most eight
// roundings, a relative error below 10 * 2^-53.
#include "host_util.h"
#include "wave.h"

namespace stalloc {

struct TmpAcc {
    uint64_t limb[3];      // sums of bits 0-31, 32-63, 64-95 of the products
    uint32_t t_first;      // min t_alloc
    uint32_t t_last;       // max t_free
};

__global__ void tmp_init(TmpAcc* acc)
{
    if (threadIdx.x == 0) { acc->limb[0] = acc->limb[1] = acc->limb[2] = 0; acc->t_first = 0xffffffffu; acc->t_last = 0; }
}

__global__ void __launch_bounds__(256)
tmp_used(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, const uint32_t* __restrict__ tf, uint32_t n,
         TmpAcc* acc, const uint32_t* status)
{
    __shared__ uint64_t part[4][3];
    __shared__ uint32_t t_lo[4], t_hi[4];
    if (*status != STALLOC_OK) return;
    uint64_t l0 = 0, l1 = 0, l2 = 0;
    uint32_t first = 0xffffffffu, last = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint64_t s = size[i];
        const uint32_t a = ta[i], f = tf[i];
        const uint64_t life = f - a;
        const uint64_t low = (s & 0xffffffffull) * life;           // < 2^64
        const uint64_t high = (s >> 32) * life + (low >> 32);       // bits 32.. of the product; < 2^64
        l0 += low & 0xffffffffull;
        l1 += high & 0xffffffffull;
        l2 += high >> 32;
        first = a < first ? a : first;
        last = f > last ? f : last;
    }
    l0 = wave_sum64(l0); l1 = wave_sum64(l1); l2 = wave_sum64(l2);
    const uint32_t w_first = 0xffffffffu - (uint32_t)wave_max64(0xffffffffu - first), w_last = (uint32_t)wave_max64(last);
    if (lane_id() == 0) {
        part[wave_id()][0] = l0; part[wave_id()][1] = l1; part[wave_id()][2] = l2;
        t_lo[wave_id()] = w_first; t_hi[wave_id()] = w_last;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) {
            l0 += part[w][0]; l1 += part[w][1]; l2 += part[w][2];
        }
        uint32_t lo = t_lo[0], hi = t_hi[0];
        for (int w = 1; w < 4; ++w) { lo = t_lo[w] < lo ? t_lo[w] : lo; hi = t_hi[w] > hi ? t_hi[w] : hi; }
        atomicAdd((unsigned long long*)&acc->limb[0], (unsigned long long)l0);
        atomicAdd((unsigned long long*)&acc->limb[1], (unsigned long long)l1);
        atomicAdd((unsigned long long*)&acc->limb[2], (unsigned long long)l2);
        atomicMin(&acc->t_first, lo);
        atomicMax(&acc->t_last, hi);
    }
}

__global__ void __launch_bounds__(256)
tmp_per_plan(const TmpAcc* __restrict__ acc, const uint64_t* __restrict__ extents, uint32_t P, double* tmp,
             const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    const double used = ((double)acc->limb[2] * 4294967296.0 + (double)acc->limb[1]) * 4294967296.0 + (double)acc->limb[0];
    const double span = (double)(acc->t_last - acc->t_first);
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < P; p += gridDim.x * blockDim.x)
        tmp[p] = used / ((double)extents[p] * span);
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_tmp(const stalloc_trace* tr, const uint64_t* extents, uint32_t P, double* tmp,
                           uint32_t* device_status, void* workspace, size_t* workspace_bytes, void* hip_stream)
{
    if (!trace_args_ok(tr) || P == 0 || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    TmpAcc* sums = cv.take<TmpAcc>(1);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!extents || !tmp || !device_status || *workspace_bytes < cv.used ||
        (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    launch_trace_check(*tr, acc, device_status, stream);
    hipLaunchKernelGGL(tmp_init, dim3(1), dim3(64), 0, stream, sums);
    uint32_t blocks = (tr->n + 255) / 256;
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(tmp_used, dim3(blocks), dim3(256), 0, stream, tr->size, tr->t_alloc, tr->t_free, tr->n, sums,
                       device_status);
    uint32_t pb = (P + 255) / 256;
    if (pb > 1024) pb = 1024;
    hipLaunchKernelGGL(tmp_per_plan, dim3(pb), dim3(256), 0, stream, sums, extents, P, tmp, device_status);
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
