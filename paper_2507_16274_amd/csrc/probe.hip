// stalloc_probe: three plain kernels that measure what the chip delivers, for the roofline
// figures reported beside the placement kernels: a device-memory copy, an LDS read loop and an
// integer ALU loop.  They only enqueue work; the caller times them with events.
#include "host_util.h"
#include "wave.h"

namespace stalloc {

constexpr int kProbeThreads = 1024;

// dst[i] = src[i] over 16-byte words, grid-stride.
__global__ void __launch_bounds__(256) probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t words)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Every thread reads 16 bytes of LDS `iters` times, lane after lane so that the 64 reads of a wave
// fall into all banks; the running XOR keeps the reads alive, one word per thread is written out.
__global__ void __launch_bounds__(kProbeThreads) probe_lds_read(uint32_t iters, uint32_t* out)
{
    __shared__ uint4 tile[4096];                                     // 64 KB
    for (uint32_t i = threadIdx.x; i < 4096; i += kProbeThreads) tile[i] = make_uint4(i, i * 3u, i * 5u, i * 7u);
    __syncthreads();
    uint4 acc = make_uint4(0, 0, 0, 0);
    uint32_t at = threadIdx.x;
    for (uint32_t k = 0; k < iters; k += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint4 v = tile[(at + 1024u * u) & 4095u];
            acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
        }
        at += 64u;
    }
    out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

// Eight independent chains of 32-bit integer operations per thread (add, max, xor, and in turn):
// 8 lane operations per inner step and thread.
__global__ void __launch_bounds__(256) probe_int_alu(uint32_t iters, uint32_t seed, uint32_t* out)
{
    uint32_t a0 = threadIdx.x + seed, a1 = a0 * 3u, a2 = a0 * 5u, a3 = a0 * 7u, a4 = a0 + 11u, a5 = a0 + 13u, a6 = a0 ^ 17u,
             a7 = a0 ^ 19u;
    for (uint32_t k = 0; k < iters; ++k) {
        a0 += a4; a1 = a1 > a5 ? a1 : a5; a2 ^= a6; a3 &= a7 | k;
        a4 += a1; a5 = a5 > a2 ? a5 : a2; a6 ^= a3; a7 += a0;
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = a0 ^ a1 ^ a2 ^ a3 ^ a4 ^ a5 ^ a6 ^ a7;
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_probe(uint32_t what, void* buffer, size_t buffer_bytes, uint32_t iters, uint64_t* work_done,
                             void* hip_stream)
{
    if (!buffer || !work_done || (reinterpret_cast<uintptr_t>(buffer) & 15)) return STALLOC_ERR_INVALID_ARG;
    DeviceInfo di;
    if (!device_info(&di)) return STALLOC_ERR_DEVICE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint32_t cus = (uint32_t)di.cus;
    if (what == STALLOC_PROBE_COPY) {
        const size_t words = buffer_bytes / 32;                      // first half -> second half
        if (words == 0) return STALLOC_ERR_INVALID_ARG;
        uint4* base = static_cast<uint4*>(buffer);
        hipLaunchKernelGGL(probe_copy, dim3(cus * 16), dim3(256), 0, stream, base, base + words, words);
        *work_done = (uint64_t)words * 32;                           // bytes read + bytes written
    } else if (what == STALLOC_PROBE_LDS_READ) {
        const uint32_t blocks = cus * 2;
        if (buffer_bytes < (size_t)blocks * kProbeThreads * 4 || iters == 0) return STALLOC_ERR_INVALID_ARG;
        const uint32_t rounds = (iters + 3) / 4 * 4;
        hipLaunchKernelGGL(probe_lds_read, dim3(blocks), dim3(kProbeThreads), 0, stream, rounds, static_cast<uint32_t*>(buffer));
        *work_done = (uint64_t)blocks * kProbeThreads * rounds * 16; // bytes read from LDS
    } else if (what == STALLOC_PROBE_INT_ALU) {
        const uint32_t blocks = cus * 32;
        if (buffer_bytes < (size_t)blocks * 256 * 4 || iters == 0) return STALLOC_ERR_INVALID_ARG;
        hipLaunchKernelGGL(probe_int_alu, dim3(blocks), dim3(256), 0, stream, iters, 7u, static_cast<uint32_t*>(buffer));
        *work_done = (uint64_t)blocks * 256 * iters * 8;             // lane operations
    } else {
        return STALLOC_ERR_INVALID_ARG;
    }
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
