// Two-word sort keys (compared word by word) and the in-LDS sort of one tile of 256 of them,
// shared by the kernels that order requests: placement orders, HomoSize groups, decisions by
// address.  The tiles are merged by launch_merge_tiles (host_util.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stalloc {

constexpr int kSortTile = 256;

__device__ __forceinline__ bool key_before(const ulonglong2& x, const ulonglong2& y)
{
    return x.x < y.x || (x.x == y.x && x.y < y.y);
}

// The key of slot e past the end of a row: behind every real key as long as no real key starts
// with ~0 and carries all ones in the upper half of its second word; distinct from slot to slot.
__device__ __forceinline__ ulonglong2 filler_key(uint32_t e) { return make_ulonglong2(~0ull, 0xffffffff00000000ull | e); }

// Bitonic network over k[0..255] in LDS; called by all 256 threads of the workgroup with their
// own key already stored at k[threadIdx.x]; sorted when it returns.
__device__ __forceinline__ void sort_tile(ulonglong2 (&k)[kSortTile])
{
    const uint32_t t = threadIdx.x;
    for (uint32_t span = 2; span <= (uint32_t)kSortTile; span <<= 1) {
        for (uint32_t gap = span >> 1; gap > 0; gap >>= 1) {
            __syncthreads();
            const uint32_t other = t ^ gap;
            if (other > t) {
                const ulonglong2 x = k[t], y = k[other];
                const bool ascending = (t & span) == 0;
                if (key_before(y, x) == ascending) { k[t] = y; k[other] = x; }
            }
        }
    }
    __syncthreads();
}

}  // namespace stalloc
