// Host-side helpers shared by the entry points: argument checks, workspace carving,
// cached device properties.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "../../include/stalloc.h"

namespace stalloc {

constexpr size_t kAlign = 256;

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

struct DeviceInfo {
    int device = -1;
    int cus = 0;
    size_t lds_per_block = 0;   // largest LDS allocation one workgroup may use
};

// Properties of the current device (queried once per device; callable from several host threads).
inline bool device_info(DeviceInfo* out)
{
    static DeviceInfo cache[64];
    static std::mutex guard;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(guard);
    DeviceInfo& c = cache[dev];
    if (c.device != dev) {
        int cus = 0, lds = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return false;
        c.cus = cus;
        c.lds_per_block = (size_t)lds;
        c.device = dev;
    }
    *out = c;
    return true;
}

inline bool trace_args_ok(const stalloc_trace* tr)
{
    return tr && tr->n >= 1 && tr->n < 0x80000000u && tr->t_end >= 1 && tr->t_end < 0x80000000u &&
           tr->size && tr->t_alloc && tr->t_free;
}

// Carves 256-byte aligned pieces out of a caller-provided workspace.
struct Carver {
    unsigned char* base;
    size_t used = 0;
    explicit Carver(void* p) : base(static_cast<unsigned char*>(p)) {}
    template <typename T>
    T* take(size_t count)
    {
        T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
        used += align_up(count * sizeof(T));
        return p;
    }
};

// Shared device-side trace check (defined in trace_check.hip).
// acc: device uint64_t[kAccWords] scratch {sum of high halves, sum of low halves, flags,
// OR of all sizes, mode, largest size, sum of sizes in granules}.  mode = log2(address granule)
// | kModeNarrow when 32-bit granule counts can hold every address | kModeCompact when 16-bit
// counts can | kModeBitmap when the sizes suit one-bit-per-granule occupancy bitmaps | kModeTry32
// when only plans that stack nearly everything would overflow 32-bit counts.
constexpr int kAccWords = 16;
constexpr int kAccMode = 4;
constexpr int kAccMaxSize = 5;
constexpr int kAccGranules = 6;                // sum of sizes in granules
constexpr int kAccSplit = 7;                   // bit 0: the kernel that keeps only long-lived blocks in its list places the
                                               // trace; bits 8..31: its lifetime threshold; bits 32..63: long-lived requests
constexpr int kAccKernel = 8;                  // which placement kernel took the trace (stalloc_plan_kernel in stalloc.h)
constexpr int kAccWidePlans = 9;               // plans that outgrew 32-bit granule counts and were placed with 64-bit addresses
constexpr int kAccLargeShort = 10;             // long-list kernel: size (granules) from which a short-lived block counts as large
                                               // (0xffffffff: none does); bits 32..63: how many do
constexpr uint64_t kModeNarrow = 1ull << 8;
constexpr uint64_t kModeCompact = 1ull << 9;   // sum of sizes in granules below 2^16 as well
constexpr uint64_t kModeBitmap = 1ull << 10;   // sum <= kBitmapGranules and every size <= kBitmapMaxSize granules
constexpr uint64_t kModeTry32 = 1ull << 11;    // not narrow, but every size < 2^30 granules: 32-bit counts are tried plan by plan
constexpr uint32_t kBitmapGranules = 1u << 21; // a placed block's address has 22 bits in the kernel's table
constexpr uint32_t kBitmapMaxSize = 31;        // a block touches at most two bitmap words, its size fits 5 bits
void launch_trace_check(const stalloc_trace& tr, uint64_t* acc, uint32_t* device_status, hipStream_t stream);

// Exclusive sums of in[0..m) into out (defined in layers.hip): three launches; chunk_sum needs
// (m + 1023) / 1024 words; total[0] receives the sum of all; nothing happens unless *status is OK.
void launch_scan(const uint32_t* in, uint32_t m, uint32_t* out, uint32_t* chunk_sum, uint32_t* total,
                 const uint32_t* status, hipStream_t stream);

// Rows of n_pad two-word keys (n_pad a multiple of 256, all keys of a row distinct, compared word
// by word), every tile of 256 already sorted: merges the tiles of each row (defined in orders.hip),
// one launch per doubling of the run length, `keys` and `spare` in turn; returns the one that
// holds the sorted rows.
ulonglong2* launch_merge_tiles(ulonglong2* keys, ulonglong2* spare, uint32_t n_pad, uint32_t rows, const uint32_t* status,
                               hipStream_t stream);

}  // namespace stalloc
