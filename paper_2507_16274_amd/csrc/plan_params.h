// Arguments shared by the placement kernels of stalloc_plan (sorted-list and occupancy-bitmap
// variants), and the launcher of the bitmap variant.
#pragma once

#include "host_util.h"

namespace stalloc {

struct PlanParams {
    const uint64_t* size;
    const uint32_t* ta;
    const uint32_t* tf;
    const uint32_t* orders;
    uint64_t* offsets;       // [P][n] or nullptr
    uint64_t* peaks;         // [P]
    uint32_t* status;
    const uint64_t* acc;     // trace-check accumulators (mode word)
    unsigned char* slabs;    // list in the workspace: gridDim.x slabs of 2 * n entries
    uint32_t* nbr_begin;     // bitmap variant: [n + 2] row starts of the lifetime-conflict index (+ a cursor)
    uint16_t* nbr;           // bitmap variant: 4 * (index of a request with an overlapping lifetime)
    uint32_t n;
    uint32_t P;
    uint32_t compact_enqueued;   // the compact 32-bit instantiation is part of this call
    uint32_t bitmap_enqueued;    // the occupancy-bitmap kernel is part of this call
    uint32_t bitmap_pool_words;  // bitmap variant: LDS words the bitmaps of a batch are carved from
};

// True when the kernels of the bitmap variant were enqueued for this call: they do the work
// (and the sorted-list kernels return at once) when the trace's mode word has kModeBitmap.
bool bitmap_plan_possible(uint32_t n, const DeviceInfo& di);
size_t bitmap_index_entries(uint32_t n);             // uint16_t entries of PlanParams::nbr
bool launch_plan_bitmap(const PlanParams& prm, const DeviceInfo& di, hipStream_t stream);

}  // namespace stalloc
