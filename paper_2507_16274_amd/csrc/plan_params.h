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
    uint32_t* wide_plans;    // [P] list variant: 1 = the plan outgrew 32-bit granule counts, the 64-bit kernel places it
    uint32_t* nbr_begin;     // bitmap variant: [n + 2] row starts of the lifetime-conflict index
    uint16_t* nbr;           // bitmap variant: indices of the requests with an overlapping lifetime, row by row
    uint32_t n;
    uint32_t P;
    uint32_t compact_enqueued;   // the compact 32-bit instantiation is part of this call
    // The occupancy-bitmap kernel is enqueued in up to two shapes: [0] eight waves per workgroup,
    // several workgroups per CU; [1] sixteen waves, one workgroup per CU (all of the LDS).  Per
    // shape: the LDS words its bitmaps are carved from, 0 = not part of this call.
    uint32_t bitmap_pool_words[2];
};

constexpr int kBitmapShapes = 2;
__host__ __device__ constexpr uint32_t bitmap_shape_waves(int shape) { return shape == 0 ? 8u : 16u; }

// Which shape of the bitmap kernel places a trace with this mode word and sum of sizes in
// granules (-1: none, the sorted-list kernels do).  Half of the pool (two batches are in
// flight) must be able to hold one bitmap of the whole address range plus one word per
// request of two batches and a little slack.  Every kernel of a call evaluates this same
// rule, so exactly one of them does the work.
__host__ __device__ inline int bitmap_shape(uint64_t mode, uint64_t granules, const uint32_t (&pool_words)[kBitmapShapes])
{
    if (!(mode & kModeBitmap)) return -1;
    for (int shape = 0; shape < kBitmapShapes; ++shape)
        if (pool_words[shape] != 0 && granules / 32 + 2 * bitmap_shape_waves(shape) + 5 <= pool_words[shape] / 2) return shape;
    return -1;
}

// The variant that keeps only long-lived blocks in its sorted list (plan_split.hip): pieces of
// the workspace, their sizes, and the launcher of its preparation and placement kernels.  The
// preparation decides on the device whether the variant places the trace (acc[kAccSplit]).
struct SplitWorkspace {
    uint32_t* hist;
    uint32_t* gate;
    ulonglong2* keys;
    ulonglong2* spare;
    uint4* by_rank;
    uint32_t* size_by_rank;
    uint32_t* rank_of;
    uint4* record;
    uint2* fit_by_rank;
    uint32_t* addr;
    uint2* group_span;
    uint32_t* is_large;
    uint32_t* large_before;
    uint32_t* scan_chunks;
    uint32_t* scan_total;
    uint2* large_fit;
    uint32_t* large_addr;
    uint32_t* allocated_at;      // list with ranks in place of times: marks per timestamp, their exclusive sums, size classes
    uint32_t* released_at;
    uint32_t* class_size;
    uint32_t* allocated_before;
    uint32_t* released_before;
    uint32_t slots, large_slots, n_pad, grid, times;
};
size_t split_workspace(uint32_t n, uint32_t t_end, const DeviceInfo& di, Carver& cv, SplitWorkspace* ws);
bool launch_plan_split(const PlanParams& prm, uint32_t t_end, const SplitWorkspace& ws, const DeviceInfo& di, hipStream_t stream);

// Fills PlanParams::bitmap_pool_words for a trace of n requests; false if no shape fits.
bool bitmap_plan_shapes(uint32_t n, const DeviceInfo& di, uint32_t (&pool_words)[kBitmapShapes]);
size_t bitmap_index_entries(uint32_t n);             // uint16_t entries of PlanParams::nbr
bool launch_plan_bitmap(const PlanParams& prm, const DeviceInfo& di, hipStream_t stream);

}  // namespace stalloc
