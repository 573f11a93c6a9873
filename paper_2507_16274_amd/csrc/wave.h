// Wave64 building blocks for gfx950: DPP scans / reductions on 64-bit unsigned values.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stalloc {

constexpr int kWave = 64;

__device__ __forceinline__ uint64_t umax64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

// DPP controls (GFX9 encoding)
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143, kDppWaveShr1 = 0x138;
constexpr int kDppRowRor1 = 0x121, kDppRowRor2 = 0x122, kDppRowRor4 = 0x124, kDppRowRor8 = 0x128;

// Lanes whose DPP source does not exist, or whose row is masked out, receive `fill`.
template <int kCtrl, int kRowMask = 0xf>
__device__ __forceinline__ uint64_t dpp64(uint64_t fill, uint64_t v)
{
    uint32_t lo = __builtin_amdgcn_update_dpp((uint32_t)fill, (uint32_t)v, kCtrl, kRowMask, 0xf, false);
    uint32_t hi = __builtin_amdgcn_update_dpp((uint32_t)(fill >> 32), (uint32_t)(v >> 32), kCtrl, kRowMask, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t readlane64(uint64_t v, int lane)
{
    uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, lane);
    uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// Inclusive running maximum over the 64 lanes of a wave (all lanes must be active).
__device__ __forceinline__ uint64_t wave_scan_max64(uint64_t v)
{
    v = umax64(v, dpp64<kDppRowShr1>(0, v));
    v = umax64(v, dpp64<kDppRowShr2>(0, v));
    v = umax64(v, dpp64<kDppRowShr4>(0, v));
    v = umax64(v, dpp64<kDppRowShr8>(0, v));
    v = umax64(v, dpp64<kDppRowBcast15, 0xa>(0, v));
    v = umax64(v, dpp64<kDppRowBcast31, 0xc>(0, v));
    return v;
}

// Value of the previous lane; lane 0 receives `fill`.
__device__ __forceinline__ uint64_t wave_shift_up64(uint64_t v, uint64_t fill)
{
    return dpp64<kDppWaveShr1>(fill, v);
}

__device__ __forceinline__ uint64_t wave_max64(uint64_t v) { return readlane64(wave_scan_max64(v), 63); }

// 32-bit helpers ------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_sum32(uint32_t v)
{
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr2, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr4, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr8, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowBcast15, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowBcast31, 0xc, 0xf, false);
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v)
{
    v += dpp64<kDppRowShr1>(0, v);
    v += dpp64<kDppRowShr2>(0, v);
    v += dpp64<kDppRowShr4>(0, v);
    v += dpp64<kDppRowShr8>(0, v);
    v += dpp64<kDppRowBcast15, 0xa>(0, v);
    v += dpp64<kDppRowBcast31, 0xc>(0, v);
    return readlane64(v, 63);
}

__device__ __forceinline__ uint64_t wave_or64(uint64_t v)
{
    v |= dpp64<kDppRowShr1>(0, v);
    v |= dpp64<kDppRowShr2>(0, v);
    v |= dpp64<kDppRowShr4>(0, v);
    v |= dpp64<kDppRowShr8>(0, v);
    v |= dpp64<kDppRowBcast15, 0xa>(0, v);
    v |= dpp64<kDppRowBcast31, 0xc>(0, v);
    return readlane64(v, 63);
}

__device__ __forceinline__ uint64_t wave_min64(uint64_t v)
{
    const uint64_t top = ~0ull;
    v = umin64(v, dpp64<kDppRowShr1>(top, v));
    v = umin64(v, dpp64<kDppRowShr2>(top, v));
    v = umin64(v, dpp64<kDppRowShr4>(top, v));
    v = umin64(v, dpp64<kDppRowShr8>(top, v));
    v = umin64(v, dpp64<kDppRowBcast15, 0xa>(top, v));
    v = umin64(v, dpp64<kDppRowBcast31, 0xc>(top, v));
    return readlane64(v, 63);
}

// Width-generic wrappers used by the placement kernel (addresses are 32- or 64-bit) ----------
__device__ __forceinline__ uint32_t wave_scan_max(uint32_t v)
{
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr1, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr2, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr4, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr8, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowBcast15, 0xa, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowBcast31, 0xc, 0xf, false));
    return v;
}
__device__ __forceinline__ uint64_t wave_scan_max(uint64_t v) { return wave_scan_max64(v); }

// Running maximum inside each row of 16 lanes only.
__device__ __forceinline__ uint32_t row_scan_max(uint32_t v)
{
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr1, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr2, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr4, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowShr8, 0xf, 0xf, false));
    return v;
}
// Maximum over each row of 16 lanes, in all of its lanes (rotations inside the row).
__device__ __forceinline__ uint32_t row_max(uint32_t v)
{
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowRor1, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowRor2, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowRor4, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0u, v, kDppRowRor8, 0xf, 0xf, false));
    return v;
}
// The value of the lane before, inside each row of 16 lanes; `fill` in the row's first lane.
__device__ __forceinline__ uint32_t row_shift_up(uint32_t v, uint32_t fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, kDppRowShr1, 0xf, 0xf, false);
}
__device__ __forceinline__ uint64_t row_scan_max(uint64_t v)
{
    v = umax64(v, dpp64<kDppRowShr1>(0, v));
    v = umax64(v, dpp64<kDppRowShr2>(0, v));
    v = umax64(v, dpp64<kDppRowShr4>(0, v));
    v = umax64(v, dpp64<kDppRowShr8>(0, v));
    return v;
}

__device__ __forceinline__ uint32_t wave_shift_up(uint32_t v, uint32_t fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, kDppWaveShr1, 0xf, 0xf, false);
}
__device__ __forceinline__ uint64_t wave_shift_up(uint64_t v, uint64_t fill) { return wave_shift_up64(v, fill); }

__device__ __forceinline__ uint32_t read_lane(uint32_t v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ uint64_t read_lane(uint64_t v, int lane) { return readlane64(v, lane); }

// v with lane `lane` replaced by the (uniform) value.
__device__ __forceinline__ uint32_t write_lane(uint32_t v, uint32_t value, int lane)
{
    return (int)(threadIdx.x & (kWave - 1)) == lane ? value : v;
}
__device__ __forceinline__ uint64_t write_lane(uint64_t v, uint64_t value, int lane)
{
    return (int)(threadIdx.x & (kWave - 1)) == lane ? value : v;
}

// Value held by lane `src` (any lane index per lane; goes through the LDS crossbar).
__device__ __forceinline__ uint32_t lane_gather(uint32_t v, int src)
{
    return (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)v);
}
__device__ __forceinline__ uint64_t lane_gather(uint64_t v, int src)
{
    uint32_t lo = lane_gather((uint32_t)v, src), hi = lane_gather((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}

// Lane masks straight from a vector compare (one v_cmp, no per-lane boolean in between).
__device__ __forceinline__ uint64_t lanes_lt(uint32_t a, uint32_t b) { return __builtin_amdgcn_uicmp(a, b, 36); }
__device__ __forceinline__ uint64_t lanes_lt(uint64_t a, uint64_t b) { return __builtin_amdgcn_uicmpl(a, b, 36); }
__device__ __forceinline__ uint64_t lanes_ge(uint32_t a, uint32_t b) { return __builtin_amdgcn_uicmp(a, b, 35); }
__device__ __forceinline__ uint64_t lanes_ge(uint64_t a, uint64_t b) { return __builtin_amdgcn_uicmpl(a, b, 35); }

// Per lane: mask bit set ? v : 0.  The trailing wait states keep the result safe for a DPP
// consumer scheduled right behind the statement (the compiler does not track hazards of
// instructions inside an asm statement).
__device__ __forceinline__ uint32_t keep_lanes(uint64_t mask, uint32_t v)
{
    uint32_t r;
    asm("v_cndmask_b32_e64 %0, 0, %1, %2\n\ts_nop 1" : "=v"(r) : "v"(v), "s"(mask));
    return r;
}
// Four selections at once; one pair of wait states covers all of them.
__device__ __forceinline__ void keep_lanes4(const uint64_t (&mask)[4], uint32_t v, uint32_t (&out)[4])
{
    asm("v_cndmask_b32_e64 %0, 0, %4, %5\n\t"
        "v_cndmask_b32_e64 %1, 0, %4, %6\n\t"
        "v_cndmask_b32_e64 %2, 0, %4, %7\n\t"
        "v_cndmask_b32_e64 %3, 0, %4, %8\n\t"
        "s_nop 1"
        : "=&v"(out[0]), "=&v"(out[1]), "=&v"(out[2]), "=&v"(out[3])
        : "v"(v), "s"(mask[0]), "s"(mask[1]), "s"(mask[2]), "s"(mask[3]));
}
__device__ __forceinline__ void keep_lanes4(const uint64_t (&mask)[4], uint64_t v, uint64_t (&out)[4])
{
    for (int q = 0; q < 4; ++q) out[q] = ((uint64_t)keep_lanes(mask[q], (uint32_t)(v >> 32)) << 32) | keep_lanes(mask[q], (uint32_t)v);
}

__device__ __forceinline__ uint64_t keep_lanes(uint64_t mask, uint64_t v)
{
    return ((uint64_t)keep_lanes(mask, (uint32_t)(v >> 32)) << 32) | keep_lanes(mask, (uint32_t)v);
}

// Number of set bits of `mask` in lanes below the calling lane.
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint64_t umax(uint64_t a, uint64_t b) { return a > b ? a : b; }

// A value that is the same in all lanes of the wave (read by every lane from one LDS word, say),
// as a scalar: the compiler cannot know, and would otherwise branch on it with lane masks.
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Waits until every vector-memory access this wave has issued is complete.  Placed where that is
// the case anyway (long after the last one was issued), it tells the compiler so: without it, a load
// left unread on some path through a loop keeps its register marked as in flight, and the first
// write to that register -- in the middle of a run of loads meant to go out together -- is made to
// wait for all of them.
__device__ __forceinline__ void vector_memory_done() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0), nothing else

// A value loaded from memory is not looked at before this point: without it the compiler may move
// the first use (and with it the wait for the load) up to where the load was issued.
// (For a value that is the same in all lanes; it is handed on as a scalar.)
__device__ __forceinline__ void not_before_here(uint32_t& v)
{
    asm volatile("" : "+v"(v));
    v = __builtin_amdgcn_readfirstlane(v);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
// The wave's number within its workgroup, the same in all 64 lanes: taken from the first lane so that
// the compiler keeps it, and what is computed from it (loop bounds, shares of a list), in scalar
// registers and branches on it without lane masks.
__device__ __forceinline__ int wave_id() { return (int)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

}  // namespace stalloc
