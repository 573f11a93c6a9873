// stalloc_memory_layers: memory-layer construction for the HomoSize groups of a trace
// (Sec. 5.1, HomoSize Group Planning, Algorithm 1), and stalloc_expand_layers.
//
// A HomoSize group holds the requests of one size; requests of a group whose lifetimes do not
// overlap share one range of that size, a memory-layer.  The group's requests are taken by
// allocation time; each goes to the free layer whose last request ended latest (lifetimes are
// half-open: a layer released at t is free at t), the one opened first among equals; if none is
// free a new layer is opened.  Layers are numbered group by group in descending size, inside
// a group in the order in which they were opened.
//
//   sort     Requests are sorted by (size descending, allocation time, request number): tiles
//            of 256 keys sorted in LDS (bitonic network), merged in log2(n / 256) passes (an
//            element's place is its place in its own run plus the number of elements of the
//            partner run that sort before it, found by binary search).
//   groups   A group starts where the size changes in the sorted sequence; exclusive sums of
//            the start flags number the groups.
//   build    One wave per group walks its requests in order -- the construction is
//            sequential by nature, the groups are what runs in parallel.  The ends of the
//            first 1024 layers of the group live in registers (lane = layer mod 64); finding
//            the free layer with the latest end is a 32-bit wave maximum (DPP) and a ballot,
//            in code chosen once per 64 requests for the registers they can come to use.
//            Further layers, if a group ever needs them, are kept in memory.
//   number   Exclusive sums of the groups' layer counts give every group its first layer.
//   emit     layer_of per request; size, first allocation and last release per layer.
#include "host_util.h"
#include "sort_keys.h"
#include "wave.h"

namespace stalloc {

constexpr int kLyTile = kSortTile;
constexpr int kLyRegs = 16;                      // 64 layers per register: 1024 layers of a group in registers
static_assert(kLyRegs == 16, "ly_build dispatches on one to sixteen registers in use");

__global__ void ly_init(uint32_t* v, uint32_t n)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) v[i] = 0;
}

// One tile of 256 requests per workgroup, sorted in LDS; slot e past the end holds a key behind
// every real one, (~0, ~0 << 32 | e) (sizes are > 0, so no real key starts with ~0).
__global__ void __launch_bounds__(kLyTile)
ly_sort_tiles(const uint64_t* __restrict__ size, const uint32_t* __restrict__ ta, uint32_t n, ulonglong2* keys,
              const uint32_t* status)
{
    __shared__ ulonglong2 k[kLyTile];
    if (*status != STALLOC_OK) return;
    const uint32_t t = threadIdx.x, i = blockIdx.x * kLyTile + t;
    // (size descending, allocation time, request number) as two ascending 64-bit words
    k[t] = i < n ? make_ulonglong2(~size[i], ((uint64_t)ta[i] << 32) | i) : filler_key(i);
    sort_tile(k);
    keys[blockIdx.x * kLyTile + t] = k[t];
}

// sorted[k] = request at sorted position k
__global__ void __launch_bounds__(256)
ly_ids(const ulonglong2* __restrict__ keys, uint32_t n, uint32_t* sorted, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x) {
        const uint32_t i = (uint32_t)keys[k].y;
        sorted[k] = i < n ? i : 0u;                           // (the first n sorted keys are the real ones)
    }
}

__global__ void __launch_bounds__(256)
ly_flags(const uint64_t* __restrict__ size, const uint32_t* __restrict__ sorted, uint32_t n, uint32_t* flag,
         const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x)
        flag[k] = (k == 0 || size[sorted[k]] != size[sorted[k - 1]]) ? 1u : 0u;
}

// Exclusive sums of m 32-bit values in three launches: sums of 1024-value chunks, their
// exclusive sums (one workgroup), and the values' own.  total[0] receives the sum of all.
constexpr int kScanChunk = 1024;

__global__ void __launch_bounds__(256)
scan_chunk_sums(const uint32_t* __restrict__ in, uint32_t m, uint32_t* chunk_sum, const uint32_t* status)
{
    __shared__ uint32_t part[4];
    if (*status != STALLOC_OK) return;
    const uint32_t base = blockIdx.x * kScanChunk;
    uint32_t s = 0;
    for (uint32_t j = threadIdx.x; j < (uint32_t)kScanChunk; j += 256)
        if (base + j < m) s += in[base + j];
    s = wave_sum32(s);
    if (lane_id() == 0) part[wave_id()] = s;
    __syncthreads();
    if (threadIdx.x == 0) chunk_sum[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

__global__ void __launch_bounds__(256)
scan_of_chunk_sums(uint32_t* chunk_sum, uint32_t chunks, uint32_t* total, const uint32_t* status)
{
    __shared__ uint32_t part[4];
    __shared__ uint32_t carry;
    if (*status != STALLOC_OK) return;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (uint32_t c0 = 0; c0 < chunks; c0 += 256) {
        const uint32_t c = c0 + threadIdx.x;
        const uint32_t v = c < chunks ? chunk_sum[c] : 0u;
        // inclusive sums inside the wave, then across the four waves
        uint32_t incl = v;
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr1, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr2, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr4, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr8, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowBcast15, 0xa, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowBcast31, 0xc, 0xf, false);
        if (lane_id() == kWave - 1) part[wave_id()] = incl;
        __syncthreads();
        uint32_t before_wave = carry;
        for (int w = 0; w < wave_id(); ++w) before_wave += part[w];
        if (c < chunks) chunk_sum[c] = before_wave + incl - v;
        __syncthreads();
        if (threadIdx.x == 0) carry += part[0] + part[1] + part[2] + part[3];
        __syncthreads();
    }
    if (threadIdx.x == 0) *total = carry;
}

__global__ void __launch_bounds__(256)
scan_apply(const uint32_t* __restrict__ in, uint32_t m, const uint32_t* __restrict__ chunk_sum, uint32_t* out,
           const uint32_t* status)
{
    __shared__ uint32_t part[4];
    if (*status != STALLOC_OK) return;
    const uint32_t base = blockIdx.x * kScanChunk;
    uint32_t run = chunk_sum[blockIdx.x];
    for (uint32_t j0 = 0; j0 < (uint32_t)kScanChunk; j0 += 256) {                 // (uniform trip count)
        const uint32_t j = base + j0 + threadIdx.x;
        const uint32_t v = j < m ? in[j] : 0u;
        uint32_t incl = v;
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr1, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr2, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr4, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowShr8, 0xf, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowBcast15, 0xa, 0xf, false);
        incl += __builtin_amdgcn_update_dpp(0u, incl, kDppRowBcast31, 0xc, 0xf, false);
        __syncthreads();                                                        // (part[] of the previous round consumed)
        if (lane_id() == kWave - 1) part[wave_id()] = incl;
        __syncthreads();
        uint32_t before_wave = run;
        for (int w = 0; w < wave_id(); ++w) before_wave += part[w];
        if (j < m) out[j] = before_wave + incl - v;
        run += part[0] + part[1] + part[2] + part[3];
    }
}

// group_start[g] = sorted position at which group g starts (g = number of flags before k).
__global__ void __launch_bounds__(256)
ly_group_starts(const uint32_t* __restrict__ flag, const uint32_t* __restrict__ flags_before, uint32_t n,
                uint32_t* group_start, const uint32_t* status)
{
    if (*status != STALLOC_OK) return;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x)
        if (flag[k]) group_start[flags_before[k]] = k;
}

struct LyBuild {
    const uint32_t* ta;
    const uint32_t* tf;
    const uint32_t* sorted;          // [n] request numbers by (size descending, allocation time, number)
    const uint32_t* group_start;     // [groups]
    const uint32_t* n_groups;        // [1]
    uint32_t* local;                 // [n] by sorted position: the request's layer inside its group
    uint32_t* first_ts;              // [n] slot group_start + l: allocation time of layer l's first request
    uint32_t* ends;                  // [n] slot group_start + l: free time of layer l's last request
    uint32_t* group_layers;          // [groups] layers of the group
    const uint32_t* status;
    uint32_t n;
};

// Groups with at most this many registers of layers are tested for being idle: the groups of small
// transient tensors, a few layers each, are idle between most of their requests; those with hundreds
// of layers hardly ever (and the number of registers in use only grows, so once a group is past
// the limit the record below is no longer needed).
constexpr int kLyIdleRegs = 2;

// The group's layer that was released last (the lowest-numbered of several released together): when a
// request starts at or after that release, every layer of the group is free and this is the one it
// takes -- no search.  Kept up to date as requests are appended to layers.
struct LastReleased {
    uint32_t end, layer;             // (uniform)
    __device__ __forceinline__ void appended(uint32_t te, uint32_t to_layer)
    {
        if (te > end) { end = te; layer = to_layer; }
        else if (te == end && to_layer < layer) layer = to_layer;
    }
};

// One request of a group whose layers all sit in the first kRegs registers (a layer it opens
// included): returns its layer and makes the request the layer's last one.  `layers` is uniform.
template <int kRegs>
__device__ __forceinline__ uint32_t take_layer(uint32_t (&end_of)[kLyRegs], uint32_t ts, uint32_t te, uint32_t layers,
                                               const LastReleased& last)
{
    const uint32_t lane = (uint32_t)lane_id();
    uint32_t layer = layers;                                              // a new one unless a free layer is found
    if (kRegs <= kLyIdleRegs && layers != 0 && ts >= last.end) {
        layer = last.layer;                                               // the whole group is idle
    } else {
        // latest end among the free layers (an end is a free time, hence >= 1; 0 = not opened)
        uint32_t latest = 0;
#pragma unroll
        for (int r = 0; r < kRegs; ++r) latest = umax(latest, end_of[r] <= ts ? end_of[r] : 0u);
        const uint32_t best = __builtin_amdgcn_readlane(wave_scan_max(latest), kWave - 1);
        if (best != 0) {
            bool found = false;
#pragma unroll
            for (int r = 0; r < kRegs; ++r) {
                const uint64_t hit = __builtin_amdgcn_ballot_w64(end_of[r] == best);
                if (!found && hit) { layer = (uint32_t)r * kWave + (uint32_t)__builtin_ctzll(hit); found = true; }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kRegs; ++r) end_of[r] = ((uint32_t)r == layer / kWave && lane == layer % kWave) ? te : end_of[r];
    return layer;
}

// The (up to 64) requests a wave has loaded, lane q holding request q, taken one by one while all
// layers the group can have by the end of the block sit in the first kRegs registers.  Returns the
// layer of the request this lane loaded; `layers` and `last` are kept up to date.
template <int kRegs>
__device__ __forceinline__ uint32_t take_block(uint32_t (&end_of)[kLyRegs], uint32_t ts_k, uint32_t te_k, int members,
                                               uint32_t& layers, LastReleased& last, uint32_t* first_ts)
{
    const int lane = lane_id();
    uint32_t mine = 0;
    uint32_t opened = layers;                                             // (uniform)
    LastReleased lr = last;
    for (int q = 0; q < members; ++q) {
        const uint32_t ts = __builtin_amdgcn_readlane(ts_k, q), te = __builtin_amdgcn_readlane(te_k, q);
        const uint32_t layer = take_layer<kRegs>(end_of, ts, te, opened, lr);
        if (layer == opened) {
            if (lane == 0) first_ts[opened] = ts;
            ++opened;
        }
        if (kRegs <= kLyIdleRegs) lr.appended(te, layer);
        if (lane == q) mine = layer;
    }
    layers = opened;
    last = lr;
    return mine;
}

__global__ void __launch_bounds__(256) ly_build(LyBuild g)
{
    if (*g.status != STALLOC_OK) return;
    const int lane = lane_id();
    const uint32_t groups = *g.n_groups;
    // (the wave's number, the same in all its lanes, as a scalar: the loops below then run on scalar
    // counters and branches instead of lane masks)
    const uint32_t first_group = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (uint32_t)wave_id());
    for (uint32_t grp = first_group; grp < groups; grp += gridDim.x * 4) {
        const uint32_t s = g.group_start[grp];
        const uint32_t e = grp + 1 < groups ? g.group_start[grp + 1] : g.n;
        uint32_t end_of[kLyRegs];        // lane holds the ends of layers lane, 64 + lane, ...; 0 = not opened
#pragma unroll
        for (int r = 0; r < kLyRegs; ++r) end_of[r] = 0;
        uint32_t layers = 0;             // (uniform) layers opened so far
        LastReleased last = {0, 0};
        uint32_t regs = 0;               // (uniform) registers of end_of in use
        // the lifetimes of the next 64 requests are on their way while these 64 are taken one by one
        uint32_t ts_next = 0, te_next = 0;
        if (s + lane < e) {
            const uint32_t i = g.sorted[s + lane];
            ts_next = g.ta[i];
            te_next = g.tf[i];
        }
        for (uint32_t base = s; base < e; base += kWave) {
            const uint32_t k = base + lane;
            const uint32_t ts_k = ts_next, te_k = te_next;
            if (k + kWave < e) {
                const uint32_t i = g.sorted[k + kWave];
                ts_next = g.ta[i];
                te_next = g.tf[i];
            }
            uint32_t mine = 0;           // layer of the request this lane loaded
            const int members = e - base < (uint32_t)kWave ? (int)(e - base) : kWave;
            layers = __builtin_amdgcn_readfirstlane(layers);
            // registers that hold every layer the group can have once these requests are placed (never
            // fewer than for an earlier block, a short last one included: see kLyIdleRegs)
            regs = umax(regs, (layers + (uint32_t)members + kWave - 1) / kWave);
            if (regs <= (uint32_t)kLyRegs) {
                // the usual case: everything in registers, code specialised for the registers in use
                uint32_t* const first_ts = g.first_ts + s;
                switch (regs) {
                    case 1: mine = take_block<1>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 2: mine = take_block<2>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 3: mine = take_block<3>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 4: mine = take_block<4>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 5: mine = take_block<5>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 6: mine = take_block<6>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 7: mine = take_block<7>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 8: mine = take_block<8>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 9: mine = take_block<9>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 10: mine = take_block<10>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 11: mine = take_block<11>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 12: mine = take_block<12>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 13: mine = take_block<13>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 14: mine = take_block<14>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    case 15: mine = take_block<15>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                    default: mine = take_block<16>(end_of, ts_k, te_k, members, layers, last, first_ts); break;
                }
                if (k < e) g.local[k] = mine;
                continue;
            }
            // a group that may pass 1024 layers: the further ones are kept in memory
            for (int q = 0; q < members; ++q) {
                const uint32_t ts = __builtin_amdgcn_readlane(ts_k, q), te = __builtin_amdgcn_readlane(te_k, q);
                layers = __builtin_amdgcn_readfirstlane(layers);
                uint32_t latest = 0;
#pragma unroll
                for (int r = 0; r < kLyRegs; ++r)
                    if ((uint32_t)r * kWave < layers) latest = umax(latest, end_of[r] <= ts ? end_of[r] : 0u);   // (uniform)
                const uint32_t in_regs = __builtin_amdgcn_readlane(wave_scan_max(latest), kWave - 1);
                uint32_t in_mem = 0;
                for (uint32_t l0 = kLyRegs * kWave; l0 < layers; l0 += kWave) {
                    const uint32_t l = l0 + lane;
                    const uint32_t v = l < layers ? __hip_atomic_load(&g.ends[s + l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
                    in_mem = umax(in_mem, __builtin_amdgcn_readlane(wave_scan_max(v <= ts ? v : 0u), kWave - 1));
                }
                const uint32_t best = umax(in_regs, in_mem);
                uint32_t layer = layers;                                          // a new one unless a free layer is found
                if (best != 0) {
                    bool found = false;
                    if (in_regs == best) {
#pragma unroll
                        for (int r = 0; r < kLyRegs; ++r) {
                            if (found || (uint32_t)r * kWave >= layers) continue;                      // (uniform)
                            const uint64_t hit = __builtin_amdgcn_ballot_w64(end_of[r] == best);
                            if (hit) { layer = (uint32_t)r * kWave + (uint32_t)__builtin_ctzll(hit); found = true; }
                        }
                    }
                    for (uint32_t l0 = kLyRegs * kWave; !found && l0 < layers; l0 += kWave) {
                        const uint32_t l = l0 + lane;
                        const uint32_t v = l < layers ? __hip_atomic_load(&g.ends[s + l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
                        const uint64_t hit = __builtin_amdgcn_ballot_w64(v == best);
                        if (hit) { layer = l0 + (uint32_t)__builtin_ctzll(hit); found = true; }
                    }
                } else {
                    if (lane == 0) g.first_ts[s + layers] = ts;
                    ++layers;
                }
                // the request becomes the layer's last one
                if (layer < (uint32_t)(kLyRegs * kWave)) {
#pragma unroll
                    for (int r = 0; r < kLyRegs; ++r)
                        if ((uint32_t)r == layer / kWave) end_of[r] = (uint32_t)lane == layer % kWave ? te : end_of[r];   // (uniform test)
                } else if (lane == 0) {
                    __hip_atomic_store(&g.ends[s + layer], te, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (lane == q) mine = layer;
            }
            if (k < e) g.local[k] = mine;
        }
#pragma unroll
        for (int r = 0; r < kLyRegs; ++r) {
            const uint32_t l = (uint32_t)r * kWave + lane;
            if (l < layers) g.ends[s + l] = end_of[r];
        }
        if (lane == 0) g.group_layers[grp] = layers;
    }
}

struct LyEmit {
    const uint64_t* size;
    const uint32_t* sorted;
    const uint32_t* flag;            // [n] 1 where a group starts
    const uint32_t* flags_before;    // [n] exclusive sums of flag
    const uint32_t* group_start;
    const uint32_t* group_layers;
    const uint32_t* group_base;      // [groups] exclusive sums of group_layers
    const uint32_t* local;
    const uint32_t* first_ts;
    const uint32_t* ends;
    uint32_t* layer_of;
    uint64_t* layer_size;
    uint32_t* layer_ta;
    uint32_t* layer_tf;
    const uint32_t* status;
    uint32_t n;
};

__global__ void __launch_bounds__(256) ly_emit(LyEmit g)
{
    if (*g.status != STALLOC_OK) return;
    for (uint32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < g.n; k += gridDim.x * blockDim.x) {
        const uint32_t i = g.sorted[k];
        const uint32_t grp = g.flags_before[k] + g.flag[k] - 1;
        const uint32_t s = g.group_start[grp], base = g.group_base[grp];
        g.layer_of[i] = base + g.local[k];
        const uint32_t l = k - s;                    // slot of the group: a layer if the group has that many
        if (l < g.group_layers[grp]) {
            g.layer_size[base + l] = g.size[i];
            g.layer_ta[base + l] = g.first_ts[k];
            g.layer_tf[base + l] = g.ends[k];
        }
    }
}

__global__ void ly_expand_init(uint32_t* status)
{
    if (threadIdx.x == 0) *status = STALLOC_OK;
}

// offsets[p][i] = layer_offsets[p][layer_of[i]]; a layer number that does not exist is reported.
__global__ void __launch_bounds__(256)
ly_expand(const uint32_t* __restrict__ layer_of, const uint64_t* __restrict__ layer_offsets, uint32_t n_layers,
          uint32_t n, uint64_t* offsets, uint32_t* status)
{
    const uint64_t* row = layer_offsets + (size_t)blockIdx.y * n_layers;
    uint64_t* out = offsets + (size_t)blockIdx.y * n;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint32_t l = layer_of[i];
        if (l < n_layers) out[i] = row[l];
        else atomicMax(status, (uint32_t)STALLOC_ERR_BAD_LAYER);
    }
}

// Exclusive sums of in[0..m) into out; total[0] = sum.  chunk_sum: (m + 1023) / 1024 words.
void launch_scan(const uint32_t* in, uint32_t m, uint32_t* out, uint32_t* chunk_sum, uint32_t* total,
                 const uint32_t* status, hipStream_t stream)
{
    const uint32_t chunks = (m + kScanChunk - 1) / kScanChunk;
    hipLaunchKernelGGL(scan_chunk_sums, dim3(chunks), dim3(256), 0, stream, in, m, chunk_sum, status);
    hipLaunchKernelGGL(scan_of_chunk_sums, dim3(1), dim3(256), 0, stream, chunk_sum, chunks, total, status);
    hipLaunchKernelGGL(scan_apply, dim3(chunks), dim3(256), 0, stream, in, m, chunk_sum, out, status);
}

}  // namespace stalloc

using namespace stalloc;

extern "C" int stalloc_memory_layers(const stalloc_trace* tr, uint32_t* layer_of, uint32_t* n_layers,
                                     uint64_t* layer_size, uint32_t* layer_t_alloc, uint32_t* layer_t_free,
                                     uint32_t* device_status, void* workspace, size_t* workspace_bytes,
                                     void* hip_stream)
{
    if (!trace_args_ok(tr) || !workspace_bytes) return STALLOC_ERR_INVALID_ARG;
    DeviceInfo di;
    if (!device_info(&di)) return STALLOC_ERR_DEVICE;
    const uint32_t n = tr->n;
    const uint32_t tiles = (n + kLyTile - 1) / kLyTile;
    const uint32_t chunks = (n + kScanChunk - 1) / kScanChunk;

    Carver cv(workspace);
    uint64_t* acc = cv.take<uint64_t>(kAccWords);
    ulonglong2* keys = cv.take<ulonglong2>((size_t)tiles * kLyTile);
    ulonglong2* spare = cv.take<ulonglong2>((size_t)tiles * kLyTile);
    uint32_t* sorted = cv.take<uint32_t>(n);
    uint32_t* flag = cv.take<uint32_t>(n);
    uint32_t* flags_before = cv.take<uint32_t>(n);
    uint32_t* group_start = cv.take<uint32_t>(n);
    uint32_t* group_layers = cv.take<uint32_t>(n);
    uint32_t* group_base = cv.take<uint32_t>(n);
    uint32_t* local = cv.take<uint32_t>(n);
    uint32_t* first_ts = cv.take<uint32_t>(n);
    uint32_t* ends = cv.take<uint32_t>(n);
    uint32_t* chunk_sum = cv.take<uint32_t>(chunks);
    uint32_t* n_groups = cv.take<uint32_t>(1);
    if (!workspace) { *workspace_bytes = cv.used; return STALLOC_OK; }
    if (!layer_of || !n_layers || !layer_size || !layer_t_alloc || !layer_t_free || !device_status ||
        *workspace_bytes < cv.used || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)))
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    launch_trace_check(*tr, acc, device_status, stream);

    uint32_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(ly_sort_tiles, dim3(tiles), dim3(kLyTile), 0, stream, tr->size, tr->t_alloc, n, keys, device_status);
    const ulonglong2* by_key = launch_merge_tiles(keys, spare, tiles * kLyTile, 1, device_status, stream);
    hipLaunchKernelGGL(ly_ids, dim3(blocks), dim3(256), 0, stream, by_key, n, sorted, device_status);
    hipLaunchKernelGGL(ly_flags, dim3(blocks), dim3(256), 0, stream, tr->size, sorted, n, flag, device_status);
    launch_scan(flag, n, flags_before, chunk_sum, n_groups, device_status, stream);
    hipLaunchKernelGGL(ly_group_starts, dim3(blocks), dim3(256), 0, stream, flag, flags_before, n, group_start,
                       device_status);

    LyBuild b;
    b.ta = tr->t_alloc; b.tf = tr->t_free; b.sorted = sorted; b.group_start = group_start; b.n_groups = n_groups;
    b.local = local; b.first_ts = first_ts; b.ends = ends; b.group_layers = group_layers; b.status = device_status;
    b.n = n;
    // Only the device knows how many groups there are: the layer counts of all n slots are summed,
    // the slots past the last group hold none.
    hipLaunchKernelGGL(ly_init, dim3(blocks), dim3(256), 0, stream, group_layers, n);
    uint32_t build_blocks = (n + 3) / 4;                  // at most n groups, four waves to a workgroup
    if (build_blocks > (uint32_t)di.cus * 8) build_blocks = (uint32_t)di.cus * 8;
    hipLaunchKernelGGL(ly_build, dim3(build_blocks), dim3(256), 0, stream, b);
    launch_scan(group_layers, n, group_base, chunk_sum, n_layers, device_status, stream);

    LyEmit e;
    e.size = tr->size; e.sorted = sorted; e.flag = flag; e.flags_before = flags_before; e.group_start = group_start;
    e.group_layers = group_layers; e.group_base = group_base; e.local = local; e.first_ts = first_ts; e.ends = ends;
    e.layer_of = layer_of; e.layer_size = layer_size; e.layer_ta = layer_t_alloc; e.layer_tf = layer_t_free;
    e.status = device_status; e.n = n;
    hipLaunchKernelGGL(ly_emit, dim3(blocks), dim3(256), 0, stream, e);
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}

extern "C" int stalloc_expand_layers(uint32_t n, uint32_t P, const uint32_t* layer_of, const uint64_t* layer_offsets,
                                     uint32_t n_layers, uint64_t* offsets, uint32_t* device_status, void* hip_stream)
{
    if (n == 0 || n >= 0x80000000u || P == 0 || n_layers == 0 || !layer_of || !layer_offsets || !offsets || !device_status)
        return STALLOC_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t blocks = (n + 255) / 256;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(ly_expand_init, dim3(1), dim3(64), 0, stream, device_status);
    for (uint32_t p0 = 0; p0 < P; p0 += 32768) {           // grid.y is limited to 65535
        const uint32_t py = P - p0 < 32768 ? P - p0 : 32768;
        hipLaunchKernelGGL(ly_expand, dim3(blocks, py), dim3(256), 0, stream, layer_of, layer_offsets + (size_t)p0 * n_layers,
                           n_layers, n, offsets + (size_t)p0 * n, device_status);
    }
    return hipGetLastError() == hipSuccess ? STALLOC_OK : STALLOC_ERR_DEVICE;
}
