// stalloc_plan, occupancy-bitmap variant: the same rule as the sorted-list kernel (Sec. 5.1:
// requests in the given order, each at the lowest address where it conflicts with no earlier
// request of the plan in lifespan and address range at once; extent = max(a + s), Eq. 2), for
// traces whose requests are short when counted in granules.
//
// With g the largest power of two dividing all sizes, every address is a multiple of g and lies
// below the sum of sizes.  When no request is longer than 31 granules and a bitmap of one bit per
// granule of that whole range fits the LDS left over by the plan's table of placed blocks, "which
// addresses are blocked for request r" is such a bitmap, which a single wave searches in a few steps:
//
//   index    Once per call: for every request the list of requests whose lifetime overlaps its
//            own (the potential conflicts of Sec. 5.1 do not depend on the order), rows padded
//            to 256 entries with a dummy request that is never placed.
//   build    One workgroup per plan, K requests per batch, one bitmap per request.  The rows of
//            the K requests are cut into chunks of 256 entries which are dealt out to the waves,
//            so that every wave has the same amount of work whatever the row lengths.  A wave
//            looks every neighbour of its chunk up in the plan's table of placed blocks (LDS,
//            4 bytes per request: address and the two word masks in a compressed form, 0 = not
//            placed yet) and ORs the neighbour's granules into the bitmap of the request the
//            chunk belongs to (LDS atomics: any wave may add to any bitmap).
//   search   Wave r finds the first run of size_r zero bits in bitmap r: the lowest fit against
//            what the bitmap holds.
//   settle   Wave 0 takes the K requests in order.  A candidate stands unless a block the bitmap
//            may have missed -- one of the batch before, or one settled earlier in the same
//            batch -- overlaps it in lifetime and in address range; only then are those blocks
//            ORed into the request's bitmap and the search repeated.  Adding blocks can only
//            remove free runs, so an untouched candidate is still the lowest.
//
// Batches are software-pipelined over two halves of the bitmap pool: batch B is settled while
// batch B + 1 is built.  Nothing is sorted or merged and no placement needs a second pass.
#include "host_util.h"
#include "plan_params.h"
#include "wave.h"

namespace stalloc {

#ifndef STALLOC_BITMAP_REFILL
#define STALLOC_BITMAP_REFILL 16      // requests fetched per refill, per wave of the workgroup
#endif
#ifndef STALLOC_BITMAP_SHARES
#define STALLOC_BITMAP_SHARES 2
#endif
constexpr int kRefillPerWave = STALLOC_BITMAP_REFILL;   // (the pipeline of batches drains at every refill)
constexpr uint32_t kShares = STALLOC_BITMAP_SHARES; // chunks a building wave takes for every one wave 0 takes
constexpr int kBmWords = 1056;           // a pool of twice this many words is asked for before workgroups share a CU
constexpr int kRowPad = 256;             // index rows are padded to this many entries (4 per lane)

constexpr uint32_t kBmMaxRequests = 32768;         // index entries are 16-bit request numbers; the index has n^2 of them at worst

template <int kWaves>
struct BitmapLds {
    static constexpr int kBmBatch = kRefillPerWave * kWaves;     // 128 requests with eight waves, 256 with sixteen
    uint32_t rq_id[kBmBatch];
    uint32_t rq_s[kBmBatch];             // size in granules
    uint32_t rq_ta[kBmBatch];
    uint32_t rq_tf[kBmBatch];
    uint32_t rq_x[kBmBatch];             // address in granules
    uint32_t rq_row[kBmBatch];           // first chunk of the request's row of the index
    uint32_t rq_chunks[kBmBatch];        // chunks in that row
    uint32_t cand[kWaves];               // lowest fit of each request of the batch against what its bitmap holds
    uint32_t top;                        // extent so far, granules
    uint32_t pad[3];
};
// Behind it in LDS: the plan's table of placed blocks (n + 1 words) and the pool the bitmaps are
// carved from, one half per batch in flight.  A bitmap is only as long as the plan's extent
// needs, so a half holds a full batch of them as long as the extent is moderate, and fewer
// (smaller batches) beyond that; the rule that admits a trace makes sure it always holds one.

// ---------------------------------------------------------------------------------------------
// Lifetime-conflict index.  begin[i] .. begin[i + 1] are the 256-entry chunks of request i's row;
// an entry is j for a request j != i with t_alloc_j < t_free_i and t_alloc_i < t_free_j, or n (a
// dummy that is never placed) -- stored as 4 * j, the byte offset into the plan's table, while
// 4 * n fits 16 bits (the build phase then needs one instruction less per lookup).  begin[] first
// holds the degrees, then their exclusive prefix sum in chunks.
constexpr uint32_t kScaledEntriesBelow = 16384;      // n below this: entries are 4 * j
__host__ __device__ inline uint32_t entry_shift(uint32_t n) { return n < kScaledEntriesBelow ? 2u : 0u; }

__device__ __forceinline__ bool index_wanted(const PlanParams& prm)
{
    return *prm.status == STALLOC_OK && bitmap_shape(prm.acc[kAccMode], prm.acc[kAccGranules], prm.bitmap_pool_words) >= 0;
}

__global__ void __launch_bounds__(256) nbr_count(PlanParams prm)
{
    __shared__ uint32_t total;
    if (!index_wanted(prm)) return;
    const uint32_t i = blockIdx.x, n = prm.n;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    const uint32_t ta = prm.ta[i], tf = prm.tf[i];
    uint32_t c = 0;
    for (uint32_t j = threadIdx.x; j < n; j += 256) c += (j != i && prm.ta[j] < tf && ta < prm.tf[j]);
    c = wave_sum32(c);
    if (lane_id() == 0) atomicAdd(&total, c);
    __syncthreads();
    if (threadIdx.x == 0) prm.nbr_begin[i] = total;
}

__global__ void __launch_bounds__(1024) nbr_scan(PlanParams prm)
{
    __shared__ uint32_t part[1024];
    if (!index_wanted(prm)) return;
    const uint32_t n = prm.n;
    const uint32_t per = (n + 1023) / 1024;
    const uint32_t lo = threadIdx.x * per, hi = lo + per < n ? lo + per : n;
    uint32_t sum = 0;
    for (uint32_t i = lo; i < hi; ++i) sum += (prm.nbr_begin[i] + kRowPad - 1) / kRowPad;
    part[threadIdx.x] = sum;
    __syncthreads();
    for (uint32_t d = 1; d < 1024; d <<= 1) {            // inclusive scan of the per-thread sums
        const uint32_t add = threadIdx.x >= d ? part[threadIdx.x - d] : 0u;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t run = part[threadIdx.x] - sum;
    for (uint32_t i = lo; i < hi; ++i) {
        const uint32_t chunks = (prm.nbr_begin[i] + kRowPad - 1) / kRowPad;
        prm.nbr_begin[i] = run;
        run += chunks;
    }
    if (threadIdx.x == 1023) prm.nbr_begin[n] = part[1023];
}

// Fills row i.  The order of a row's entries is free (the bitmap is an OR over the row), so it is
// chosen for the table lookups of the build phase: one lookup instruction reads the table cells
// of 64 consecutive entries of this order, and LDS serves them fastest when they lie in different
// banks (cell j is in bank j mod 32).  Entries are ordered by (rank, bank), rank = how many
// entries of the same bank come before: any 64 in a row then hold every bank about twice.
// Within a chunk of 256, entry e belongs to lane e / 4 and lookup e mod 4, hence the transposition.
__global__ void __launch_bounds__(256) nbr_fill(PlanParams prm)
{
    constexpr uint32_t kMaxRank = kBmMaxRequests / 32;
    __shared__ uint32_t per_thread[256];
    __shared__ uint32_t in_bank[32];
    __shared__ uint32_t before_rank[kMaxRank + 1];      // entries with a lower rank
    __shared__ uint32_t banks_at_rank[kMaxRank + 1];    // banks that have an entry of this rank
    if (!index_wanted(prm)) return;
    const uint32_t i = blockIdx.x, n = prm.n, t = threadIdx.x;
    const uint32_t bank = t & 31u;                      // thread t sees j = t, t + 256, ...: all in one bank
    const uint32_t ta = prm.ta[i], tf = prm.tf[i];
    uint32_t mine = 0;
    for (uint32_t j = t; j < n; j += 256) mine += (j != i && prm.ta[j] < tf && ta < prm.tf[j]);
    per_thread[t] = mine;
    __syncthreads();
    uint32_t rank = 0, total = 0;                       // of the 8 threads of a bank, the lower ones come first
    for (uint32_t m = 0; m < 8; ++m) {
        const uint32_t c = per_thread[bank + 32 * m];
        if (m < (t >> 5)) rank += c;
        total += c;
    }
    if (t < 32) in_bank[t] = total;
    __syncthreads();
    for (uint32_t r = t; r <= kMaxRank; r += 256) {
        uint32_t before = 0, banks = 0;
        for (uint32_t b = 0; b < 32; ++b) {
            const uint32_t c = in_bank[b];
            before += c < r ? c : r;
            banks |= (c > r ? 1u : 0u) << b;
        }
        before_rank[r] = before;
        banks_at_rank[r] = banks;
    }
    __syncthreads();
    uint16_t* row = prm.nbr + (size_t)prm.nbr_begin[i] * kRowPad;
    const uint32_t room = (prm.nbr_begin[i + 1] - prm.nbr_begin[i]) * kRowPad;
    auto slot = [](uint32_t pos) {                      // position in the order -> entry of the row
        const uint32_t p = pos % kRowPad;
        return pos - p + 4 * (p % kWave) + p / kWave;
    };
    for (uint32_t j = t; j < n; j += 256) {
        if (j != i && prm.ta[j] < tf && ta < prm.tf[j]) {
            const uint32_t pos = before_rank[rank] + (uint32_t)__builtin_popcount(banks_at_rank[rank] & ((1u << bank) - 1u));
            if (pos < room) row[slot(pos)] = (uint16_t)(j << entry_shift(n));
            ++rank;
        }
    }
    const uint32_t filled = before_rank[kMaxRank];      // = number of entries
    for (uint32_t pos = filled + t; pos < room; pos += 256) row[slot(pos)] = (uint16_t)(n << entry_shift(n));
}

// ---------------------------------------------------------------------------------------------

// A placed block as the build phase wants it: bits 0-21 address in granules (bits 0-4 = first bit
// b in its first word, bits 5-21 = that word), bits 22-26 size in granules (1..31), bits 27-31 the
// number of granules that spill into the next word.  0 = not placed.
constexpr uint32_t kCellSizeAt = 22, kCellSpillAt = 27;
__device__ __forceinline__ uint32_t make_cell(uint32_t x, uint32_t sz)
{
    const uint32_t reach = (x & 31) + sz;
    return x | (sz << kCellSizeAt) | ((reach > 32 ? reach - 32 : 0u) << kCellSpillAt);
}

// ((1 << width) - 1) << offset with both taken modulo 32.
__device__ __forceinline__ uint32_t bit_field_mask(uint32_t width, uint32_t offset)
{
    uint32_t r;
    asm("v_bfm_b32 %0, %1, %2" : "=v"(r) : "v"(width), "v"(offset));
    return r;
}

typedef __attribute__((address_space(3))) uint32_t lds_word;

// LDS address of the first bitmap word of the block of `cell`: field extract, shift-add.
__device__ __forceinline__ lds_word* first_word(uint32_t* bm, uint32_t cell)
{
    const uint32_t base = (uint32_t)reinterpret_cast<uintptr_t>((lds_word*)bm);
    uint32_t at;
    asm("v_bfe_u32 %0, %1, 5, 17\n\tv_lshl_add_u32 %0, %0, 2, %2" : "=&v"(at) : "v"(cell), "s"(base));
    return reinterpret_cast<lds_word*>((uintptr_t)at);
}

// ORs the block of `cell` into the bitmap; cell == 0 adds nothing.
__device__ __forceinline__ void mark_cell(uint32_t* bm, uint32_t cell)
{
    lds_word* word = first_word(bm, cell);
    const uint32_t first = bit_field_mask(cell >> kCellSizeAt, cell);      // ((1 << size) - 1) << b, low 32 bits
    const uint32_t spill = bit_field_mask(cell >> kCellSpillAt, 0u);       // (1 << spilled) - 1
    if (cell) __hip_atomic_fetch_or(word, first, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (cell >= (1u << kCellSpillAt)) __hip_atomic_fetch_or(word + 1, spill, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// The same for four cells per lane, looking before ORing.  Blocks that are alive at different
// times share addresses (that is the point of the plan), so most blocks of a row only repeat
// bits that are already set, and many lanes of one instruction aim at the same few words.  LDS
// serialises atomics on one address lane by lane but broadcasts reads of one address, hence:
// read the words, and send only the lanes that still add a bit into the atomic.  (A word read
// just before another wave's OR merely causes a redundant OR.)  Address and masks are worked
// out for every lane; idle lanes have empty masks and drop out with the rest.
__device__ __forceinline__ void mark_cells(uint32_t* bm, const uint32_t (&cell)[4])
{
    lds_word* word[4];
    uint32_t first[4], spill[4], seen[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        word[k] = first_word(bm, cell[k]);
        first[k] = bit_field_mask(cell[k] >> kCellSizeAt, cell[k]);
        spill[k] = bit_field_mask(cell[k] >> kCellSpillAt, 0u);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) seen[k] = *word[k];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (first[k] & ~seen[k]) __hip_atomic_fetch_or(word[k], first[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cell[k] >= (1u << kCellSpillAt)) __hip_atomic_fetch_or(word[k] + 1, spill[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// Lowest bit position x such that bits [x, x + s) of the bitmap are zero; words at and beyond
// `limit` count as free.  1 <= s <= 32, s and limit uniform.  Whole wave, uniform result.
__device__ __forceinline__ uint32_t first_fit(const uint32_t* bm, uint32_t limit, uint32_t s)
{
    const int lane = lane_id();
    for (uint32_t t = 0;; t += kWave) {
        const uint32_t w = t + lane;
        const uint32_t here = w < limit ? bm[w] : 0u;
        const uint32_t next = w + 1 < limit ? bm[w + 1] : 0u;
        uint64_t free_run = ~((uint64_t)here | ((uint64_t)next << 32));     // bit b: granule 32 w + b is free
        for (uint32_t len = 1; len < s;) {                                  // bit b: free for `len` granules from b
            const uint32_t step = len < s - len ? len : s - len;
            free_run &= free_run >> step;
            len += step;
        }
        const uint32_t starts = (uint32_t)free_run;                         // runs that begin inside word w
        const uint64_t any = __builtin_amdgcn_uicmp(starts, 0u, 33);        // != 0
        if (any) {
            const int f = __builtin_ctzll(any);
            return (t + (uint32_t)f) * 32 + (uint32_t)__builtin_ctz(read_lane(starts, f));
        }
    }
}

// Inclusive prefix sum inside each row of 16 lanes.
__device__ __forceinline__ uint32_t row_scan_add(uint32_t v)
{
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr2, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr4, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0u, v, kDppRowShr8, 0xf, 0xf, false);
    return v;
}

// (eight-wave shape: 8 waves per SIMD = 64 VGPRs at most, so that four workgroups share a CU)
template <int kWaves, bool kScaledEntries>
__global__ void __launch_bounds__(kWaves * kWave, kWaves == 8 ? 8 : 4) plan_bitmap_kernel(PlanParams prm)
{
    using Lds = BitmapLds<kWaves>;
    constexpr int kThreads = kWaves * kWave;
    constexpr int kShape = kWaves == 8 ? 0 : 1;
    constexpr int kAhead = kWaves == 8 ? 8 : 12;      // chunks per wave and batch whose index entries are fetched ahead
    static_assert(bitmap_shape_waves(kShape) == (uint32_t)kWaves, "shape table and instantiation disagree");
    extern __shared__ __align__(16) unsigned char smem[];
    Lds& sh = *reinterpret_cast<Lds*>(smem);
    uint32_t* cells = reinterpret_cast<uint32_t*>(smem + sizeof(Lds));     // [n + 1] placed blocks, see make_cell
    uint32_t* pool = cells + (prm.n + 1);
    const uint32_t n = prm.n;

    if (*prm.status != STALLOC_OK) return;
    if (bitmap_shape(prm.acc[kAccMode], prm.acc[kAccGranules], prm.bitmap_pool_words) != kShape) return;
    const uint32_t shift = (uint32_t)(prm.acc[kAccMode] & 63);
    if (blockIdx.x == 0 && threadIdx.x == 0) const_cast<uint64_t*>(prm.acc)[kAccKernel] = STALLOC_KERNEL_BITMAP | (22u << 8);
    const uint32_t pool_words = prm.bitmap_pool_words[kShape];
    const uint32_t half_words = pool_words / 2;        // two batches are in flight, each in its half of the pool
    // the rule above keeps every address of a well-formed plan at or below `highest`; a malformed
    // order row (repeated requests) is clamped to it so that a bitmap never outgrows its half
    const uint32_t highest = 32u * (half_words - 2 * kWaves - 5) + 31u;
    const int lane = lane_id(), wave = (int)uniform((uint32_t)wave_id());
    const uint2* index = reinterpret_cast<const uint2*>(prm.nbr) + lane;   // a chunk: 64 lanes x 4 entries

    for (uint32_t p = blockIdx.x; p < prm.P; p += gridDim.x) {
        const uint32_t* order = prm.orders + (size_t)p * n;
        uint64_t* out = prm.offsets ? prm.offsets + (size_t)p * n : nullptr;
        for (uint32_t i = threadIdx.x; i <= n; i += kThreads) cells[i] = 0;     // nothing placed; cell n pads the rows
        if (threadIdx.x == 0) sh.top = 0;

        for (uint32_t r0 = 0; r0 < n; r0 += Lds::kBmBatch) {
            const uint32_t staged = n - r0 < (uint32_t)Lds::kBmBatch ? n - r0 : (uint32_t)Lds::kBmBatch;
            __syncthreads();                                  // previous refill fully consumed
            if (threadIdx.x < staged) {
                uint32_t i = order[r0 + threadIdx.x];
                if (i >= n) { atomicMax(prm.status, (uint32_t)STALLOC_ERR_BAD_ORDER); i = 0; }
                sh.rq_id[threadIdx.x] = i;
                sh.rq_s[threadIdx.x] = (uint32_t)(prm.size[i] >> shift);
                sh.rq_ta[threadIdx.x] = prm.ta[i];
                sh.rq_tf[threadIdx.x] = prm.tf[i];
                const uint32_t c0 = prm.nbr_begin[i];
                sh.rq_row[threadIdx.x] = c0;
                sh.rq_chunks[threadIdx.x] = prm.nbr_begin[i + 1] - c0;
            }
            __syncthreads();

            // A batch: requests first .. first + nb - 1 of the refill, their bitmaps `stride` words apart
            // and `limit` words long in one half of the pool.  A batch is sized when its half is cleared:
            // two batches are in flight, so every block that can exist while it is in use ends below
            // the extent at that moment plus 2 * kWaves of the longest requests.
            struct Batch { uint32_t first, nb, limit, stride; };
            auto size_batch = [&](uint32_t first) -> Batch {
                Batch b;
                b.first = first;
                b.limit = uniform(sh.top) / 32 + 2 * kWaves + 2;
                b.stride = b.limit | 1u;
                uint32_t fit = half_words / b.stride;             // >= 1
                if (fit > (uint32_t)kWaves) fit = kWaves;
                b.nb = first >= staged ? 0u : (staged - first < fit ? staged - first : fit);
                return b;
            };
            // Which chunks a wave takes: wave 0 settles the previous batch while the others already
            // build, so it gets a smaller share -- of every kShares * (kWaves - 1) + 1 chunks, kShares
            // go to each of the waves 1 .. kWaves - 1 and the last one to wave 0.
            constexpr uint32_t kPeriod = kShares * (kWaves - 1) + 1;
            auto chunk_of = [&](uint32_t j) -> uint32_t {          // the wave's j-th chunk (ascending in j)
                return wave == 0 ? j * kPeriod + (kPeriod - 1)
                                 : (j / kShares) * kPeriod + (j % kShares) * (kWaves - 1) + (uint32_t)(wave - 1);
            };
            auto chunks_of_wave = [&](uint32_t total) -> uint32_t { // how many of `total` chunks are the wave's
                const uint32_t full = total / kPeriod, rest = total % kPeriod;
                if (wave == 0) return full;
                uint32_t c = full * kShares;
                for (uint32_t k = 0; k < kShares; ++k) c += k * (kWaves - 1) + (uint32_t)(wave - 1) < rest ? 1u : 0u;
                return c;
            };
            // The rows of a batch, cut into chunks and numbered through.  Lane q < 16 describes the row
            // of request q of the batch; `mine` = how many of the chunks are this wave's.
            struct Rows { uint32_t row, chunks, end, total, mine; };
            auto rows_of = [&](const Batch& b) -> Rows {
                Rows r = {0, 0, 0, 0, 0};
                if (lane < (int)b.nb) { r.row = sh.rq_row[b.first + lane]; r.chunks = sh.rq_chunks[b.first + lane]; }
                r.end = row_scan_add(r.chunks);                   // (nb <= 16: one DPP row)
                r.total = read_lane(r.end, 15);
                r.mine = chunks_of_wave(r.total);
                return r;
            };
            // chunk f belongs to request q = number of rows that end at or before f
            auto locate = [&](const Rows& r, uint32_t f, uint32_t& q) -> const uint2* {
                q = (uint32_t)__builtin_popcountll(lanes_ge(f, r.end) & 0xffffull);
                const uint32_t at = read_lane(r.row, (int)q) + f - (read_lane(r.end, (int)q) - read_lane(r.chunks, (int)q));
                return index + (size_t)at * (kRowPad / 4);
            };
            // The index entries of a wave's first kAhead chunks of a batch are fetched when the batch is
            // sized, a whole batch before they are used: the index is far larger than the L2 and a
            // fetch takes about as long as a chunk takes to process.
            uint2 ahead[kAhead];
            uint32_t ahead_q[kAhead];
            auto fetch_ahead = [&](const Rows& r) {
#pragma unroll
                for (int j = 0; j < kAhead; ++j) {
                    ahead_q[j] = 0;
                    if ((uint32_t)j < r.mine) ahead[j] = *locate(r, chunk_of((uint32_t)j), ahead_q[j]);
                }
            };
            auto lookup = [&](const uint2& ids, uint32_t (&cell)[4]) {
                const uint32_t e[4] = {ids.x & 0xffffu, ids.x >> 16, ids.y & 0xffffu, ids.y >> 16};
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    cell[k] = kScaledEntries ? *reinterpret_cast<const uint32_t*>(reinterpret_cast<const unsigned char*>(cells) + e[k])
                                             : cells[e[k]];
            };
            auto clear = [&](uint32_t* bitmaps, const Batch& b) {
                if ((uint32_t)wave < b.nb)
                    for (uint32_t w = lane; w < b.limit; w += kWave) bitmaps[(uint32_t)wave * b.stride + w] = 0;
            };
            // build: table lookups of one chunk are in flight while the previous one is marked
            auto build = [&](uint32_t* bitmaps, const Batch& b, const Rows& rows) {
                uint32_t cell[4] = {0, 0, 0, 0}, looked[4] = {0, 0, 0, 0};
                if (rows.mine) lookup(ahead[0], cell);
#pragma unroll
                for (int j = 0; j < kAhead; ++j) {
                    if ((uint32_t)j < rows.mine) {
                        if (j + 1 < kAhead && (uint32_t)j + 1 < rows.mine) lookup(ahead[j + 1 < kAhead ? j + 1 : j], looked);
                        mark_cells(bitmaps + ahead_q[j] * b.stride, cell);
#pragma unroll
                        for (int k = 0; k < 4; ++k) cell[k] = looked[k];
                    }
                }
                for (uint32_t j = kAhead; j < rows.mine; ++j) {                           // (long rows only)
                    uint32_t q;
                    const uint2 ids = *locate(rows, chunk_of(j), q);
                    lookup(ids, cell);
                    mark_cells(bitmaps + q * b.stride, cell);
                }
            };
            // search: lowest fit of request q of the batch against what its bitmap holds
            auto search = [&](uint32_t* bitmaps, const Batch& b) {
                if ((uint32_t)wave < b.nb) {
                    const uint32_t x = first_fit(bitmaps + (uint32_t)wave * b.stride, b.limit, uniform(sh.rq_s[b.first + wave]));
                    if (lane == 0) sh.cand[wave] = x;
                }
            };
            // settle (one wave): the requests of the batch in order.  The bitmaps hold every block
            // placed before the batch except possibly those of the batch just before it (they were
            // being settled while these bitmaps were built).  A candidate stands unless one of those,
            // or a request settled earlier in this batch, overlaps it in lifetime and in address
            // range; only then are those blocks ORed into the request's bitmap and the search
            // repeated (adding blocks only removes free runs; ORing a block twice changes nothing).
            // Lanes 0 .. kWaves-1: the batch before (settled); lanes kWaves .. : this batch.
            auto settle = [&](uint32_t* bitmaps, const Batch& b, uint32_t nb_prev) {
                uint32_t my_s = 0, my_ta = 0xffffffffu, my_tf = 0, mine = 0;     // empty lifetime: conflicts with nothing
                const bool prev = lane < kWaves && (uint32_t)(kWaves - lane) <= nb_prev;    // request first - (kWaves - lane)
                const bool cur = lane >= kWaves && (uint32_t)(lane - kWaves) < b.nb;
                if (prev || cur) {
                    const uint32_t at = b.first + (uint32_t)lane - kWaves;
                    my_s = sh.rq_s[at];
                    my_ta = sh.rq_ta[at];
                    my_tf = sh.rq_tf[at];
                    mine = prev ? sh.rq_x[at] : sh.cand[lane - kWaves];
                }
                uint32_t top = sh.top;
                for (uint32_t r = 0; r < b.nb; ++r) {
                    const int at = kWaves + (int)r;
                    const uint32_t s = read_lane(my_s, at), ta = read_lane(my_ta, at), tf = read_lane(my_tf, at);
                    uint32_t x = read_lane(mine, at);
                    const bool rival = lane < at && my_ta < tf && ta < my_tf;
                    if (__builtin_amdgcn_ballot_w64(rival && mine < x + s && x < mine + my_s)) {
                        if (rival) mark_cell(bitmaps + r * b.stride, make_cell(mine, my_s));
                        x = first_fit(bitmaps + r * b.stride, b.limit, s);
                    }
                    if (x > highest) x = highest;                          // only reachable with a malformed order row
                    if (lane == at) mine = x;
                    top = umax(top, x + s);
                }
                if (cur) {
                    cells[sh.rq_id[b.first + lane - kWaves]] = make_cell(mine, my_s);
                    sh.rq_x[b.first + lane - kWaves] = mine;
                }
                if (lane == 0) sh.top = top;
            };

            // Software pipeline over the batches of the refill: while wave 0 settles batch B in one
            // half of the pool, all waves (wave 0 once it is done) build the bitmaps of batch B + 1 in
            // the other half; then B + 1 is searched, and the half of B is cleared for B + 2.
            uint32_t* half[2] = {pool, pool + half_words};
            int h = 0;
            Batch cur = size_batch(0);
            Rows rows = rows_of(cur);
            fetch_ahead(rows);
            clear(half[0], cur);
            __syncthreads();
            build(half[0], cur, rows);
            Batch nxt = size_batch(cur.nb);
            if (nxt.nb) {
                rows = rows_of(nxt);
                fetch_ahead(rows);
                clear(half[1], nxt);
            }
            __syncthreads();
            search(half[0], cur);
            __syncthreads();
            uint32_t nb_prev = 0;
            while (cur.nb) {
                if (wave == 0) settle(half[h], cur, nb_prev);
                if (nxt.nb) build(half[h ^ 1], nxt, rows);
                __syncthreads();
                Batch after = {0, 0, 0, 0};
                if (nxt.nb) {
                    search(half[h ^ 1], nxt);
                    after = size_batch(nxt.first + nxt.nb);
                    if (after.nb) {
                        rows = rows_of(after);
                        fetch_ahead(rows);
                        clear(half[h], after);
                    }
                    __syncthreads();
                }
                nb_prev = cur.nb;
                cur = nxt;
                nxt = after;
                h ^= 1;
            }
            if (out && threadIdx.x < staged) out[sh.rq_id[threadIdx.x]] = (uint64_t)sh.rq_x[threadIdx.x] << shift;
        }
        if (threadIdx.x == 0) prm.peaks[p] = (uint64_t)sh.top << shift;
        __syncthreads();                                      // sh.top read before the next plan clears it
    }
}

// Workgroups per CU of the eight-wave shape for a trace of n requests, and the words of its
// bitmap pool: as many workgroups as leave each a pool of 2 * kBmWords words.  0 = none.
static uint32_t shared_cu_residency(uint32_t n, const DeviceInfo& di, uint32_t* pool_words)
{
    const size_t fixed = sizeof(BitmapLds<8>) + ((size_t)n + 1) * sizeof(uint32_t);
    for (uint32_t wgs = 4; wgs >= 2; --wgs) {
        const size_t budget = di.lds_per_block / wgs / 512 * 512;       // LDS is handed out in 512-byte pieces
        if (budget < fixed + 2 * (size_t)kBmWords * sizeof(uint32_t)) continue;
        *pool_words = (uint32_t)((budget - fixed) / sizeof(uint32_t));
        return wgs;
    }
    return 0;
}

bool bitmap_plan_shapes(uint32_t n, const DeviceInfo& di, uint32_t (&pool_words)[kBitmapShapes])
{
    pool_words[0] = pool_words[1] = 0;
    if (n > kBmMaxRequests) return false;
    shared_cu_residency(n, di, &pool_words[0]);
    const size_t fixed = sizeof(BitmapLds<16>) + ((size_t)n + 1) * sizeof(uint32_t);
    if (di.lds_per_block >= fixed + (size_t)kBmWords * sizeof(uint32_t))
        pool_words[1] = (uint32_t)((di.lds_per_block - fixed) / sizeof(uint32_t));
    return pool_words[0] != 0 || pool_words[1] != 0;
}

size_t bitmap_index_entries(uint32_t n)
{
    return (size_t)n * (((size_t)n - 1 + kRowPad - 1) / kRowPad * kRowPad);
}

template <int kWaves>
static bool launch_shape(const PlanParams& prm, uint32_t wgs_per_cu, uint32_t pool_words, const DeviceInfo& di,
                         hipStream_t stream)
{
    auto kernel = entry_shift(prm.n) ? &plan_bitmap_kernel<kWaves, true> : &plan_bitmap_kernel<kWaves, false>;
    const size_t lds = sizeof(BitmapLds<kWaves>) + ((size_t)prm.n + 1 + pool_words) * sizeof(uint32_t);
    static std::atomic<bool> attr_set[64][2] = {};     // (set twice at worst when threads race)
    if (!attr_set[di.device][entry_shift(prm.n) ? 1 : 0]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)di.lds_per_block) != hipSuccess)
            return false;
        attr_set[di.device][entry_shift(prm.n) ? 1 : 0] = true;
    }
    uint32_t grid = (uint32_t)di.cus * wgs_per_cu;
    if (grid > prm.P) grid = prm.P;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kWaves * kWave), lds, stream, prm);
    return true;
}

// Enqueues the index build and every shape of the placement kernel that prm.bitmap_pool_words names.
bool launch_plan_bitmap(const PlanParams& prm, const DeviceInfo& di, hipStream_t stream)
{
    hipLaunchKernelGGL(nbr_count, dim3(prm.n), dim3(256), 0, stream, prm);
    hipLaunchKernelGGL(nbr_scan, dim3(1), dim3(1024), 0, stream, prm);
    hipLaunchKernelGGL(nbr_fill, dim3(prm.n), dim3(256), 0, stream, prm);
    bool ok = true;
    if (prm.bitmap_pool_words[0]) {
        uint32_t pool_words = 0;
        const uint32_t wgs = shared_cu_residency(prm.n, di, &pool_words);
        ok = ok && wgs != 0 && pool_words == prm.bitmap_pool_words[0] && launch_shape<8>(prm, wgs, pool_words, di, stream);
    }
    if (prm.bitmap_pool_words[1]) ok = ok && launch_shape<16>(prm, 1, prm.bitmap_pool_words[1], di, stream);
    return ok;
}

}  // namespace stalloc
