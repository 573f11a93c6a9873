/*
 * stalloc -- offline spatio-temporal placement of an allocation trace on one GPU.
 *
 * A trace is the list M of memory request events of one training iteration
 * (Sec. 4): request i is the rectangle  size[i] bytes x [t_alloc[i], t_free[i]).
 * A plan gives every request a start address (allocation decision d = m + (a),
 * Sec. 5.1) such that no two decisions conflict in lifespan and in address range
 * at the same time (the constraint of Sec. 5.1).  The extent of a plan is
 * max_i (a_i + size_i) (Eq. 2, Eq. 6); memory efficiency is E = M_a / M_r (Eq. 1)
 * with M_a the maximum over time of live bytes and M_r the extent.
 *
 * Conventions shared by all entry points
 *   - Every data pointer is a DEVICE pointer owned by the caller; nothing is
 *     allocated or freed by the library.  `stalloc_trace` itself and
 *     `workspace_bytes` live in HOST memory.
 *   - Work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream) of
 *     the current device and is asynchronous: outputs are valid once the stream
 *     has been synchronised.
 *   - Query-then-call workspace: with workspace == NULL the required size is
 *     written to *workspace_bytes and nothing else happens.  Otherwise
 *     *workspace_bytes must be at least that size and `workspace` 256-byte aligned.
 *   - Return value: a stalloc_status for everything the host can see (NULL
 *     pointers, n == 0, P == 0, workspace too small, launch failure).  Defects only
 *     visible on the device (size 0, t_alloc >= t_free, t_free > t_end, sum of sizes
 *     >= 2^63, an order entry >= n, an empty time window, a layer number that does not
 *     exist) are written as a stalloc_status to
 *     `device_status[0]` (0 when clean); when it is non-zero every other output of
 *     that call is unspecified, but all kernels still terminate normally.
 *   - Lifetimes and address ranges are half-open; no alignment is applied; byte
 *     quantities are uint64_t; timestamps are uint32_t event ranks below t_end.
 *   - Calls that share a workspace or outputs must be ordered by the caller; otherwise the
 *     entry points may be called from several host threads at once.
 */
#ifndef STALLOC_H
#define STALLOC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum stalloc_status {
    STALLOC_OK = 0,
    STALLOC_ERR_INVALID_ARG = 1, /* NULL pointer, n == 0, P == 0, size limits, workspace too small */
    STALLOC_ERR_BAD_TRACE = 2,   /* size 0, t_alloc >= t_free or t_free > t_end                  */
    STALLOC_ERR_OVERFLOW = 3,    /* sum of sizes >= 2^63: addresses could wrap                    */
    STALLOC_ERR_NOMEM = 4,       /* reserved                                                      */
    STALLOC_ERR_DEVICE = 5,      /* a HIP call failed                                             */
    STALLOC_ERR_BAD_ORDER = 6,   /* an entry of `orders` is >= n                                  */
    STALLOC_ERR_BAD_WINDOW = 7,  /* a time window with w_lo >= w_hi                               */
    STALLOC_ERR_BAD_LAYER = 8,   /* an entry of `layer_of` is >= n_layers                         */
    STALLOC_ERR_TOO_LARGE = 9    /* the trace exceeds what an entry point without workspace holds */
} stalloc_status;

/* Structure-of-arrays trace (Sec. 4: s, t_s, t_e of every request event). */
typedef struct stalloc_trace {
    uint32_t n;              /* number of requests, 1 <= n < 2^31                          */
    uint32_t t_end;          /* number of timestamps: every t_free <= t_end < 2^31         */
    const uint64_t *size;    /* device [n], bytes, > 0                                     */
    const uint32_t *t_alloc; /* device [n]                                                 */
    const uint32_t *t_free;  /* device [n], t_alloc[i] < t_free[i] <= t_end                */
} stalloc_trace;

/*
 * Batched greedy placement: P candidate placement orders are evaluated
 * independently and the plan with the smallest extent is kept.
 *
 * For plan p the requests are taken in the order orders[p][0..n-1]; each one gets
 * the lowest address at which it conflicts with no request placed before it in
 * that plan (the lowest-fit rule of Sec. 5.1; large-first orders let small
 * requests fill the unused intervals of larger ones, Sec. 5.1 Global Planning).
 * For a given trace and order the result is unique.
 *
 *   orders        device [P][n] uint32, each row a permutation of 0..n-1.  A row
 *                 with an entry >= n sets device_status to STALLOC_ERR_BAD_ORDER; a
 *                 row that repeats entries is not detected and yields an unspecified
 *                 (but memory-safe) plan.
 *   offsets       device [P][n], address of request i in plan p at offsets[p*n+i];
 *                 may be NULL when only extents / the best plan are wanted.
 *   peaks         device [P], extent of each plan (Eq. 2).
 *   best_offsets  device [n], addresses of the best plan; may be NULL.
 *   best_plan     device [1], index of the smallest extent, lowest index among equals.
 *   device_status device [1], see above; must not be NULL.
 *   workspace     sized for whatever the trace may turn out to need, which only the device
 *                 learns: for n <= 32768 this includes an index of the request pairs with
 *                 overlapping lifetimes at its upper bound of about 2 n^2 bytes (76 MB for
 *                 n = 6144, 0.8 GB for n = 19840); plus (P x n) x 8 bytes when best_offsets
 *                 is wanted without offsets.
 */
int stalloc_plan(const stalloc_trace *trace, const uint32_t *orders, uint32_t P,
                 uint64_t *offsets, uint64_t *peaks, uint64_t *best_offsets,
                 uint32_t *best_plan, uint32_t *device_status,
                 void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * stalloc_plan for a caller that knows something about its sizes (same rule, same results; Sec. 5.1).
 * Which kernel places a trace is decided on the device, so stalloc_plan sizes its workspace for all
 * of them, among them the one for traces of few granules with its index of lifetime-overlapping pairs
 * (about 2 n^2 bytes for n <= 32768).  With
 *   largest_size  no request is larger than this many bytes (> 0), and
 *   granule       a power of two that divides every size (1 if nothing better is known),
 * a call whose sizes cannot suit that kernel (largest_size / granule > 31) leaves it and its index out
 * of the launch and of the workspace.  The figures are only used to leave work out: wrong ones cost
 * time or memory, never correctness.  The workspace query and the call must be given the same two.
 */
int stalloc_plan_sized(const stalloc_trace *trace, const uint32_t *orders, uint32_t P,
                       uint64_t *offsets, uint64_t *peaks, uint64_t *best_offsets,
                       uint32_t *best_plan, uint32_t *device_status,
                       uint64_t largest_size, uint64_t granule,
                       void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * Pairwise check of the constraint of Sec. 5.1 for P plans of one trace.
 *
 *   offsets     device [P][n].  offsets + size must stay below 2^64 for every request of every
 *               plan: a range that would wrap sets device_status to STALLOC_ERR_OVERFLOW (it is
 *               then counted as reaching up to 2^64 - 1)
 *   conflicts   device [P], number of unordered pairs (i, j) whose lifetimes
 *               overlap and whose address ranges overlap
 *   first_pair  device [P][2], the lexicographically first such pair with i < j,
 *               {0xFFFFFFFF, 0xFFFFFFFF} when the plan is valid
 */
int stalloc_validate(const stalloc_trace *trace, const uint64_t *offsets, uint32_t P,
                     uint64_t *conflicts, uint32_t *first_pair, uint32_t *device_status,
                     void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * M_a of Eq. 1: the maximum over t in [0, t_end) of the bytes alive at t, found
 * with a prefix sum over the allocation/release events.  No plan can have a
 * smaller extent.
 *
 *   lower_bound device [1]
 *   t_at_max    device [1], the earliest t reaching the maximum; may be NULL
 */
int stalloc_lower_bound(const stalloc_trace *trace, uint64_t *lower_bound, uint32_t *t_at_max,
                        uint32_t *device_status,
                        void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * stalloc_lower_bound for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same outputs as
 * stalloc_lower_bound, no workspace argument: the net-change array and the partial results
 * live in a fixed buffer inside the library (STALLOC_STATIC_MAX_T_END + 1 64-bit words plus
 * about 3 KB, 4 MiB in all, resident on every GPU the library runs on until the process
 * ends).  Neither this call nor anything it calls allocates or frees memory.
 *
 *   trace->t_end above STALLOC_STATIC_MAX_T_END returns STALLOC_ERR_TOO_LARGE; nothing is
 *   enqueued then.
 *   All calls on one GPU share that GPU's buffer: calls that can overlap in time on one GPU
 *   (different streams, several host threads) race and must be ordered by the caller.  The
 *   buffer keeps the previous call's contents between calls; every call rewrites what it reads.
 */
#define STALLOC_STATIC_MAX_T_END 524288u
int stalloc_lower_bound_static(const stalloc_trace *trace, uint64_t *lower_bound, uint32_t *t_at_max,
                               uint32_t *device_status, void *hip_stream);

/*
 * Dynamic reusable space of one plan (Sec. 5.2): for each of k time windows
 * T = [w_lo, w_hi) the address intervals of the pool that stay idle throughout T, so
 * that requests living inside T can be served from them without touching any planned
 * decision.  With D the plan's decisions: A_o(T) is the union of the address ranges
 * R_s(d) of the d in D whose lifespan R_t(d) meets T; A = [min d.a, max (d.a + d.s));
 * the result is A_i(T) = A minus A_o(T), as its maximal intervals in ascending order.
 * Windows are half-open like lifespans: d meets T iff t_alloc < w_hi and w_lo < t_free.
 *
 *   offsets     device [n], the plan (for instance best_offsets of stalloc_plan); it need
 *               not be conflict-free, but offsets[i] + size[i] must not wrap
 *   windows     device [k][2] uint32 {w_lo, w_hi}; w_lo >= w_hi sets device_status to
 *               STALLOC_ERR_BAD_WINDOW
 *   max_ranges  capacity of one row of `ranges` (n + 1 always suffices)
 *   ranges      device [k][max_ranges][2] {lo, hi}: the first max_ranges intervals of each
 *               window; may be NULL when max_ranges == 0
 *   counts      device [k], number of intervals of each window (may exceed max_ranges)
 *   idle_bytes  device [k], total length of all intervals of each window; may be NULL
 *
 * The workspace size depends on n and k: query it with the k of the call.
 */
int stalloc_reusable_space(const stalloc_trace *trace, const uint64_t *offsets,
                           const uint32_t *windows, uint32_t k, uint32_t max_ranges,
                           uint64_t *ranges, uint32_t *counts, uint64_t *idle_bytes,
                           uint32_t *device_status,
                           void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * Memory-layer construction for every HomoSize group of the trace (Sec. 5.1, HomoSize
 * Group Planning, Algorithm 1).  A HomoSize group holds the requests of one size;
 * requests of a group whose lifetimes do not overlap can share one range of that
 * size, a memory-layer.  The requests of a group are taken by allocation time
 * (request number among equals); each joins, as its last request, the layer that is
 * free at its allocation time and whose last request was released latest (the layer
 * opened first among equals), so that the layer idles least; if no layer is free a
 * new one is opened.  Lifetimes are half-open: a layer whose last request is released
 * at t is free for a request allocated at t.  A group gets as few layers as any
 * assignment can have.
 *
 * Layers are numbered group by group in descending size and, inside a group, in the
 * order in which they were opened.  A layer planned as one request of its size from
 * the allocation of its first request to the release of its last one (the local plan
 * of the group becomes part of the global plan, Sec. 5.1) gives all its requests one
 * address: (layer_size, layer_t_alloc, layer_t_free) is a trace of *n_layers requests
 * that stalloc_plan accepts, with t_end of the original trace.
 *
 *   layer_of       device [n], layer of every request
 *   n_layers       device [1]
 *   layer_size     device [n], the first *n_layers entries are written
 *   layer_t_alloc  device [n], likewise
 *   layer_t_free   device [n], likewise
 */
int stalloc_memory_layers(const stalloc_trace *trace, uint32_t *layer_of, uint32_t *n_layers,
                          uint64_t *layer_size, uint32_t *layer_t_alloc, uint32_t *layer_t_free,
                          uint32_t *device_status,
                          void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * Plans of the layers back to plans of the requests: every request takes the address of
 * its layer, offsets[p][i] = layer_offsets[p][layer_of[i]].  Plans that are free of
 * conflicts for the layer trace are free of conflicts for the requests and have the
 * same extent.
 *
 *   layer_of       device [n], as written by stalloc_memory_layers
 *   layer_offsets  device [P][n_layers], for instance `offsets` of stalloc_plan on the
 *                  layer trace
 *   n_layers       host value (read back from stalloc_memory_layers); an entry of
 *                  layer_of that is >= n_layers sets device_status to STALLOC_ERR_BAD_LAYER
 *   offsets        device [P][n]
 *   device_status  device [1], written (STALLOC_OK or the error); no workspace is needed
 */
int stalloc_expand_layers(uint32_t n, uint32_t P, const uint32_t *layer_of,
                          const uint64_t *layer_offsets, uint32_t n_layers, uint64_t *offsets,
                          uint32_t *device_status, void *hip_stream);

/*
 * Time-memory product of Eq. 2 for P plans of one trace, the whole plan taken as the
 * group: the memory-time the requests use, sum of size * (t_free - t_alloc), over the
 * memory-time the plan reserves, extent * (max t_free - min t_alloc).  1 means no
 * spatio-temporal bubble; plans of one trace differ in their extent only.
 *
 *   extents  device [P], extent max(a + s) of every plan (`peaks` of stalloc_plan);
 *            an extent of 0 yields infinity
 *   tmp      device [P], double precision; the numerator is summed exactly, the result
 *            is within 10 * 2^-53 (relative) of the exact ratio
 */
int stalloc_tmp(const stalloc_trace *trace, const uint64_t *extents, uint32_t P, double *tmp,
                uint32_t *device_status,
                void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * Candidate placement orders, produced on the device: rows first_plan .. first_plan + P - 1
 * of the family below, each a permutation of 0 .. n-1 (the stable sort of the requests by the
 * row's key), ready for stalloc_plan.
 *   row 0          size descending, then allocation time: large requests first, so that
 *                  smaller ones fill the intervals they leave (Sec. 5.1, Global Planning)
 *   row 1          lifetime descending, then size descending
 *   row 2          allocation time (the order in which Algorithm 1 takes a group's requests)
 *   rows >= 3, odd   a 64-bit pseudo-random key k(p, i): a uniform random permutation
 *   rows >= 4, even  (c(i) + 1) * 2^32 + (k(p, i) >> 31), c(i) = number of distinct sizes larger
 *                  than request i's: size descending, with a random order inside each size
 *                  and a shift of up to one size to either side
 * k(p, i) = mix(i * 0xD1342543DE82EF95 + mix(seed + p)) modulo 2^64, where mix(x) is the output
 * of the SplitMix64 generator (Steele, Lea, Flood, OOPSLA 2014) whose state before the step is
 * x.  Any window of rows can be produced on its own.
 *
 *   orders   device [P][n]
 * The workspace holds the sort buffers of up to 1 GiB worth of rows at a time.
 */
int stalloc_make_orders(const stalloc_trace *trace, uint32_t first_plan, uint32_t P, uint64_t seed,
                        uint32_t *orders, uint32_t *device_status,
                        void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * Candidate fusions of HomoPhase groups, k of them at once (Sec. 5.1, HomoPhase Group Planning;
 * the accept test compares time-memory products, Eq. 2).
 *
 * A HomoPhase group holds the requests that are allocated in one computation phase and released
 * in one other phase; its local plan packs them contiguously, so that plan's extent is the sum
 * of their sizes.  Two plans are fused by inserting the smaller (by extent; the second if equal)
 * into the larger: the larger plan's requests are packed from address 0 in descending order of
 * release time (request number among equals); an address pointer starts at the lowest start
 * address of the larger plan; the smaller plan's requests are tried in order of allocation time
 * (request number among equals), the first that conflicts with nothing placed so far when put at
 * the pointer is placed there and the pointer moves up by its size; if none fits, the pointer
 * moves to the next higher start address of the larger plan; when there is none, the requests
 * still left are packed on top of everything placed, in the same order.  The fusion is accepted
 * when the fused plan's time-memory product exceeds the average of the two plans' products
 * weighted by the memory-time each reserves (extent times span from first allocation to last
 * release), which is the case exactly if the fused plan reserves less memory-time than the two
 * plans together; the comparison is made in exact integers.
 *
 *   members       device [m]: the request numbers of all pairs, pair after pair; pair p owns
 *                 members[pair_begin[p] .. pair_begin[p+1]), its first group's requests first.
 *                 The requests of one pair must be distinct (not detected: the result is then
 *                 unspecified, but memory-safe); an entry >= n sets device_status to
 *                 STALLOC_ERR_BAD_ORDER.
 *   pair_begin    device [k+1], ascending, pair_begin[0] = 0, pair_begin[k] <= m (a pair that reaches
 *                 beyond m, or backwards, sets device_status to STALLOC_ERR_INVALID_ARG).
 *   count1        device [k]: how many of pair p's requests belong to its first group; both
 *                 groups must be non-empty (else device_status = STALLOC_ERR_INVALID_ARG).
 *   largest_pair  the largest pair_begin[p+1] - pair_begin[p]; a pair lives in one workgroup's
 *                 LDS (32 bytes per request): beyond about 5000 requests the call returns
 *                 STALLOC_ERR_TOO_LARGE; a pair larger than largest_pair sets device_status to it.
 *   order         device [m]: per pair, the request numbers in the fused plan's order: the larger
 *                 group's in packing order, then the smaller group's by allocation time.
 *   addr          device [m]: the addresses of those requests in the fused plan.
 *   extents       device [k][3]: extent of plan 1, of plan 2, of the fused plan.
 *   accepted      device [k]: 1 if the fusion is accepted, else 0.
 * Outputs of a pair are written only when device_status stays STALLOC_OK up to its turn.
 */
int stalloc_fuse_groups(const stalloc_trace *trace, const uint32_t *members, const uint32_t *pair_begin,
                        const uint32_t *count1, uint32_t k, uint32_t m, uint32_t largest_pair, uint32_t *order,
                        uint64_t *addr, uint64_t *extents, uint32_t *accepted, uint32_t *device_status,
                        void *workspace, size_t *workspace_bytes, void *hip_stream);

/*
 * Informational: what the stalloc_plan call that last used `workspace` did with its trace.
 * Synchronises `hip_stream` (the stream of that call) and reads a few words back; `info` is HOST
 * memory.  Which kernel places a trace is decided on the device, from the trace alone:
 *   STALLOC_KERNEL_BITMAP       per-plan table of placed blocks plus per-request occupancy bitmaps
 *                               in LDS (every size at most 31 granules, n <= 32768, few granules)
 *   STALLOC_KERNEL_LIST_LDS     list of all placed blocks sorted by address, in LDS
 *   STALLOC_KERNEL_LIST_MEMORY  the same list in the workspace (traces too long for LDS)
 *   STALLOC_KERNEL_LONG_LIST    sorted list of the long-lived blocks in LDS, short-lived blocks in
 *                               a per-plan table ordered by allocation time (long traces in which
 *                               at most an eighth of the requests outlive `lifetime_threshold`)
 * granule_log2: addresses are multiples of 2^granule_log2 bytes (the largest power of two that
 * divides every size); granules: sum of sizes in that unit.  plans_64bit: plans whose extent
 * approached 2^32 granules and that were therefore placed again with 64-bit byte addresses.
 */
typedef enum stalloc_plan_kernel {
    STALLOC_KERNEL_NONE = 0,
    STALLOC_KERNEL_BITMAP = 1,
    STALLOC_KERNEL_LIST_LDS = 2,
    STALLOC_KERNEL_LIST_MEMORY = 3,
    STALLOC_KERNEL_LONG_LIST = 4
} stalloc_plan_kernel;

typedef struct stalloc_plan_info {
    uint32_t kernel;             /* a stalloc_plan_kernel                                        */
    uint32_t granule_log2;
    uint64_t granules;
    uint32_t plans_64bit;
    uint32_t lifetime_threshold; /* STALLOC_KERNEL_LONG_LIST: requests living longer are "long"   */
    uint32_t long_requests;      /* ... and how many there are                                    */
    uint32_t address_bits;       /* width of the addresses the kernel keeps per placed block: 16, 22, 32 (counts of
                                    granules) or 64 (bytes)                                       */
    uint64_t large_size;         /* STALLOC_KERNEL_LONG_LIST: short-lived requests of at least this many bytes are
                                    kept in a table of their own as well (0: none are)            */
    uint32_t large_requests;     /* ... and how many there are                                    */
    uint32_t list_entry_bytes;   /* STALLOC_KERNEL_LONG_LIST: bytes of a block in the sorted list: 16 (address range and
                                    lifetime; two workgroups per CU) or 8 (start address, ranks among the long-lived
                                    requests' allocation and release times in place of the times, size class; three
                                    workgroups per CU); 0 for the other kernels                    */
} stalloc_plan_info;

int stalloc_plan_report(const void *workspace, stalloc_plan_info *info, void *hip_stream);

/*
 * Measurement aid: enqueues one plain kernel that exercises one resource of the chip, so that the
 * rates of the planning kernels can be set against what the device delivers (the caller times it
 * with events on `hip_stream`).
 *   STALLOC_PROBE_COPY      copies the first half of `buffer` to its second half (16-byte words);
 *                           work_done = bytes read + bytes written
 *   STALLOC_PROBE_LDS_READ  2 workgroups of 1024 threads per CU, every thread reads 16 bytes of LDS
 *                           `iters` times; work_done = bytes read from LDS
 *   STALLOC_PROBE_INT_ALU   32 workgroups of 256 threads per CU, 8 independent 32-bit integer
 *                           operations per thread and step, `iters` steps; work_done = lane operations
 * buffer: device memory, 16-byte aligned; the last two kinds write 4 bytes per thread into it
 * (8 KiB resp. 32 KiB per CU).  work_done: HOST memory.
 */
typedef enum stalloc_probe_kind {
    STALLOC_PROBE_COPY = 0,
    STALLOC_PROBE_LDS_READ = 1,
    STALLOC_PROBE_INT_ALU = 2
} stalloc_probe_kind;

int stalloc_probe(uint32_t what, void *buffer, size_t buffer_bytes, uint32_t iters, uint64_t *work_done,
                  void *hip_stream);

/* Human-readable name of a stalloc_status; never NULL.  Host memory, static storage. */
const char *stalloc_status_string(int status);

/* Informational: the largest n for which stalloc_plan keeps 16-byte list entries (32-bit granule
 * counts) of all placed blocks in LDS on the current device; 0 if there is no device. */
uint32_t stalloc_plan_lds_capacity(void);

#ifdef __cplusplus
}
#endif
#endif /* STALLOC_H */
