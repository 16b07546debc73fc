/*
 * rapidgnn.h -- C ABI of the MI355X (gfx950) data path of RapidGNN (arxiv 2505.10806).
 *
 * The library implements the steps of the paper's Algorithm 1 that move data:
 *   line 1     precompute the mini-batches of an epoch with a seeded sampler  -> rg_epoch_schedule, rg_sample_blocks
 *   line 2-3   access frequencies of the precomputed input nodes, TopHot      -> rg_access_histogram[_epoch], rg_build_cache
 *   line 4     VectorPull of the hot rows into the steady cache C_s           -> rg_build_cache (bulk pull), or pulls in order
 *              (and the prefetcher of Section III, Fig. 4)                       of first use ahead of the gathers:
 *                                                                                rg_plan_prefetch + rg_prefetch_planned,
 *                                                                                rg_prefetch_cache_rows
 *   line 12-14 per-batch feature assembly from local store, cache and         -> rg_gather_features
 *              fallback pull of the misses from the remote store
 * and two companions: rg_mean_aggregate (Eq. 1 with AGG = mean over a sampled block, the consumer of the
 * gathered rows) and rg_cache_hit_curve (Section V: remote fetches against cache size).
 * Every step runs in HIP kernels on the device; there is no CPU fallback.
 *
 * Conventions
 *  - "device" pointers are HBM allocations of the ctx's GPU; "host" pointers are ordinary
 *    host memory read during the call; "mapped" pointers are device-accessible memory that
 *    may live in pinned host memory (hipHostMalloc / torch pin_memory) or in HBM.
 *  - All buffers are caller-owned and only borrowed for the call (until the work queued on
 *    the stream has finished).  The library owns nothing but the scratch inside rg_ctx.
 *  - Calls are asynchronous on the given hipStream_t (passed as void*; NULL = the default
 *    stream).  Device-resident outputs are valid once that stream has been synchronised.
 *  - Every call validates its arguments on the host before launching anything and returns
 *    RG_ERR_INVALID_ARG / RG_ERR_CAPACITY without side effects when they are wrong;
 *    rg_last_error() then holds a message.  A remote store that is neither device memory nor
 *    pinned / registered host memory is refused (RG_ERR_INVALID_ARG).  Node ids out of
 *    [0, num_nodes) inside device arrays are a precondition violation and are not checked.
 *  - One rg_ctx serves one host thread.  Calls of the same kind (two samplers, two gathers)
 *    share scratch and must be ordered on the stream(s) they use; calls of different kinds
 *    use disjoint scratch.
 *  - Location word (used by home[] and loc[]): (tag << 30) | row as uint32 stored in int32;
 *    tag 0 = row of the local store, 1 = row (slot) of the cache, 2 = row of the remote store.
 *  - Row strides are in floats.  Rows are copied with 16-byte accesses when every base
 *    pointer is 16-byte aligned and every stride is a multiple of 4 floats; then up to 3 floats
 *    of padding behind a source row are read (they lie inside the row's stride).  Writes
 *    cover exactly floats [0, dim) of a destination row, whatever the access width: the padding
 *    of output, cache and aggregate rows is never touched.
 *  - Launch shapes can be overridden for re-tuning on another device by environment variables
 *    that rg_create reads once per context: RG_GATHER_UNROLL (2, 4 or 8 chunks in flight per
 *    lane of the HBM gather), RG_GATHER_BLOCKS_PER_CU (grid cap of the HBM gather, default
 *    none), RG_PULL_BLOCKS / RG_PULL_THREADS (grid of the host-link pull kernels, default
 *    16 x 1024), RG_PULL_ROWS (rows in flight per lane group of the pull kernel, 4 or 8), RG_MISS_BLOCKS /
 *    RG_MISS_THREADS (grid of the miss-row kernel, default 192 x 256), RG_XCD_MAP=0 (sampler workgroups in
 *    batch-major order instead of one batch of a group per XCD).
 */
#ifndef RAPIDGNN_H
#define RAPIDGNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#ifndef RG_API
#if defined(__GNUC__) || defined(__clang__)
#define RG_API __attribute__((visibility("default")))
#else
#define RG_API
#endif
#endif

typedef enum {
    RG_OK = 0,
    RG_ERR_INVALID_ARG = 1,   /* null pointer, negative size, bad stride, unsupported value */
    RG_ERR_CAPACITY = 2,      /* an output buffer is smaller than the static bound (see rg_blocks_bounds) */
    RG_ERR_OOM = 3,           /* scratch allocation failed */
    RG_ERR_HIP = 4,           /* a HIP runtime call failed; message in rg_last_error */
    RG_ERR_STATE = 5          /* call not valid in the ctx's current state (rg_gather_run on an unprepared ticket) */
} rg_status;

#define RG_TAG_LOCAL 0u
#define RG_TAG_CACHE 1u
#define RG_TAG_REMOTE 2u
#define RG_TAG_SHIFT 30
#define RG_ROW_MASK ((1u << RG_TAG_SHIFT) - 1u)

/* Largest per-hop fan-out drawn with Floyd's algorithm.  RG_FANOUT_ALL takes every neighbour. */
#define RG_MAX_FANOUT 1024
#define RG_FANOUT_ALL (-1)
#define RG_MAX_HOPS 8
/* Most batches one rg_sample_blocks_group call samples side by side. */
#define RG_MAX_GROUP 16

typedef struct rg_ctx rg_ctx;

/* Create / destroy a context bound to HIP device `device`.  rg_destroy synchronises the
 * device and frees the scratch.  rg_last_error returns a ctx-owned string (never freed by
 * the caller; valid until the next failing call); with ctx == NULL it returns the message of
 * the last failed rg_create. */
RG_API rg_status rg_create(int device, rg_ctx** out);
RG_API void rg_destroy(rg_ctx* ctx);
RG_API const char* rg_last_error(const rg_ctx* ctx);
RG_API const char* rg_version(void);

/* Pre-size the scratch so later sampling, histogram, TopHot, plan and gather calls allocate nothing:
 * graphs of up to num_nodes nodes, cumulative frontiers of up to max_frontier nodes, sampler
 * calls of up to sample_group batches (1 for rg_sample_blocks), gathers and per-batch prefetch
 * passes of up to max_rows rows.  Optional: every call grows the scratch on demand (a
 * synchronising allocation).  1 <= sample_group <= RG_MAX_GROUP. */
RG_API rg_status rg_reserve(rg_ctx* ctx, int64_t num_nodes, int64_t max_frontier, int64_t max_rows, int32_t sample_group);

/* CSR adjacency in HBM: row v lists the nodes whose features v aggregates (Eq. 1, eta(v)). */
typedef struct {
    int64_t num_nodes;
    int64_t num_edges;
    const void* row_ptr;      /* device, int32[num_nodes+1] or int64[num_nodes+1] */
    int32_t row_ptr_bits;     /* 32 or 64 */
    const int32_t* col_idx;   /* device, int32[num_edges] */
} rg_csr;

/* ---- Alg. 1 line 1, the epoch's batch order -------------------------------------------
 * order_out = train_ids sorted ascending by (key64(v), v), key64(v) = first two words of the
 * Philox4x32-10 block with counter (v, 0xFFFFFFFF, 0, epoch) and key (seed lo, seed hi).
 * Batches are consecutive chunks of the order; the partial last chunk is a batch
 * (Section II-E counts ceil(n/B) batches).
 * train_ids: device int32[n] (distinct ids); order_out: device int32[n]; n >= 0. */
RG_API rg_status rg_epoch_schedule(rg_ctx* ctx, const int32_t* train_ids, int64_t n, uint64_t seed,
                            uint32_t epoch, int32_t* order_out, void* stream);

/* ---- Alg. 1 line 1, one precomputed mini-batch b_i^e ------------------------------------
 * Node-wise neighbour sampling SAMPLE(eta(v), k) (Section II-B) over num_hops hops.
 *   frontier_0 = seeds (given order).  For hop h: every node v of frontier_h draws
 *   m = min(fanouts[h], deg v) distinct neighbours (all of them, in row order, when
 *   deg v <= fanouts[h] or fanouts[h] == RG_FANOUT_ALL; otherwise Floyd's subset algorithm on
 *   row positions, draw i = word i&3 of the Philox4x32-10 block with counter
 *   (v, h, i>>2, epoch) and key (seed lo, seed hi), bounded by the high word of draw*(j+1));
 *   indptr[h] = exclusive prefix sum of m in frontier order; nbr[h] = neighbours in frontier
 *   order, per node in insertion order; tier_{h+1} = ids in nbr[h] not in frontier_h, unique,
 *   ascending; frontier_{h+1} = frontier_h ++ tier_{h+1}; nbr_local[h][e] = position of
 *   nbr[h][e] in frontier_{h+1}.  nodes = frontier_H is the batch's input-node list N_i^e;
 *   tier_off[t] = start of tier t in nodes (tier 0 = seeds), tier_off[num_hops+1] = |N_i^e|.
 * The result depends only on (graph, seeds, fanouts, seed, epoch): bit-reproducible.
 */
typedef struct {
    int32_t* nodes;            /* device int32[nodes_cap] */
    int64_t nodes_cap;         /* in; on RG_ERR_CAPACITY out: the required size */
    int32_t* tier_off;         /* device int32[num_hops + 2] */
    int32_t* const* indptr;    /* host array[num_hops] of device int32[indptr_cap[h]] */
    int64_t* indptr_cap;       /* host int64[num_hops]; in, on RG_ERR_CAPACITY out: the required sizes */
    int32_t* const* nbr;       /* host array[num_hops] of device int32[nbr_cap[h]] */
    int32_t* const* nbr_local; /* host array[num_hops] of device int32[nbr_cap[h]], or NULL to skip relabelling */
    int64_t* nbr_cap;          /* host int64[num_hops]; in, on RG_ERR_CAPACITY out: the required sizes */
    int32_t* num_edges;        /* device int32[num_hops] or NULL: |nbr[h]| (the same value as indptr[h][|frontier_h|]) */
} rg_blocks;

/* Static bounds the output buffers of rg_sample_blocks must meet:
 *   frontier_ub[0] = min(N, B);
 *   edges_ub[h]    (h = 0..num_hops-1) bounds |nbr[h]|:     min(nnz, frontier_ub[h] * F_h), nnz for RG_FANOUT_ALL;
 *   frontier_ub[h+1] bounds |frontier_{h+1}|:                min(N, frontier_ub[h] + edges_ub[h])
 *                                                            (<= min(N, B * prod_{t<=h} (1+F_t))).
 * Required: nodes_cap >= frontier_ub[num_hops], indptr_cap[h] >= frontier_ub[h] + 1,
 * nbr_cap[h] >= edges_ub[h].  Host arrays, written by the call. */
RG_API rg_status rg_blocks_bounds(int64_t num_nodes, int64_t num_edges, int64_t num_seeds,
                           const int32_t* fanouts, int32_t num_hops,
                           int64_t* frontier_ub, int64_t* edges_ub);

/* seeds: device int32[num_seeds], distinct, num_seeds >= 0; fanouts: host int32[num_hops],
 * each in [0, RG_MAX_FANOUT] or RG_FANOUT_ALL; 1 <= num_hops <= RG_MAX_HOPS.
 * Errors: RG_ERR_INVALID_ARG; RG_ERR_OOM; RG_ERR_CAPACITY when a buffer is below its bound: nothing
 * is launched and nodes_cap, indptr_cap[h] and nbr_cap[h] of the offending rg_blocks are overwritten
 * with the required sizes (the values rg_blocks_bounds gives), so the caller can reallocate and retry. */
RG_API rg_status rg_sample_blocks(rg_ctx* ctx, const rg_csr* csr, const int32_t* seeds, int32_t num_seeds,
                           const int32_t* fanouts, int32_t num_hops, uint64_t seed, uint32_t epoch,
                           rg_blocks* out, void* stream);

/* The same for `group` batches at once (1 <= group <= RG_MAX_GROUP): batch g has seeds[g]
 * (num_seeds[g] of them) and writes out[g]; fan-outs, seed and epoch are shared.  The results are
 * exactly those of `group` separate calls; the kernels of a hop take all the batches in one launch
 * (most per-batch kernels are far smaller than the device).  seeds: host array[group] of device
 * pointers; num_seeds: host int32[group]; out: host array[group].
 * node_order chooses the order of the nodes inside a new tier (Section IV: the precomputed batches
 * fix "the order of the input nodes"; the paper leaves the order itself open):
 *   RG_ORDER_ASCENDING   ascending by id (what rg_sample_blocks produces);
 *   RG_ORDER_FIRST_SEEN  the order in which nbr[h] (frontier order, per node in insertion order) first
 *                        names them: the order a block-building pass over the sampled edges produces.
 * Which nodes a tier holds and what every node draws do not depend on the order; nodes, nbr_local
 * and the order of the rows of later hops do.  rg_access_histogram_epoch needs ascending tiers. */
#define RG_ORDER_ASCENDING 0
#define RG_ORDER_FIRST_SEEN 1
RG_API rg_status rg_sample_blocks_group(rg_ctx* ctx, const rg_csr* csr, int32_t group, const int32_t* const* seeds,
                                        const int32_t* num_seeds, const int32_t* fanouts, int32_t num_hops,
                                        uint64_t seed, uint32_t epoch, int32_t node_order, rg_blocks* out, void* stream);

/* ---- Alg. 1 line 2 / Section IV: access frequency freq(n) -------------------------------
 * counts[v] += number of occurrences of v in nodes[0..n).  counts accumulates over calls
 * (the caller zeroes it to start a new period) and covers every node; the remote filter is
 * applied by rg_build_cache.
 * nodes: device int32[>= n]; counts: device uint32[num_nodes].
 * n_dev: optional device int32* holding the actual entry count (e.g. tier_off + num_hops + 1
 * of a batch sampled on the same stream); when non-NULL, n is only an upper bound used to
 * size the launch and min(n, *n_dev) entries are read. */
RG_API rg_status rg_access_histogram(rg_ctx* ctx, const int32_t* nodes, int64_t n, const int32_t* n_dev,
                              uint32_t* counts, int64_t num_nodes, void* stream);

/* The same histogram over a whole precomputed epoch in one call: batch b's input nodes are
 * nodes[b * batch_stride .. + tier_off[b][num_hops + 1]), with tier_off[b] the num_hops + 2 tier
 * offsets rg_sample_blocks wrote for that batch.  Equivalent to one rg_access_histogram call per
 * batch, but ids that recur across batches are accumulated in LDS-private counters: each workgroup
 * owns an id range, finds its entries in every ascending tier by binary search and adds the range to
 * counts once.  Precondition: tiers 1..num_hops of every batch are ascending by id (as produced by
 * rg_sample_blocks); tier 0 (at most max_seeds seeds per batch) may be in any order.
 * With first_batch != NULL the same pass also records when each node is first needed:
 * first_batch[v] = min(first_batch[v], smallest b whose list contains v); the caller sets the array
 * to 0xFFFFFFFF beforehand (input of rg_plan_prefetch).
 * nodes: device int32; tier_off: device int32[num_batches * (num_hops + 2)]; counts: device
 * uint32[num_nodes], accumulated; first_batch: device uint32[num_nodes] or NULL;
 * 0 <= num_batches <= 65535. */
RG_API rg_status rg_access_histogram_epoch(rg_ctx* ctx, const int32_t* nodes, int64_t batch_stride,
                                           const int32_t* tier_off, int32_t num_batches, int32_t num_hops,
                                           int32_t max_seeds, uint32_t* counts, uint32_t* first_batch,
                                           int64_t num_nodes, void* stream);

/* The same counts without reading any id list (Section IV, offline stage: frequencies are taken as
 * the batches are precomputed): adds the input-node sets of the `group` batches that the last
 * rg_sample_blocks / rg_sample_blocks_group call of this context sampled, straight from the
 * sampler's membership bitmaps: counts[v] += number of those batches whose input nodes contain v.
 * Works for either node order.  With first_batch != NULL, first_batch[v] = min(first_batch[v],
 * smallest batch_index[g] over those batches), as rg_access_histogram_epoch records it.
 * Must follow that sampling call on the same stream, before the context samples again; group and
 * num_nodes must match it (RG_ERR_STATE otherwise).  batch_index: host int32[group], the batches'
 * indices within the period (may be NULL when first_batch is NULL). */
RG_API rg_status rg_access_histogram_sampled(rg_ctx* ctx, int32_t group, const int32_t* batch_index, uint32_t* counts,
                                             uint32_t* first_batch, int64_t num_nodes, void* stream);

/* ---- Alg. 1 lines 3-4: TopHot + VectorPull -----------------------------------------------
 * Candidates = nodes whose home word is remote and whose count >= 1, ranked by
 * (count descending, id ascending).  K_eff = min(capacity_rows, #candidates) are selected;
 * cache_ids = selected ids ascending, slot = rank in that order; loc[v] = cache word for the
 * selected nodes and home[v] for all others; *num_cached = K_eff.
 * With remote_store != NULL the rows are pulled at once: cache_rows[slot] = remote_store row of
 * the node (one bulk pull over the host link) and, if `filled` is given, every selected slot is
 * marked resident.  With remote_store == NULL only the selection is made and `filled` (required
 * then) is cleared: rows are pulled later, batch by batch, by rg_prefetch_cache_rows.
 * (A mirrored cache, see rg_cache.mirror_rows, is select-only and keeps `filled`.)
 */
typedef struct {
    int32_t* cache_ids;       /* device int32[capacity_rows] */
    float* cache_rows;        /* device float[capacity_rows * row_stride] */
    int64_t capacity_rows;    /* >= 0 */
    int64_t row_stride;       /* floats, >= dim */
    int32_t* loc;             /* device int32[num_nodes] location words */
    int64_t* num_cached;      /* device int64[1], written by rg_build_cache */
    uint32_t* filled;         /* device uint32[ceil(min(capacity_rows, num_nodes) / 32)] or NULL: bit s set = row of slot s is resident */
    /* Mirrored layout, for a cache that can hold the whole remote partition (capacity_rows >= number of rows of the
     * remote store).  Every remote row a batch names will be selected then, so where it goes can be fixed before
     * TopHot has run: mirror_rows = number of rows of the remote store (0 = the layout above) puts the row of a
     * cached node at cache_rows[its remote-store row] instead of cache_rows[its slot]; cache_ids, loc, num_cached
     * and the statistics keep their meaning.  `filled` is then indexed by remote-store row; rg_build_cache (select
     * only) leaves it alone, so rows pulled while the batches were still being sampled, or in an earlier period,
     * stay valid: the caller clears it to start cold.  rg_prefetch_cache_rows pulls the not-yet-resident remote rows
     * a batch names and needs no TopHot result; rg_plan_sampled + rg_prefetch_planned do the same per sampler
     * group from the sampler's bitmaps; rg_plan_prefetch does not apply.  home: the home words
     * (device int32[num_nodes]), required when mirror_rows > 0. */
    int64_t mirror_rows;
    const int32_t* home;
} rg_cache;

/* counts: device uint32[num_nodes]; home: device int32[num_nodes] (never modified);
 * remote_store: mapped float[n_remote * remote_stride] or NULL (select only); dim >= 1. */
RG_API rg_status rg_build_cache(rg_ctx* ctx, const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                         const float* remote_store, int64_t remote_stride, int32_t dim,
                         const rg_cache* cache, void* stream);

/* ---- remote fetches against cache size (the relation of Section V, "impact of cache size on
 * remote-fetch volume") without building any cache: for each capacity K_j,
 *   hits[j] = sum of the counts of the K_j best candidates in TopHot order
 * = the number of row requests a cache of that capacity serves over the period the counts cover
 * (ties at the threshold all have the threshold's count, so the sum does not depend on the
 * tie-break); *remote_total = sum of the counts of all candidates = all requests for remote
 * rows.  Remote fetches = remote_total - hits[j]; hit % = hits[j] / remote_total.
 * capacities: host int64[num_capacities], each >= 0; hits: device uint64[num_capacities];
 * remote_total: device uint64[1] or NULL. */
RG_API rg_status rg_cache_hit_curve(rg_ctx* ctx, const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                                    const int64_t* capacities, int32_t num_capacities, uint64_t* hits,
                                    uint64_t* remote_total, void* stream);

/* ---- prefetcher (Section III: features of upcoming batches are prepared ahead of their use) ----
 * Pulls, over the host link, the rows of those cached nodes among input_nodes[0..n) whose slot is
 * not yet resident, and marks them resident.  Called batch by batch ahead of rg_gather_features
 * (typically on its own stream, with an event per batch), it fills the cache in order of first
 * use, so the transfer of later rows overlaps the gathers of earlier batches; over an epoch every
 * selected row is pulled exactly once, the same traffic as the bulk pull.
 * Calls on one cache must be ordered with each other and with rg_build_cache; a gather may only
 * read a batch after the prefetch of that batch has completed.
 * input_nodes: device int32[>= n]; n_dev as for rg_access_histogram; cache->filled required. */
RG_API rg_status rg_prefetch_cache_rows(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                                        const rg_cache* cache, const int32_t* home,
                                        const float* remote_store, int64_t remote_stride, int32_t dim,
                                        void* stream);

/* ---- planned prefetch: the same pulls as rg_prefetch_cache_rows without a pass over each batch ----
 * The precomputed schedule says in which batch every selected node is first needed
 * (rg_access_histogram_epoch's first_batch).  rg_plan_prefetch groups the selected slots by that
 * batch once per epoch: list[offsets[b] .. offsets[b+1]) holds the (slot, remote row) pairs first
 * needed by batch b, b = 0..num_batches-1; segment num_batches holds the slots no planned batch
 * uses.  rg_prefetch_planned(b) pulls segment b over the host link and marks its slots resident.
 * Pulled in batch order ahead of the gathers (one event per batch), every selected row arrives
 * exactly once and before its first use, and the prefetch stream carries nothing but pulls.
 * With at most 1023 batches every segment lists its slots in ascending order (ascending remote rows,
 * which the host link serves faster than scattered ones); beyond that the order inside a segment is
 * unspecified. */
typedef struct {
    int32_t* list;            /* device int32[2 * list_capacity] */
    int64_t list_capacity;    /* pairs; >= min(cache capacity_rows, num_nodes) */
    int32_t* offsets;         /* device int32[num_batches + 2] */
    int32_t num_batches;      /* 0..65535 */
} rg_prefetch_plan;

/* With a mirrored cache (rg_cache.mirror_rows) a plan can also be grown while the period is being sampled, one segment
 * per sampler call, by rg_plan_sampled below; rg_prefetch_planned then pulls segment by segment as for a planned period. */
/* after rg_build_cache (select only) on the same stream; first_batch: device uint32[num_nodes]. */
RG_API rg_status rg_plan_prefetch(rg_ctx* ctx, const rg_cache* cache, const int32_t* home, const uint32_t* first_batch,
                                  int64_t num_nodes, const rg_prefetch_plan* plan, void* stream);
/* 0 <= batch <= plan->num_batches. */
RG_API rg_status rg_prefetch_planned(rg_ctx* ctx, const rg_prefetch_plan* plan, int32_t batch, const rg_cache* cache,
                                     const float* remote_store, int64_t remote_stride, int32_t dim, void* stream);

/* ---- the prefetcher's row lists straight from the sampler (Section III, prefetcher; Alg. 1 line 4, VectorPull:
 * the rows go over the link in a few vectorised pulls instead of one request per row) ----
 * Mirrored cache only: appends segment `segment` to the plan = the remote rows that the group of batches sampled
 * last on this context (rg_sample_blocks / rg_sample_blocks_group) is the first to name, as (row, row) pairs in
 * ascending row order, read off the sampler's membership bitmaps (no pass over the batches' id lists).
 * `claimed` (device uint32[ceil(num_nodes / 32)]) holds every node an earlier call has named; the call adds the
 * group's; the caller zeroes it to start cold, or keeps it to keep the rows of earlier periods.  Segments are
 * appended in order: the caller sets offsets[0] = 0 at the start of a period, the call reads offsets[segment] and
 * writes offsets[segment + 1]; calls on one plan / bitmap are ordered by the caller (one stream).  It must follow the
 * sampling call before the context samples again; group and num_nodes must match it (RG_ERR_STATE otherwise).
 * plan->list_capacity >= cache->mirror_rows, 0 <= segment < plan->num_batches. */
RG_API rg_status rg_plan_sampled(rg_ctx* ctx, int32_t group, const rg_cache* cache, uint32_t* claimed,
                                 const rg_prefetch_plan* plan, int32_t segment, int64_t num_nodes, void* stream);

/* ---- Alg. 1 lines 12-14: feature assembly for one batch ---------------------------------
 * out[i][0:dim] = feature row of input_nodes[i], read from the store loc[] names: local
 * store (HBM), cache (HBM, GetFeatureFromCache) or remote store (fallback pull of the
 * misses only).  stats = {#local rows, #cache hits, #misses}.
 * Rows served from HBM are copied on hit_stream; the miss rows are copied on miss_stream
 * concurrently (if it differs from hit_stream) and joined back: when the call returns, all
 * work is ordered before anything queued later on hit_stream.
 * input_nodes: device int32[>= n]; n_dev: as for rg_access_histogram; out: device
 * float[n * out_stride]; stats: device int64[3]. */
typedef struct { int64_t n_local, n_hit, n_miss; } rg_gather_stats;

RG_API rg_status rg_gather_features(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                             const rg_cache* cache,
                             const float* local_store, int64_t local_stride,
                             const float* remote_store, int64_t remote_stride,
                             int32_t dim, float* out, int64_t out_stride,
                             rg_gather_stats* stats, void* hit_stream, void* miss_stream);

/* The same assembly in two steps.  rg_gather_prepare resolves, for `count` batches in one launch,
 * every output row to its source (one lookup of loc[] per row), counts the three classes into
 * stats[k] and lists the miss rows, into the ctx's scratch entries ("tickets") first_ticket ..
 * first_ticket + count - 1; rg_gather_run copies the rows of one prepared ticket (HBM rows on
 * hit_stream, miss rows on miss_stream, joined as in rg_gather_features).  Preparing several batches
 * at once pays the lookup launch once per group and leaves one copy kernel per batch on the stream.
 * rg_gather_features = prepare (ticket 0, one batch) + run.  A ticket is busy from its prepare until
 * the work of its run has finished; prepare and run of a ticket are given the same n, n_dev and
 * cache and are ordered on their streams by the caller (trivially so on one stream).
 * rg_gather_run returns RG_ERR_STATE if the ticket was not prepared for n rows.
 * input_nodes, n_dev, stats: host arrays[count] of device pointers (n_dev may be NULL, or hold
 * NULLs); n: host int64[count]; 0 <= first_ticket, first_ticket + count <= RG_GATHER_TICKETS. */
#define RG_GATHER_TICKETS 8
RG_API rg_status rg_gather_prepare(rg_ctx* ctx, int32_t first_ticket, int32_t count, const int32_t* const* input_nodes,
                                   const int64_t* n, const int32_t* const* n_dev, const rg_cache* cache,
                                   rg_gather_stats* const* stats, void* stream);
RG_API rg_status rg_gather_run(rg_ctx* ctx, int32_t ticket, int64_t n, const int32_t* n_dev, const rg_cache* cache,
                               const float* local_store, int64_t local_stride,
                               const float* remote_store, int64_t remote_stride,
                               int32_t dim, float* out, int64_t out_stride, void* hit_stream, void* miss_stream);

/* One half of rg_gather_run on one stream, with no fork or join: part = RG_GATHER_PART_HBM copies the rows served
 * from the local store and the cache, RG_GATHER_PART_MISS the miss rows (Section III: the fallback pulls of a batch
 * overlap other work).  A caller that runs the miss halves of consecutive batches on a stream of their own keeps the
 * host link busy from one batch to the next instead of forking and joining per batch; it orders the streams itself:
 * both halves after the ticket's rg_gather_prepare, the batch complete when both are done, and a reused output buffer
 * free of the earlier batch's halves.  Arguments as for rg_gather_run. */
#define RG_GATHER_PART_HBM 1
#define RG_GATHER_PART_MISS 2
RG_API rg_status rg_gather_run_part(rg_ctx* ctx, int32_t ticket, int32_t part, int64_t n, const int32_t* n_dev,
                                    const rg_cache* cache, const float* local_store, int64_t local_stride,
                                    const float* remote_store, int64_t remote_stride, int32_t dim, float* out,
                                    int64_t out_stride, void* stream);

/* ---- feature assembly for callers that cannot allocate -----------------------------------
 * The same result as rg_gather_features (same arguments, same stream semantics), for callers
 * that must not trigger a device allocation: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The per-row lookup results and the miss list go to a
 * file-scope device array inside the library instead of the context's growable scratch, so the
 * call never calls hipMalloc / hipFree, whatever n was in earlier calls.  The array holds
 * RG_STATIC_GATHER_MAX_ROWS rows (12 B per row, about 12.6 MB, resident on every GPU the
 * library has run on until the process ends); n above that returns RG_ERR_CAPACITY and queues
 * nothing.  Every call on one GPU, from any context, shares that GPU's array: calls that
 * overlap in time on one GPU race, so the caller orders them (one stream, or events).  The
 * kernels are not bracketed for rg_profile_read. */
#define RG_STATIC_GATHER_MAX_ROWS (1 << 20)
RG_API rg_status rg_gather_features_static(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                                           const rg_cache* cache,
                                           const float* local_store, int64_t local_stride,
                                           const float* remote_store, int64_t remote_stride,
                                           int32_t dim, float* out, int64_t out_stride,
                                           rg_gather_stats* stats, void* hit_stream, void* miss_stream);

/* ---- consumer of the gathered rows: Eq. 1 with AGG = mean (GraphSAGE, Section II-A) -------------
 * For the block of one hop (destination i = position in frontier_h, sources = positions in
 * frontier_{h+1} given by nbr_local[h]):
 *   agg[i][0:dim] = (1 / m_i) * sum_{e = indptr[i]}^{indptr[i+1]-1} feat[nbr_local[e]][0:dim],
 *   m_i = indptr[i+1] - indptr[i]; a destination without sampled neighbours gets a zero row.
 * The sum is accumulated in fp32 in edge order and divided by m_i (IEEE division).
 * For the outermost hop, feat is the output of rg_gather_features (rows in input-node order).
 * indptr: device int32[n_dst + 1]; nbr_local: device int32[indptr[n_dst]]; n_dst_dev: optional
 * device count as for rg_access_histogram; feat: device float[rows * feat_stride]; agg: device
 * float[n_dst * agg_stride].  Only floats [0, dim) of an agg row are written. */
RG_API rg_status rg_mean_aggregate(rg_ctx* ctx, const int32_t* indptr, const int32_t* nbr_local, int64_t n_dst,
                                   const int32_t* n_dst_dev, const float* feat, int64_t feat_stride, int32_t dim,
                                   float* agg, int64_t agg_stride, void* stream);

/* ---- kernel timing for the benchmark ------------------------------------------------------
 * With profiling on, every launch of the listed kernels is bracketed by hipEvents on its own
 * stream.  rg_profile_read synchronises the recorded events and returns the summed duration
 * and launch count since the last rg_profile_reset. */
typedef enum {
    RG_K_GATHER_HBM = 0,   /* rows served from the local store and the cache */
    RG_K_GATHER_MISS = 1,  /* rows pulled from the remote store */
    RG_K_SAMPLE = 2,       /* per-hop draw + neighbour read kernel */
    RG_K_HISTOGRAM = 3,
    RG_K_CACHE_FILL = 4,   /* bulk pull and per-batch prefetch pulls */
    RG_K_AGGREGATE = 5,
    RG_K_COUNT_
} rg_kernel_id;

RG_API rg_status rg_profile_enable(rg_ctx* ctx, int on);
/* Brackets only the kernels whose bit (1u << rg_kernel_id) is set in kernel_mask (default: all).  Two event
 * records per launch on every stream shift what runs beside what; a pass that brackets one kernel alone times
 * that kernel closest to an unbracketed run. */
RG_API rg_status rg_profile_select(rg_ctx* ctx, uint32_t kernel_mask);
RG_API rg_status rg_profile_reset(rg_ctx* ctx);
RG_API rg_status rg_profile_read(rg_ctx* ctx, int kernel_id, double* total_ms, int64_t* launches);

/* ---- streams bound to a share of the compute units ----------------------------------------
 * A HIP stream whose kernels are placed only on compute units [first_cu, first_cu + num_cus) of
 * the device's enumeration (the runtime's compute-unit mask; how the enumeration maps to XCDs is
 * the driver's business).  Kernels that pull rows over the host link keep their few wavefronts
 * waiting on the link; giving their stream a few compute units of its own, and every other stream
 * the rest, keeps other kernels' wavefronts from sharing, and stalling behind, those units.
 * The stream synchronises with the NULL stream like any stream created without
 * hipStreamNonBlocking.  rg_stream_destroy waits for the stream's work, then destroys it; rg_destroy
 * does the same for the streams still alive, so none may be used after its context is gone. */
RG_API rg_status rg_stream_create(rg_ctx* ctx, int32_t first_cu, int32_t num_cus, void** stream);
RG_API rg_status rg_stream_destroy(rg_ctx* ctx, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RAPIDGNN_H */
