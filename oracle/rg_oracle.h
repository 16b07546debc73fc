/*
 * CPU oracle for the RapidGNN data path -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, single-threaded C implementation of what the hot path computes,
 * written from the paper (Algorithm 1, Eq. 3, Sections III-IV) and from the published
 * definition of Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel Random Numbers:
 * As Easy as 1, 2, 3", SC'11).  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP library.
 *
 * Location words (an interface format, identical to the library's):
 *   word = (tag << 30) | row, tag 0 = local store, 1 = cache, 2 = remote store.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors; Floyd subset uniformity
 * and inclusion probability k/d; every sampled neighbour is a real edge; count =
 * min(fanout, degree); BFS-ball special case against a textbook BFS (first-seen order: against the
 * visiting order of a queue BFS); histogram against
 * numpy bincount; top-K against a full lexicographic sort; gather against plain
 * indexing; the hit-rate closed form; the paper's byte-accounting example; the mean aggregation
 * against a float64 sparse matrix product (scipy).
 * Statistical fidelity of the synthetic graphs to the paper's datasets: parity unpinned.
 */
#ifndef RG_ORACLE_H
#define RG_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Philox4x32-10 block function (SC'11 paper, Section 3.3 / Table 2 constants). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Draw i of the stream keyed by (seed, epoch, node, hop): word (i & 3) of the block
 * with counter (node, hop, i >> 2, epoch) and key (seed low word, seed high word). */
uint32_t orc_draw(uint64_t seed, uint32_t epoch, uint32_t node, uint32_t hop, uint64_t i);

/* SAMPLE(eta(v), k) of Section II-B on positions 0..d-1 of v's adjacency row: uniform,
 * without replacement.  d <= k (or k < 0, "all neighbours"): positions 0..d-1 in row
 * order.  Otherwise Floyd's subset algorithm driven by orc_draw, positions reported in
 * insertion order.  Returns the number of positions written (min(k, d)). */
int64_t orc_sample_positions(uint64_t seed, uint32_t epoch, uint32_t node, uint32_t hop,
                             int64_t d, int64_t k, int64_t* pos);

/* Epoch order of the training ids (the per-epoch reshuffle behind Alg. 1 line 1): ids
 * sorted ascending by (key64(v), v), key64 = first two words of the Philox block with
 * counter (v, 0xFFFFFFFF, 0, epoch). */
void orc_epoch_schedule(const int32_t* train_ids, int64_t n, uint64_t seed, uint32_t epoch,
                        int32_t* order_out);

/* One precomputed mini-batch b_i^e (Alg. 1 line 1): multi-hop node-wise sampling. */
typedef struct orc_blocks orc_blocks;
orc_blocks* orc_sample_blocks(int64_t num_nodes, const int64_t* row_ptr, const int32_t* col_idx,
                              const int32_t* seeds, int64_t num_seeds,
                              const int32_t* fanouts, int32_t num_hops,
                              uint64_t seed, uint32_t epoch);
/* The same with a choice of the order of the nodes inside a new tier (Section IV: the precomputed batches fix "the
 * order of the input nodes"): ORC_ORDER_ASCENDING = ascending by id; ORC_ORDER_FIRST_SEEN = the order in which the
 * hop's neighbour list (frontier order, per node in insertion order) first names them, the order a block-building
 * pass over the sampled edges produces.  Which nodes a tier holds, and what every node draws, is the same. */
#define ORC_ORDER_ASCENDING 0
#define ORC_ORDER_FIRST_SEEN 1
orc_blocks* orc_sample_blocks_ordered(int64_t num_nodes, const int64_t* row_ptr, const int32_t* col_idx,
                                      const int32_t* seeds, int64_t num_seeds,
                                      const int32_t* fanouts, int32_t num_hops,
                                      uint64_t seed, uint32_t epoch, int32_t node_order);
void orc_blocks_free(orc_blocks* b);
int32_t orc_blocks_num_hops(const orc_blocks* b);
const int64_t* orc_blocks_tier_off(const orc_blocks* b);      /* [num_hops + 2] */
const int32_t* orc_blocks_nodes(const orc_blocks* b);         /* [tier_off[num_hops+1]] = N_i^e */
int64_t orc_blocks_num_edges(const orc_blocks* b, int32_t hop);
const int64_t* orc_blocks_indptr(const orc_blocks* b, int32_t hop);    /* [tier_off[hop+1] + 1] */
const int32_t* orc_blocks_nbr(const orc_blocks* b, int32_t hop);       /* global ids */
const int32_t* orc_blocks_nbr_local(const orc_blocks* b, int32_t hop); /* positions in nodes */

/* freq(n) of Section IV: counts[v] += number of occurrences of v in nodes[0..n). */
void orc_access_histogram(const int32_t* nodes, int64_t n, uint32_t* counts, int64_t num_nodes);

/* TopHot (Alg. 1 line 3): among nodes whose home is remote and whose count is >= 1,
 * the capacity_rows largest counts, ties to the lower id.  cache_ids is ascending by
 * id, slot = rank; loc[v] = cache word for selected nodes, home[v] otherwise.
 * Returns the number of cached nodes. */
int64_t orc_build_cache(const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                        int64_t capacity_rows, int32_t* cache_ids, int32_t* loc);

/* VectorPull (Alg. 1 line 4): cache_rows[slot] = X[cache_ids[slot]]. */
void orc_fill_cache(const float* X, int64_t dim, const int32_t* cache_ids, int64_t num_cached,
                    float* cache_rows, int64_t row_stride);

/* Feature assembly for one batch (Alg. 1 lines 12-14): out[i] = X[input_nodes[i]];
 * stats = {#local, #cache hits, #remote misses} according to loc. */
void orc_gather_features(const float* X, int64_t dim, const int32_t* input_nodes, int64_t n,
                         const int32_t* loc, float* out, int64_t out_stride, int64_t stats[3]);

/* Requests served by a cache of each capacity (Section V, remote fetches against cache size):
 * hits[j] = sum of the counts of the first capacities[j] candidates in TopHot order; returns the sum over
 * all candidates. */
uint64_t orc_cache_hit_curve(const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                             const int64_t* capacities, int64_t num_capacities, uint64_t* hits);

/* Eq. 1 with AGG = mean (GraphSAGE, Section II-A) over one sampled block, in fp64:
 * agg[i] = (1/m_i) sum_{e in [indptr[i], indptr[i+1])} feat[nbr_local[e]], zero row when m_i = 0. */
void orc_mean_aggregate(const int64_t* indptr, const int32_t* nbr_local, int64_t n_dst,
                        const float* feat, int64_t feat_stride, int64_t dim, double* agg);

#ifdef __cplusplus
}
#endif
#endif
