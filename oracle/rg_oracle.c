/*
 * CPU oracle for the RapidGNN data path -- TEST INFRASTRUCTURE, not a product path.
 * See rg_oracle.h for scope, citations and pins.  Plain C, single thread, no blocking,
 * no fusion: each function is the definition (or the algorithm's steps) written out.
 */
#include "rg_oracle.h"

#include <stdlib.h>
#include <string.h>

#define ORC_TAG_SHIFT 30
#define ORC_TAG_LOCAL 0u
#define ORC_TAG_CACHE 1u
#define ORC_TAG_REMOTE 2u
#define ORC_ROW_MASK ((1u << ORC_TAG_SHIFT) - 1u)

/* ---- Philox4x32-10 (SC'11, Section 3.3): 10 rounds, key bumped by the Weyl constants. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t orc_draw(uint64_t seed, uint32_t epoch, uint32_t node, uint32_t hop, uint64_t i) {
    uint32_t ctr[4] = { node, hop, (uint32_t)(i >> 2), epoch };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[i & 3];
}

/* ---- SAMPLE(eta(v), k), Section II-B: Floyd's algorithm for a uniform k-subset of
 * {0..d-1}.  Step i considers j = d-k+i, draws t uniform in [0, j] (high word of
 * draw * (j+1)), and inserts t unless it is already present, in which case it inserts j. */
int64_t orc_sample_positions(uint64_t seed, uint32_t epoch, uint32_t node, uint32_t hop,
                             int64_t d, int64_t k, int64_t* pos) {
    if (k < 0 || d <= k) {
        for (int64_t t = 0; t < d; ++t) pos[t] = t;
        return d;
    }
    for (int64_t i = 0; i < k; ++i) {
        int64_t j = d - k + i;
        uint64_t r = orc_draw(seed, epoch, node, hop, (uint64_t)i);
        int64_t t = (int64_t)((r * (uint64_t)(j + 1)) >> 32);
        int present = 0;
        for (int64_t l = 0; l < i; ++l)
            if (pos[l] == t) present = 1;
        pos[i] = present ? j : t;
    }
    return k;
}

/* ---- epoch schedule */
typedef struct { uint64_t key; int32_t id; } orc_keyed;

static int orc_keyed_cmp(const void* a, const void* b) {
    const orc_keyed* x = (const orc_keyed*)a;
    const orc_keyed* y = (const orc_keyed*)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

void orc_epoch_schedule(const int32_t* train_ids, int64_t n, uint64_t seed, uint32_t epoch,
                        int32_t* order_out) {
    orc_keyed* a = (orc_keyed*)malloc((size_t)(n > 0 ? n : 1) * sizeof(orc_keyed));
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    for (int64_t i = 0; i < n; ++i) {
        uint32_t ctr[4] = { (uint32_t)train_ids[i], 0xFFFFFFFFu, 0u, epoch };
        uint32_t w[4];
        orc_philox4x32_10(ctr, key, w);
        a[i].key = ((uint64_t)w[0] << 32) | (uint64_t)w[1];
        a[i].id = train_ids[i];
    }
    qsort(a, (size_t)n, sizeof(orc_keyed), orc_keyed_cmp);
    for (int64_t i = 0; i < n; ++i) order_out[i] = a[i].id;
    free(a);
}

/* ---- multi-hop blocks */
struct orc_blocks {
    int32_t num_hops;
    int64_t* tier_off;     /* [H+2] */
    int32_t* nodes;        /* cumulative frontier, seeds first, then one ascending tier per hop */
    int64_t* num_edges;    /* [H] */
    int64_t** indptr;      /* [H][n_h + 1] */
    int32_t** nbr;         /* [H][E_h] */
    int32_t** nbr_local;   /* [H][E_h] */
};

static int orc_i32_cmp(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

orc_blocks* orc_sample_blocks_ordered(int64_t num_nodes, const int64_t* row_ptr, const int32_t* col_idx,
                                      const int32_t* seeds, int64_t num_seeds,
                                      const int32_t* fanouts, int32_t num_hops,
                                      uint64_t seed, uint32_t epoch, int32_t node_order) {
    orc_blocks* b = (orc_blocks*)calloc(1, sizeof(orc_blocks));
    b->num_hops = num_hops;
    b->tier_off = (int64_t*)calloc((size_t)num_hops + 2, sizeof(int64_t));
    b->num_edges = (int64_t*)calloc((size_t)num_hops + 1, sizeof(int64_t));
    b->indptr = (int64_t**)calloc((size_t)num_hops + 1, sizeof(int64_t*));
    b->nbr = (int32_t**)calloc((size_t)num_hops + 1, sizeof(int32_t*));
    b->nbr_local = (int32_t**)calloc((size_t)num_hops + 1, sizeof(int32_t*));

    /* position of a node in the cumulative frontier, -1 = not a member */
    int64_t* where = (int64_t*)malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof(int64_t));
    for (int64_t v = 0; v < num_nodes; ++v) where[v] = -1;

    int64_t cap = num_seeds > 16 ? num_seeds : 16;
    int32_t* nodes = (int32_t*)malloc((size_t)cap * sizeof(int32_t));
    int64_t n = 0;
    for (int64_t i = 0; i < num_seeds; ++i) {          /* frontier_0 = seeds, given order */
        nodes[n] = seeds[i];
        where[seeds[i]] = n;
        ++n;
    }
    b->tier_off[0] = 0;
    b->tier_off[1] = n;

    int64_t* pos = NULL;
    int64_t pos_cap = 0;

    for (int32_t h = 0; h < num_hops; ++h) {
        int64_t k = fanouts[h];
        int64_t n_h = n;
        int64_t* indptr = (int64_t*)malloc((size_t)(n_h + 1) * sizeof(int64_t));
        /* pass 1: sizes (count = min(k, degree); k < 0 means every neighbour) */
        indptr[0] = 0;
        for (int64_t i = 0; i < n_h; ++i) {
            int64_t v = nodes[i];
            int64_t d = row_ptr[v + 1] - row_ptr[v];
            int64_t m = (k < 0 || d <= k) ? d : k;
            indptr[i + 1] = indptr[i] + m;
        }
        int64_t E = indptr[n_h];
        int32_t* nbr = (int32_t*)malloc((size_t)(E > 0 ? E : 1) * sizeof(int32_t));
        /* pass 2: sample every node of the cumulative frontier with the hop-h stream */
        for (int64_t i = 0; i < n_h; ++i) {
            int64_t v = nodes[i];
            int64_t d = row_ptr[v + 1] - row_ptr[v];
            int64_t m = indptr[i + 1] - indptr[i];
            if (m > pos_cap) {
                pos_cap = m * 2;
                pos = (int64_t*)realloc(pos, (size_t)pos_cap * sizeof(int64_t));
            }
            int64_t got = orc_sample_positions(seed, epoch, (uint32_t)v, (uint32_t)h, d, k, pos);
            (void)got;
            for (int64_t t = 0; t < m; ++t)
                nbr[indptr[i] + t] = col_idx[row_ptr[v] + pos[t]];
        }
        if (node_order == ORC_ORDER_FIRST_SEEN) {
            /* new tier: ids seen in nbr that are not yet frontier members, each once, in the order in which the hop's
             * neighbour list first names them */
            if (n + E > cap) {
                cap = (n + E) * 2;
                nodes = (int32_t*)realloc(nodes, (size_t)cap * sizeof(int32_t));
            }
            for (int64_t e = 0; e < E; ++e) {
                int32_t u = nbr[e];
                if (where[u] < 0) {
                    nodes[n] = u;
                    where[u] = n;
                    ++n;
                }
            }
        } else {
            /* new tier: ids seen in nbr that are not yet frontier members, unique, ascending */
            int32_t* fresh = (int32_t*)malloc((size_t)(E > 0 ? E : 1) * sizeof(int32_t));
            int64_t n_fresh = 0;
            for (int64_t e = 0; e < E; ++e)
                if (where[nbr[e]] < 0) fresh[n_fresh++] = nbr[e];
            qsort(fresh, (size_t)n_fresh, sizeof(int32_t), orc_i32_cmp);
            int64_t n_unique = 0;
            for (int64_t e = 0; e < n_fresh; ++e)
                if (e == 0 || fresh[e] != fresh[e - 1]) fresh[n_unique++] = fresh[e];
            if (n + n_unique > cap) {
                cap = (n + n_unique) * 2;
                nodes = (int32_t*)realloc(nodes, (size_t)cap * sizeof(int32_t));
            }
            for (int64_t e = 0; e < n_unique; ++e) {
                nodes[n] = fresh[e];
                where[fresh[e]] = n;
                ++n;
            }
            free(fresh);
        }
        /* neighbours relabelled to positions in frontier_{h+1} */
        int32_t* nbr_local = (int32_t*)malloc((size_t)(E > 0 ? E : 1) * sizeof(int32_t));
        for (int64_t e = 0; e < E; ++e) nbr_local[e] = (int32_t)where[nbr[e]];

        b->tier_off[h + 2] = n;
        b->num_edges[h] = E;
        b->indptr[h] = indptr;
        b->nbr[h] = nbr;
        b->nbr_local[h] = nbr_local;
    }
    b->nodes = nodes;
    free(pos);
    free(where);
    return b;
}

orc_blocks* orc_sample_blocks(int64_t num_nodes, const int64_t* row_ptr, const int32_t* col_idx,
                              const int32_t* seeds, int64_t num_seeds,
                              const int32_t* fanouts, int32_t num_hops,
                              uint64_t seed, uint32_t epoch) {
    return orc_sample_blocks_ordered(num_nodes, row_ptr, col_idx, seeds, num_seeds, fanouts, num_hops, seed, epoch,
                                     ORC_ORDER_ASCENDING);
}

void orc_blocks_free(orc_blocks* b) {
    if (!b) return;
    for (int32_t h = 0; h < b->num_hops; ++h) {
        free(b->indptr[h]);
        free(b->nbr[h]);
        free(b->nbr_local[h]);
    }
    free(b->indptr); free(b->nbr); free(b->nbr_local);
    free(b->num_edges); free(b->tier_off); free(b->nodes);
    free(b);
}

int32_t orc_blocks_num_hops(const orc_blocks* b) { return b->num_hops; }
const int64_t* orc_blocks_tier_off(const orc_blocks* b) { return b->tier_off; }
const int32_t* orc_blocks_nodes(const orc_blocks* b) { return b->nodes; }
int64_t orc_blocks_num_edges(const orc_blocks* b, int32_t hop) { return b->num_edges[hop]; }
const int64_t* orc_blocks_indptr(const orc_blocks* b, int32_t hop) { return b->indptr[hop]; }
const int32_t* orc_blocks_nbr(const orc_blocks* b, int32_t hop) { return b->nbr[hop]; }
const int32_t* orc_blocks_nbr_local(const orc_blocks* b, int32_t hop) { return b->nbr_local[hop]; }

/* ---- freq(n), Section IV (offline stage) */
void orc_access_histogram(const int32_t* nodes, int64_t n, uint32_t* counts, int64_t num_nodes) {
    (void)num_nodes;
    for (int64_t i = 0; i < n; ++i) counts[nodes[i]] += 1u;
}

/* ---- TopHot, Alg. 1 line 3 */
typedef struct { uint32_t count; int32_t id; } orc_cand;

static int orc_cand_cmp(const void* a, const void* b) {
    const orc_cand* x = (const orc_cand*)a;
    const orc_cand* y = (const orc_cand*)b;
    if (x->count != y->count) return x->count > y->count ? -1 : 1;   /* larger count first */
    if (x->id != y->id) return x->id < y->id ? -1 : 1;               /* then lower id */
    return 0;
}

int64_t orc_build_cache(const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                        int64_t capacity_rows, int32_t* cache_ids, int32_t* loc) {
    orc_cand* cand = (orc_cand*)malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof(orc_cand));
    int64_t n_cand = 0;
    for (int64_t v = 0; v < num_nodes; ++v) {
        uint32_t tag = (uint32_t)home[v] >> ORC_TAG_SHIFT;
        if (tag == ORC_TAG_REMOTE && counts[v] >= 1u) {
            cand[n_cand].count = counts[v];
            cand[n_cand].id = (int32_t)v;
            ++n_cand;
        }
    }
    qsort(cand, (size_t)n_cand, sizeof(orc_cand), orc_cand_cmp);
    int64_t k_eff = capacity_rows < n_cand ? capacity_rows : n_cand;
    if (k_eff < 0) k_eff = 0;
    for (int64_t s = 0; s < k_eff; ++s) cache_ids[s] = cand[s].id;
    qsort(cache_ids, (size_t)k_eff, sizeof(int32_t), orc_i32_cmp);
    for (int64_t v = 0; v < num_nodes; ++v) loc[v] = home[v];
    for (int64_t s = 0; s < k_eff; ++s)
        loc[cache_ids[s]] = (int32_t)((ORC_TAG_CACHE << ORC_TAG_SHIFT) | (uint32_t)s);
    free(cand);
    return k_eff;
}

/* ---- VectorPull, Alg. 1 line 4 */
void orc_fill_cache(const float* X, int64_t dim, const int32_t* cache_ids, int64_t num_cached,
                    float* cache_rows, int64_t row_stride) {
    for (int64_t s = 0; s < num_cached; ++s)
        for (int64_t c = 0; c < dim; ++c)
            cache_rows[s * row_stride + c] = X[(int64_t)cache_ids[s] * dim + c];
}

/* ---- per-batch feature assembly, Alg. 1 lines 12-14 */
void orc_gather_features(const float* X, int64_t dim, const int32_t* input_nodes, int64_t n,
                         const int32_t* loc, float* out, int64_t out_stride, int64_t stats[3]) {
    stats[0] = stats[1] = stats[2] = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t v = input_nodes[i];
        for (int64_t c = 0; c < dim; ++c) out[i * out_stride + c] = X[v * dim + c];
        uint32_t tag = (uint32_t)loc[v] >> ORC_TAG_SHIFT;
        if (tag == ORC_TAG_LOCAL) stats[0] += 1;
        else if (tag == ORC_TAG_CACHE) stats[1] += 1;
        else stats[2] += 1;
    }
}

/* ---- Eq. 1, AGG = mean over the sampled neighbours of each destination of a block (fp64) */
void orc_mean_aggregate(const int64_t* indptr, const int32_t* nbr_local, int64_t n_dst,
                        const float* feat, int64_t feat_stride, int64_t dim, double* agg) {
    for (int64_t i = 0; i < n_dst; ++i) {
        int64_t m = indptr[i + 1] - indptr[i];
        for (int64_t c = 0; c < dim; ++c) {
            double sum = 0.0;
            for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e)
                sum += (double)feat[(int64_t)nbr_local[e] * feat_stride + c];
            agg[i * dim + c] = m > 0 ? sum / (double)m : 0.0;
        }
    }
}

/* ---- requests served against cache capacity: prefix sums of the counts in TopHot order */
uint64_t orc_cache_hit_curve(const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                             const int64_t* capacities, int64_t num_capacities, uint64_t* hits) {
    orc_cand* cand = (orc_cand*)malloc((size_t)(num_nodes > 0 ? num_nodes : 1) * sizeof(orc_cand));
    int64_t n_cand = 0;
    for (int64_t v = 0; v < num_nodes; ++v)
        if (((uint32_t)home[v] >> ORC_TAG_SHIFT) == ORC_TAG_REMOTE && counts[v] >= 1u) {
            cand[n_cand].count = counts[v];
            cand[n_cand].id = (int32_t)v;
            ++n_cand;
        }
    qsort(cand, (size_t)n_cand, sizeof(orc_cand), orc_cand_cmp);
    uint64_t total = 0;
    for (int64_t s = 0; s < n_cand; ++s) total += cand[s].count;
    for (int64_t j = 0; j < num_capacities; ++j) {
        uint64_t sum = 0;
        for (int64_t s = 0; s < n_cand && s < capacities[j]; ++s) sum += cand[s].count;
        hits[j] = sum;
    }
    free(cand);
    return total;
}
