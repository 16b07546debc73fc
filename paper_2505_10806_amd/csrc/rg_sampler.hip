// Epoch schedule and multi-hop neighbour sampling (Alg. 1 line 1; SAMPLE(eta(v), k) of Section II-B).
//
// Data layout in HBM: CSR (row_ptr int32/int64, col_idx int32) is read-only; the batch's cumulative
// frontier `nodes` grows tier by tier; membership lives in two N-bit bitmaps (`visited` = members of
// the cumulative frontier, `marked` = those plus the ids the current hop has sampled) and `pos[v]` maps a member to
// its position.  All sizes that depend on the data (frontier and edge counts) stay on the device:
// launches are sized by static upper bounds and kernels read the actual counts.
#include "rg_internal.h"

namespace {

constexpr int kChunk = 256;          // frontier nodes per workgroup in the count / sample kernels
constexpr int kWordsPerBlock = 1024; // bitmap words per workgroup in the tier kernels (256 threads x 4)

template <typename RP>
__device__ __forceinline__ void rg_row_extent(const RP* __restrict__ row_ptr, int v, int64_t& start, int64_t& deg) {
    const RP a = row_ptr[v];
    const RP b = row_ptr[v + 1];
    start = (int64_t)a;
    deg = (int64_t)(b - a);
}

// ---------------------------------------------------------------------------- schedule
__global__ void __launch_bounds__(256) k_sched_keys(const int32_t* __restrict__ train_ids, int64_t n, int64_t npad,
                                                    uint32_t k0, uint32_t k1, uint32_t epoch,
                                                    uint64_t* __restrict__ keys, int32_t* __restrict__ ids) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= npad) return;
    if (i < n) {
        const int32_t v = train_ids[i];
        uint32_t w[4];
        rg_philox4x32_10((uint32_t)v, 0xFFFFFFFFu, 0u, epoch, k0, k1, w);
        keys[i] = ((uint64_t)w[0] << 32) | (uint64_t)w[1];
        ids[i] = v;
    } else {                       // padding sorts after every real entry
        keys[i] = ~0ull;
        ids[i] = 0x7FFFFFFF;
    }
}

__device__ __forceinline__ bool rg_pair_less(uint64_t ka, int32_t ia, uint64_t kb, int32_t ib) {
    return ka < kb || (ka == kb && ia < ib);
}

// One compare-exchange step of a bitonic sorting network on (key, id) pairs, ascending overall.
__global__ void __launch_bounds__(256) k_bitonic_step(uint64_t* __restrict__ keys, int32_t* __restrict__ ids,
                                                      int64_t npad, int64_t j, int64_t k) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= npad) return;
    const int64_t l = i ^ j;
    if (l <= i) return;
    const uint64_t ka = keys[i], kb = keys[l];
    const int32_t ia = ids[i], ib = ids[l];
    const bool ascending = (i & k) == 0;
    const bool out_of_order = ascending ? rg_pair_less(kb, ib, ka, ia) : rg_pair_less(ka, ia, kb, ib);
    if (out_of_order) {
        keys[i] = kb; keys[l] = ka;
        ids[i] = ib; ids[l] = ia;
    }
}

// All steps with partner distance < 2048 of one merge stage, fused in LDS (2048 pairs per workgroup).
__global__ void __launch_bounds__(1024) k_bitonic_local(uint64_t* __restrict__ keys, int32_t* __restrict__ ids,
                                                        int64_t npad, int64_t k_first, int64_t k_last) {
    __shared__ uint64_t sk[2048];
    __shared__ int32_t si[2048];
    const int64_t base = (int64_t)blockIdx.x * 2048;
    for (int t = threadIdx.x; t < 2048; t += 1024) {
        const int64_t g = base + t;
        sk[t] = g < npad ? keys[g] : ~0ull;
        si[t] = g < npad ? ids[g] : 0x7FFFFFFF;
    }
    __syncthreads();
    for (int64_t k = k_first; k <= k_last; k <<= 1) {
        for (int64_t j = (k >> 1) < 1024 ? (k >> 1) : 1024; j > 0; j >>= 1) {
            // thread t owns the pair (i, i ^ j) with bit j of i clear
            const int t = threadIdx.x;
            const int i = ((t & ~((int)j - 1)) << 1) | (t & ((int)j - 1));
            const int l = i | (int)j;
            const bool ascending = ((base + i) & k) == 0;
            const uint64_t ka = sk[i], kb = sk[l];
            const int32_t ia = si[i], ib = si[l];
            const bool out_of_order = ascending ? rg_pair_less(kb, ib, ka, ia) : rg_pair_less(ka, ia, kb, ib);
            if (out_of_order) {
                sk[i] = kb; sk[l] = ka;
                si[i] = ib; si[l] = ia;
            }
            __syncthreads();
        }
    }
    for (int t = threadIdx.x; t < 2048; t += 1024) {
        const int64_t g = base + t;
        if (g < npad) { keys[g] = sk[t]; ids[g] = si[t]; }
    }
}

__global__ void __launch_bounds__(256) k_sched_out(const int32_t* __restrict__ ids, int64_t n, int32_t* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = ids[i];
}

// ---------------------------------------------------------------------------- batches of a group
// Several batches are sampled by the same launches: blockIdx.y selects the batch, which brings its own outputs
// (SampleGroup, passed by value) and its own slice of the scratch (SampleScratch).  Most kernels of one batch are
// far smaller than the device (hop 0 of a 4096-seed batch is 16 workgroups), so a group fills it better and pays
// every launch once.
constexpr int kMaxGroup = RG_MAX_GROUP;

struct SampleGroup {
    const int32_t* seeds[kMaxGroup];
    int32_t num_seeds[kMaxGroup];
    int32_t* nodes[kMaxGroup];
    int32_t* tier_off[kMaxGroup];
    int32_t* indptr[kMaxGroup];       // of the current hop
    int32_t* nbr[kMaxGroup];
    int32_t* nbr_local[kMaxGroup];    // may be NULL
    int32_t* edges_out[kMaxGroup];    // may be NULL
};

struct SampleScratch {
    uint32_t* visited;                // [group][words]
    uint32_t* marked;                 // [group][words]
    int32_t* pos;                     // [group][num_nodes]
    int32_t* chunk_sum;               // [group][chunk_stride]
    int64_t* row_start;               // [group][frontier_stride]
    int32_t* row_deg;                 // [group][frontier_stride]
    int32_t* first_key;               // [group][num_nodes], first-seen order only: 0x7FFFFFFF - (index of the first edge of
                                      // the current hop that names the node), 0 = not named (kept all-zero between hops)
    int64_t words, num_nodes, chunk_stride, frontier_stride;
    int group;                        // batches in this call
    int xcd_map;                      // 1: consecutive workgroups belong to consecutive batches (see rg_batch)
};

// Workgroup -> (batch, block within the batch) for the per-batch kernels, launched as one 1-D grid of blocks x group
// workgroups.  The device hands consecutive workgroup ids to its 8 XCDs in turn, and every XCD has an L2 of its own.
// With xcd_map, workgroup id w works on batch w % group: with a group of 8 all workgroups of one batch run on one XCD,
// whose L2 then holds that batch's membership bitmaps (2 x N/8 bytes, probed at random by every sampled edge) instead
// of every XCD holding a share of all eight.
__device__ __forceinline__ int rg_batch(const SampleScratch& S) {
    return S.xcd_map ? (int)(blockIdx.x % (unsigned)S.group) : (int)(blockIdx.x / (gridDim.x / (unsigned)S.group));
}
__device__ __forceinline__ unsigned rg_block(const SampleScratch& S) {
    return S.xcd_map ? blockIdx.x / (unsigned)S.group : blockIdx.x % (gridDim.x / (unsigned)S.group);
}
__device__ __forceinline__ unsigned rg_blocks_per_batch(const SampleScratch& S) { return gridDim.x / (unsigned)S.group; }

// ---------------------------------------------------------------------------- batch start
__global__ void __launch_bounds__(256) k_clear_words(uint32_t* __restrict__ w, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0u;
}

__global__ void __launch_bounds__(256) k_mark_seeds(const SampleGroup G, const SampleScratch S) {
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const int num_seeds = G.num_seeds[g];
    const int i = blk * blockDim.x + threadIdx.x;
    if (i == 0) { G.tier_off[g][0] = 0; G.tier_off[g][1] = num_seeds; }
    if (i >= num_seeds) return;
    const int32_t v = G.seeds[g][i];
    G.nodes[g][i] = v;
    S.pos[g * S.num_nodes + v] = i;
    atomicOr(&S.visited[g * S.words + ((uint32_t)v >> 5)], 1u << (v & 31));
    atomicOr(&S.marked[g * S.words + ((uint32_t)v >> 5)], 1u << (v & 31));
}

// ---------------------------------------------------------------------------- per hop: sizes
// indptr[i] = exclusive prefix of m within the node's 256-node chunk; chunk_sum[b] = chunk total;
// row_start[i], row_deg[i] = the node's adjacency row.
template <typename RP>
__global__ void __launch_bounds__(kChunk) k_hop_count(const RP* __restrict__ row_ptr, const SampleGroup G, const SampleScratch S,
                                                      int hop, int fanout) {
    __shared__ int smem[kChunk / RG_WAVE + 1];
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const int n_h = G.tier_off[g][hop + 1];
    const int64_t first = (int64_t)blk * kChunk;
    if (first >= n_h) return;                       // uniform per workgroup
    const int64_t i = first + threadIdx.x;
    int m = 0;
    if (i < n_h) {
        int64_t start, deg;
        rg_row_extent(row_ptr, G.nodes[g][i], start, deg);
        m = (fanout < 0 || deg <= fanout) ? (int)deg : fanout;
        S.row_start[g * S.frontier_stride + i] = start;   // kept for the draw kernel: one coalesced read there instead
        S.row_deg[g * S.frontier_stride + i] = (int32_t)deg;   // of a second random lookup of row_ptr
    }
    int total;
    const int excl = rg_block_excl_scan<kChunk / RG_WAVE>(m, smem, &total);
    if (i < n_h) G.indptr[g][i] = excl;
    if (threadIdx.x == 0) S.chunk_sum[g * S.chunk_stride + blk] = total;
}

// In-place exclusive scan of data[0..n) by one workgroup; returns (to thread 0) the grand total.
__device__ __forceinline__ int rg_scan_in_place(int32_t* __restrict__ data, int64_t n) {
    __shared__ int smem[1024 / RG_WAVE + 1];
    __shared__ int carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int x = i < n ? data[i] : 0;
        int total;
        const int excl = rg_block_excl_scan<1024 / RG_WAVE>(x, smem, &total);
        const int carry = carry_s;
        if (i < n) data[i] = carry + excl;
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
    return carry_s;
}

// Chunk totals of a hop -> exclusive offsets; the hop's edge total goes behind the last indptr entry.
__global__ void __launch_bounds__(1024) k_scan_hop(const SampleGroup G, const SampleScratch S, int hop) {
    const int g = rg_batch(S);
    const int n_h = G.tier_off[g][hop + 1];
    const int total = rg_scan_in_place(S.chunk_sum + g * S.chunk_stride, ((int64_t)n_h + kChunk - 1) / kChunk);
    if (threadIdx.x == 0) {
        G.indptr[g][n_h] = total;
        if (G.edges_out[g]) *G.edges_out[g] = total;
    }
}

// Per-block counts of fresh ids -> exclusive offsets; the end of the new tier goes to tier_off[hop + 2].
__global__ void __launch_bounds__(1024) k_scan_tier(const SampleGroup G, const SampleScratch S, int hop, int tier_blocks) {
    const int g = rg_batch(S);
    const int total = rg_scan_in_place(S.chunk_sum + g * S.chunk_stride, tier_blocks);
    if (threadIdx.x == 0) G.tier_off[g][hop + 2] = G.tier_off[g][hop + 1] + total;
}

// ---------------------------------------------------------------------------- per hop: draw + read
// `marked` holds every id a batch has met so far: the frontier members (`visited`) plus the ids the current hop has
// sampled.  One probe per sampled edge; the hop's new tier is marked & ~visited.
__device__ __forceinline__ void rg_mark(int32_t u, uint32_t* __restrict__ marked) {
    const uint32_t w = (uint32_t)u >> 5, bit = 1u << (u & 31);
    if (marked[w] & bit) return;                      // a stale read only costs a redundant atomic
    atomicOr(&marked[w], bit);
}

// First-seen order: instead of a bit, remember the first edge of the hop that names a node outside the frontier.
__device__ __forceinline__ void rg_note_first_edge(int32_t u, int64_t e, const uint32_t* __restrict__ visited,
                                                   int32_t* __restrict__ first_key) {
    const uint32_t w = (uint32_t)u >> 5, bit = 1u << (u & 31);
    if (visited[w] & bit) return;
    const int32_t key = 0x7FFFFFFF - (int32_t)e;
    if (first_key[u] >= key) return;                  // a stale read only costs a redundant atomic
    atomicMax(&first_key[u], key);
}

// General sampler: one wavefront (= one 64-thread workgroup) per frontier node, any fan-out up to
// RG_MAX_FANOUT.  The Floyd set lives in LDS; step i tests membership of t with all lanes.
template <bool FIRST_SEEN>
__global__ void __launch_bounds__(RG_WAVE) k_hop_sample_wave(const int32_t* __restrict__ col_idx, const SampleGroup G,
                                                            const SampleScratch S, int fanout, uint32_t hop, uint32_t k0,
                                                            uint32_t k1, uint32_t epoch) {
    __shared__ uint32_t draws[RG_MAX_FANOUT];
    __shared__ uint32_t chosen[RG_MAX_FANOUT];
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const int n_h = G.tier_off[g][hop + 1];
    const int32_t* __restrict__ nodes = G.nodes[g];
    int32_t* __restrict__ indptr = G.indptr[g];
    int32_t* __restrict__ nbr = G.nbr[g];
    const int32_t* __restrict__ chunk_sum = S.chunk_sum + g * S.chunk_stride;
    const int64_t* __restrict__ row_start = S.row_start + g * S.frontier_stride;
    const int32_t* __restrict__ row_deg = S.row_deg + g * S.frontier_stride;
    const uint32_t* __restrict__ visited = S.visited + g * S.words;
    uint32_t* __restrict__ marked = S.marked + g * S.words;
    int32_t* __restrict__ first_key = FIRST_SEEN ? S.first_key + g * S.num_nodes : nullptr;
    const int lane = threadIdx.x;
    for (int64_t i = blk; i < n_h; i += rg_blocks_per_batch(S)) {
        const int32_t v = nodes[i];
        const int64_t start = row_start[i], deg = row_deg[i];
        const int base = indptr[i] + chunk_sum[i / kChunk];
        __syncthreads();                               // every lane has read indptr[i] before it is rewritten
        if (lane == 0) indptr[i] = base;
        if (fanout < 0 || deg <= fanout) {             // whole row, CSR order
            for (int64_t t = lane; t < deg; t += RG_WAVE) {
                const int32_t u = col_idx[start + t];
                nbr[base + t] = u;
                if (FIRST_SEEN) rg_note_first_edge(u, base + t, visited, first_key); else rg_mark(u, marked);
            }
            continue;
        }
        const int k = fanout;
        for (int blk = lane; blk * 4 < k; blk += RG_WAVE) {
            uint32_t w[4];
            rg_philox4x32_10((uint32_t)v, hop, (uint32_t)blk, epoch, k0, k1, w);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (blk * 4 + q < k) draws[blk * 4 + q] = w[q];
        }
        __syncthreads();
        for (int s = 0; s < k; ++s) {                  // Floyd: j = d-k+s, t uniform in [0, j]
            const uint32_t j = (uint32_t)(deg - k + s);
            const uint32_t t = __umulhi(draws[s], j + 1u);
            int found = 0;
            for (int l = lane; l < s; l += RG_WAVE) found |= (chosen[l] == t);
            found = __any(found);
            __syncthreads();
            if (lane == 0) chosen[s] = found ? j : t;
            __syncthreads();
        }
        for (int t = lane; t < k; t += RG_WAVE) {
            const int32_t u = col_idx[start + (int64_t)chosen[t]];
            nbr[base + t] = u;
            if (FIRST_SEEN) rg_note_first_edge(u, base + t, visited, first_key); else rg_mark(u, marked);
        }
    }
}

// Fast sampler for fan-outs up to 32 on graphs with fewer than 2^32 edges: one thread per frontier node
// draws (Philox + Floyd entirely in registers), the 256 nodes of a workgroup stage the col_idx offsets
// of their picks in LDS in output order, then the whole workgroup reads col_idx and writes nbr with
// consecutive lanes on consecutive output slots.
template <int KMAX, bool FIRST_SEEN>
__global__ void __launch_bounds__(kChunk) k_hop_sample_thread(const int32_t* __restrict__ col_idx, const SampleGroup G,
                                                              const SampleScratch S, int fanout, uint32_t hop, uint32_t k0,
                                                              uint32_t k1, uint32_t epoch) {
    extern __shared__ uint32_t staged[];                 // kChunk * fanout col_idx offsets
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const int n_h = G.tier_off[g][hop + 1];
    const int64_t first = (int64_t)blk * kChunk;
    if (first >= n_h) return;                            // uniform per workgroup
    int32_t* __restrict__ indptr = G.indptr[g];
    int32_t* __restrict__ nbr = G.nbr[g];
    const int32_t* __restrict__ chunk_sum = S.chunk_sum + g * S.chunk_stride;
    const uint32_t* __restrict__ visited = S.visited + g * S.words;
    uint32_t* __restrict__ marked = S.marked + g * S.words;
    int32_t* __restrict__ first_key = FIRST_SEEN ? S.first_key + g * S.num_nodes : nullptr;
    const int64_t i = first + threadIdx.x;
    const int k = fanout;
    // chunk_sum[b] is the exclusive offset of chunk b; the chunk's edge count follows from its successor
    // (or from the hop total behind the last indptr entry for the last chunk)
    const int base = chunk_sum[blk];
    const bool last_chunk = first + kChunk >= n_h;
    const int chunk_edges = (last_chunk ? indptr[n_h] : chunk_sum[blk + 1]) - base;
    if (i < n_h) {
        const int32_t v = G.nodes[g][i];
        const int64_t start = S.row_start[g * S.frontier_stride + i], deg = S.row_deg[g * S.frontier_stride + i];
        const int off = indptr[i];                       // chunk-local exclusive prefix from k_hop_count
        indptr[i] = base + off;
        if (deg <= k) {                                  // whole row, CSR order
            for (int t = 0; t < (int)deg; ++t) staged[off + t] = (uint32_t)(start + t);
        } else {
            uint32_t c[KMAX];
#pragma unroll
            for (int blk = 0; blk < KMAX / 4; ++blk) {
                if (blk * 4 < k) {
                    uint32_t w[4];
                    rg_philox4x32_10((uint32_t)v, hop, (uint32_t)blk, epoch, k0, k1, w);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int s = blk * 4 + q;
                        if (s < k) {                     // Floyd: j = d-k+s, t uniform in [0, j]
                            const uint32_t j = (uint32_t)(deg - k + s);
                            const uint32_t t = __umulhi(w[q], j + 1u);
                            bool found = false;
#pragma unroll
                            for (int l = 0; l < s; ++l) found |= (c[l] == t);
                            c[s] = found ? j : t;
                        }
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < KMAX; ++s)
                if (s < k) staged[off + s] = (uint32_t)(start + (int64_t)c[s]);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < chunk_edges; e += kChunk) {
        const int32_t u = col_idx[staged[e]];
        nbr[base + e] = u;
        if (FIRST_SEEN) rg_note_first_edge(u, base + e, visited, first_key); else rg_mark(u, marked);
    }
}

// ---------------------------------------------------------------------------- per hop: new tier
__global__ void __launch_bounds__(256) k_tier_count(const SampleScratch S) {
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const uint32_t* __restrict__ marked = S.marked + g * S.words;
    const uint32_t* __restrict__ visited = S.visited + g * S.words;
    const int64_t w0 = (int64_t)blk * kWordsPerBlock + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (w0 + q < S.words) c += __popc(marked[w0 + q] & ~visited[w0 + q]);
    c = rg_wave_sum(c);
    __shared__ int part[4];
    if (rg_lane() == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) S.chunk_sum[g * S.chunk_stride + blk] = part[0] + part[1] + part[2] + part[3];
}

// Emit the new ids (marked, not yet visited) in ascending order behind the current frontier, record their positions
// and make them frontier members (visited = marked).  chunk_sum holds exclusive block offsets.
__global__ void __launch_bounds__(256) k_tier_emit(const SampleGroup G, const SampleScratch S, int hop) {
    __shared__ int smem[256 / RG_WAVE + 1];
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const uint32_t* __restrict__ marked = S.marked + g * S.words;
    uint32_t* __restrict__ visited = S.visited + g * S.words;
    int32_t* __restrict__ nodes = G.nodes[g];
    int32_t* __restrict__ pos = S.pos + g * S.num_nodes;
    const int64_t w0 = (int64_t)blk * kWordsPerBlock + threadIdx.x * 4;
    uint32_t bits[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        bits[q] = (w0 + q < S.words) ? marked[w0 + q] & ~visited[w0 + q] : 0u;
        c += __popc(bits[q]);
    }
    int total;
    const int excl = rg_block_excl_scan<256 / RG_WAVE>(c, smem, &total);
    if (total == 0) return;                          // uniform: nothing fresh in this block
    int out = G.tier_off[g][hop + 1] + S.chunk_sum[g * S.chunk_stride + blk] + excl;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t b = bits[q];
        if (b == 0u) continue;
        visited[w0 + q] |= b;
        const int32_t id0 = (int32_t)((w0 + q) << 5);
        while (b) {
            const int bit = __ffs(b) - 1;
            b &= b - 1u;
            const int32_t id = id0 + bit;
            nodes[out] = id;
            pos[id] = out;
            ++out;
        }
    }
}

// ---------------------------------------------------------------------------- per hop: new tier in first-seen order
// Edge e opens a new node when it is the first edge of the hop naming a node outside the frontier.  Ordered
// compaction over the hop's edge list: per-block counts, the scan of k_scan_tier, then the emit below.
constexpr int kEdgesPerBlock = 1024;   // 256 threads x 4 consecutive edges

__device__ __forceinline__ bool rg_opens_node(const int32_t* __restrict__ nbr, const int32_t* __restrict__ first_key, int64_t e) {
    return first_key[nbr[e]] == 0x7FFFFFFF - (int32_t)e;
}

__global__ void __launch_bounds__(256) k_first_seen_count(const SampleGroup G, const SampleScratch S, int hop) {
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const int32_t* __restrict__ nbr = G.nbr[g];
    const int32_t* __restrict__ first_key = S.first_key + g * S.num_nodes;
    const int64_t n_edges = G.indptr[g][G.tier_off[g][hop + 1]];
    const int64_t e0 = (int64_t)blk * kEdgesPerBlock + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (e0 + q < n_edges) c += rg_opens_node(nbr, first_key, e0 + q);
    c = rg_wave_sum(c);
    __shared__ int part[4];
    if (rg_lane() == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) S.chunk_sum[g * S.chunk_stride + blk] = part[0] + part[1] + part[2] + part[3];
}

// Appends the opened nodes behind the current frontier in edge order, records their positions, marks them visited
// and clears their first-edge keys (the array is all-zero again when the hop is done).
__global__ void __launch_bounds__(256) k_first_seen_emit(const SampleGroup G, const SampleScratch S, int hop) {
    __shared__ int smem[256 / RG_WAVE + 1];
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    const int32_t* __restrict__ nbr = G.nbr[g];
    int32_t* __restrict__ first_key = S.first_key + g * S.num_nodes;
    uint32_t* __restrict__ visited = S.visited + g * S.words;
    int32_t* __restrict__ nodes = G.nodes[g];
    int32_t* __restrict__ pos = S.pos + g * S.num_nodes;
    const int64_t n_edges = G.indptr[g][G.tier_off[g][hop + 1]];
    const int64_t e0 = (int64_t)blk * kEdgesPerBlock + threadIdx.x * 4;
    if ((int64_t)blk * kEdgesPerBlock >= n_edges) return;          // uniform per workgroup
    int32_t u[4];
    bool opens[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        opens[q] = false;
        if (e0 + q < n_edges) {
            u[q] = nbr[e0 + q];
            opens[q] = first_key[u[q]] == 0x7FFFFFFF - (int32_t)(e0 + q);
        }
        c += opens[q];
    }
    int total;
    const int excl = rg_block_excl_scan<256 / RG_WAVE>(c, smem, &total);
    if (total == 0) return;                                               // uniform
    int out = G.tier_off[g][hop + 1] + S.chunk_sum[g * S.chunk_stride + blk] + excl;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (opens[q]) {
            nodes[out] = u[q];
            pos[u[q]] = out;
            ++out;
            atomicOr(&visited[(uint32_t)u[q] >> 5], 1u << (u[q] & 31));
            first_key[u[q]] = 0;                      // only the opening edge's thread touches this entry now
        }
}

// nbr_local[e] = position of nbr[e] in the extended frontier; the hop's edge count is indptr[n_h].
__global__ void __launch_bounds__(256) k_relabel(const SampleGroup G, const SampleScratch S, int hop) {
    const int g = rg_batch(S);
    const unsigned blk = rg_block(S);
    int32_t* __restrict__ nbr_local = G.nbr_local[g];
    if (!nbr_local) return;
    const int32_t* __restrict__ nbr = G.nbr[g];
    const int32_t* __restrict__ pos = S.pos + g * S.num_nodes;
    const int n = G.indptr[g][G.tier_off[g][hop + 1]];
    for (int64_t e = (int64_t)blk * blockDim.x + threadIdx.x; e < n; e += (int64_t)rg_blocks_per_batch(S) * blockDim.x)
        nbr_local[e] = pos[nbr[e]];
}

// Per-batch strides of the scratch slices for a graph of N nodes and frontiers of up to `frontier` nodes.
// max_edges: the largest per-hop edge bound when tiers are built from the edge list (first-seen order), else 0.
void sampler_scratch_shape(int64_t N, int64_t frontier, int64_t max_edges, SampleScratch& S) {
    S.words = rg_div_up(N, 32);
    S.num_nodes = N;
    S.frontier_stride = rg_max64(frontier, 1);
    S.chunk_stride = rg_max64(rg_max64(rg_div_up(S.frontier_stride, kChunk), rg_div_up(max_edges, kEdgesPerBlock)),
                              rg_max64(1, rg_div_up(S.words, kWordsPerBlock))) + 2;
    S.first_key = nullptr;
    S.group = 1;
    S.xcd_map = 1;
}

// ---------------------------------------------------------------------------- access counts straight from the bitmaps
// After the last hop a batch's `visited` bitmap is exactly its input-node set.  One thread takes bitmap word w of
// every batch of the group, counts for each of the 32 ids in how many of the batches it is set, and adds that to
// counts[] (and lowers first_batch[] to the earliest of those batches).  No id list is read.
struct BatchIndices { uint32_t v[kMaxGroup]; };

__global__ void __launch_bounds__(256) k_histogram_bitmaps(const uint32_t* __restrict__ visited, int64_t words, int group,
                                                           const BatchIndices batch, uint32_t* __restrict__ counts,
                                                           uint32_t* __restrict__ first_batch, int64_t num_nodes) {
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < words; w += (int64_t)gridDim.x * blockDim.x) {
        uint32_t bits[kMaxGroup];
        uint32_t any = 0u;
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) {
            bits[g] = g < group ? visited[g * words + w] : 0u;
            any |= bits[g];
        }
        while (any) {
            const int j = __ffs(any) - 1;
            any &= any - 1u;
            uint32_t c = 0u, first = 0xFFFFFFFFu;
#pragma unroll
            for (int g = 0; g < kMaxGroup; ++g)
                if ((bits[g] >> j) & 1u) {
                    ++c;
                    first = batch.v[g] < first ? batch.v[g] : first;
                }
            const int64_t v = (w << 5) + j;
            if (v < num_nodes) {                      // bits beyond the last node are never set; the check costs nothing
                atomicAdd(&counts[v], c);
                if (first_batch && first < first_batch[v]) atomicMin(&first_batch[v], first);
            }
        }
    }
}

int grid_for(int64_t work_items, int per_block, int64_t cap) {
    int64_t g = rg_div_up(work_items, per_block);
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

rg_status rg_sampler_reserve(rg_ctx* ctx, int64_t num_nodes, int64_t max_frontier, int group, int64_t max_edges, bool first_seen) {
    SampleScratch S;
    sampler_scratch_shape(num_nodes, max_frontier, max_edges, S);
    const size_t g = (size_t)group;
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->visited, g * S.words * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->marked, g * S.words * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->pos, g * (size_t)num_nodes * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->chunk_sum, g * S.chunk_stride * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->row_start, g * S.frontier_stride * 8)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->row_deg, g * S.frontier_stride * 4)) != RG_OK) return st;
    // first-seen order: the first-edge keys must be all-zero between hops (every hop leaves them zeroed)
    if (first_seen && (st = rg_ensure(ctx, ctx->first_key, g * (size_t)num_nodes * 4, true)) != RG_OK) return st;
    return RG_OK;
}

extern "C" {

rg_status rg_epoch_schedule(rg_ctx* ctx, const int32_t* train_ids, int64_t n, uint64_t seed, uint32_t epoch,
                            int32_t* order_out, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, n >= 0, "rg_epoch_schedule: n = %lld is negative", (long long)n);
    RG_REQUIRE(ctx, n <= (1ll << 30), "rg_epoch_schedule: n = %lld exceeds 2^30", (long long)n);
    if (n == 0) return RG_OK;
    RG_REQUIRE(ctx, train_ids && order_out, "rg_epoch_schedule: null pointer");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    int64_t npad = 2048;
    while (npad < n) npad <<= 1;
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->sched_keys, (size_t)npad * 8)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->sched_ids, (size_t)npad * 4)) != RG_OK) return st;
    uint64_t* keys = (uint64_t*)ctx->sched_keys.p;
    int32_t* ids = (int32_t*)ctx->sched_ids.p;
    const uint32_t k0 = (uint32_t)(seed & 0xffffffffu), k1 = (uint32_t)(seed >> 32);
    const int g = (int)rg_div_up(npad, 256);
    k_sched_keys<<<g, 256, 0, s>>>(train_ids, n, npad, k0, k1, epoch, keys, ids);
    RG_LAUNCH_CHECK(ctx, "k_sched_keys");
    // merge stages k = 2 .. 2048 entirely in LDS, then per stage the far steps in HBM and the near ones in LDS
    k_bitonic_local<<<(int)(npad / 2048), 1024, 0, s>>>(keys, ids, npad, 2, 2048);
    RG_LAUNCH_CHECK(ctx, "k_bitonic_local");
    for (int64_t k = 4096; k <= npad; k <<= 1) {
        for (int64_t j = k >> 1; j >= 2048; j >>= 1) {
            k_bitonic_step<<<g, 256, 0, s>>>(keys, ids, npad, j, k);
            RG_LAUNCH_CHECK(ctx, "k_bitonic_step");
        }
        k_bitonic_local<<<(int)(npad / 2048), 1024, 0, s>>>(keys, ids, npad, k, k);
        RG_LAUNCH_CHECK(ctx, "k_bitonic_local");
    }
    k_sched_out<<<(int)rg_div_up(n, 256), 256, 0, s>>>(ids, n, order_out);
    RG_LAUNCH_CHECK(ctx, "k_sched_out");
    return RG_OK;
}

rg_status rg_sample_blocks_group(rg_ctx* ctx, const rg_csr* csr, int32_t group, const int32_t* const* seeds,
                                 const int32_t* num_seeds, const int32_t* fanouts, int32_t num_hops, uint64_t seed,
                                 uint32_t epoch, int32_t node_order, rg_blocks* out, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, node_order == RG_ORDER_ASCENDING || node_order == RG_ORDER_FIRST_SEEN,
               "rg_sample_blocks: node_order = %d is neither RG_ORDER_ASCENDING nor RG_ORDER_FIRST_SEEN", node_order);
    const bool first_seen = node_order == RG_ORDER_FIRST_SEEN;
    RG_REQUIRE(ctx, group >= 1 && group <= RG_MAX_GROUP, "rg_sample_blocks: group = %d not in [1,%d]", group, RG_MAX_GROUP);
    RG_REQUIRE(ctx, csr && out && fanouts && seeds && num_seeds, "rg_sample_blocks: null argument");
    RG_REQUIRE(ctx, num_hops >= 1 && num_hops <= RG_MAX_HOPS, "rg_sample_blocks: num_hops = %d not in [1,%d]", num_hops, RG_MAX_HOPS);
    RG_REQUIRE(ctx, csr->num_nodes >= 0 && csr->num_nodes <= (int64_t)RG_ROW_MASK + 1, "rg_sample_blocks: num_nodes out of range");
    RG_REQUIRE(ctx, csr->num_edges >= 0, "rg_sample_blocks: num_edges is negative");
    RG_REQUIRE(ctx, csr->row_ptr_bits == 32 || csr->row_ptr_bits == 64, "rg_sample_blocks: row_ptr_bits must be 32 or 64");
    RG_REQUIRE(ctx, csr->row_ptr_bits == 64 || csr->num_edges < (1ll << 31), "rg_sample_blocks: 32-bit row_ptr with >= 2^31 edges");
    RG_REQUIRE(ctx, csr->row_ptr && (csr->col_idx || csr->num_edges == 0), "rg_sample_blocks: null CSR array");
    for (int h = 0; h < num_hops; ++h)
        RG_REQUIRE(ctx, fanouts[h] == RG_FANOUT_ALL || (fanouts[h] >= 0 && fanouts[h] <= RG_MAX_FANOUT),
                   "rg_sample_blocks: fanouts[%d] = %d not in [0,%d] and not RG_FANOUT_ALL", h, fanouts[h], RG_MAX_FANOUT);
    // static bounds: per batch for the capacity checks, their maximum for the launch shapes
    int64_t fub_max[RG_MAX_HOPS + 1] = {0}, eub_max[RG_MAX_HOPS] = {0};
    int32_t seeds_max = 0;
    bool capacity_error = false;
    for (int g = 0; g < group; ++g) {
        rg_blocks* o = out + g;
        RG_REQUIRE(ctx, num_seeds[g] >= 0, "rg_sample_blocks: num_seeds is negative (batch %d)", g);
        RG_REQUIRE(ctx, num_seeds[g] <= csr->num_nodes, "rg_sample_blocks: more seeds than nodes (seeds must be distinct; batch %d)", g);
        RG_REQUIRE(ctx, seeds[g] || num_seeds[g] == 0, "rg_sample_blocks: seeds is NULL (batch %d)", g);
        RG_REQUIRE(ctx, o->nodes && o->tier_off && o->indptr && o->indptr_cap && o->nbr && o->nbr_cap,
                   "rg_sample_blocks: null output pointer (batch %d)", g);
        int64_t fub[RG_MAX_HOPS + 1], eub[RG_MAX_HOPS];
        rg_blocks_bounds(csr->num_nodes, csr->num_edges, num_seeds[g], fanouts, num_hops, fub, eub);
        bool too_small = o->nodes_cap < fub[num_hops];
        for (int h = 0; h < num_hops; ++h) {
            RG_REQUIRE(ctx, eub[h] < (1ll << 31), "rg_sample_blocks: hop %d may produce >= 2^31 edges", h);
            RG_REQUIRE(ctx, o->indptr[h] && (o->nbr[h] || eub[h] == 0), "rg_sample_blocks: null buffer for hop %d (batch %d)", h, g);
            RG_REQUIRE(ctx, !o->nbr_local || o->nbr_local[h] || eub[h] == 0, "rg_sample_blocks: nbr_local[%d] is NULL (batch %d)", h, g);
            too_small = too_small || o->indptr_cap[h] < fub[h] + 1 || o->nbr_cap[h] < eub[h];
            eub_max[h] = rg_max64(eub_max[h], eub[h]);
        }
        if (too_small) {
            // the required sizes go back to the caller in place of the capacities that were passed in
            rg_set_error(ctx, RG_ERR_CAPACITY, "rg_sample_blocks: output buffers of batch %d are below the static bounds "
                         "(nodes_cap %lld < %lld, or a hop's indptr_cap / nbr_cap); the required sizes were written back",
                         g, (long long)o->nodes_cap, (long long)fub[num_hops]);
            o->nodes_cap = fub[num_hops];
            for (int h = 0; h < num_hops; ++h) { o->indptr_cap[h] = fub[h] + 1; o->nbr_cap[h] = eub[h]; }
            capacity_error = true;
        }
        for (int h = 0; h <= num_hops; ++h) fub_max[h] = rg_max64(fub_max[h], fub[h]);
        seeds_max = num_seeds[g] > seeds_max ? num_seeds[g] : seeds_max;
    }
    if (capacity_error) return RG_ERR_CAPACITY;

    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int64_t N = csr->num_nodes;
    int64_t max_edges = 0;
    if (first_seen)
        for (int h = 0; h < num_hops; ++h) max_edges = rg_max64(max_edges, eub_max[h]);
    SampleScratch S;
    sampler_scratch_shape(N, fub_max[num_hops], max_edges, S);
    const int64_t words = S.words;
    const int tier_blocks = (int)rg_max64(1, rg_div_up(words, kWordsPerBlock));
    ctx->last_sample_group = 0;                       // no membership bitmaps to add until this call has been queued
    rg_status st = rg_sampler_reserve(ctx, N, fub_max[num_hops], group, max_edges, first_seen);
    if (st != RG_OK) return st;
    S.first_key = first_seen ? (int32_t*)ctx->first_key.p : nullptr;
    S.group = group;
    S.xcd_map = ctx->knobs.xcd_map;
    S.visited = (uint32_t*)ctx->visited.p;
    S.marked = (uint32_t*)ctx->marked.p;
    S.pos = (int32_t*)ctx->pos.p;
    S.chunk_sum = (int32_t*)ctx->chunk_sum.p;
    S.row_start = (int64_t*)ctx->row_start.p;
    S.row_deg = (int32_t*)ctx->row_deg.p;
    const uint32_t k0 = (uint32_t)(seed & 0xffffffffu), k1 = (uint32_t)(seed >> 32);
    const bool rp64 = csr->row_ptr_bits == 64;

    SampleGroup G;
    for (int g = 0; g < kMaxGroup; ++g) {
        const bool live = g < group;
        G.seeds[g] = live ? seeds[g] : nullptr;
        G.num_seeds[g] = live ? num_seeds[g] : 0;
        G.nodes[g] = live ? out[g].nodes : nullptr;
        G.tier_off[g] = live ? out[g].tier_off : nullptr;
        G.indptr[g] = G.nbr[g] = G.nbr_local[g] = G.edges_out[g] = nullptr;
    }
    const unsigned ug = (unsigned)group;

    if (words > 0) {
        if (ctx->sampler_dirty && ctx->first_key.bytes) {   // an earlier first-seen call stopped between a draw kernel and its emit
            const int64_t key_words = (int64_t)(ctx->first_key.bytes / 4);
            k_clear_words<<<(int)rg_div_up(key_words, 256), 256, 0, s>>>((uint32_t*)ctx->first_key.p, key_words);
            RG_LAUNCH_CHECK(ctx, "k_clear_words");
        }
        ctx->sampler_dirty = true;       // cleared again when every launch of this call has been queued
        const int64_t group_words = (int64_t)group * words;
        k_clear_words<<<(int)rg_div_up(group_words, 256), 256, 0, s>>>(S.visited, group_words);
        RG_LAUNCH_CHECK(ctx, "k_clear_words");
        if (!first_seen) {
            k_clear_words<<<(int)rg_div_up(group_words, 256), 256, 0, s>>>(S.marked, group_words);
            RG_LAUNCH_CHECK(ctx, "k_clear_words");
        }
    }
    k_mark_seeds<<<(unsigned)(grid_for(seeds_max, 256, 1 << 30)) * ug, 256, 0, s>>>(G, S);
    RG_LAUNCH_CHECK(ctx, "k_mark_seeds");

    for (int h = 0; h < num_hops; ++h) {
        bool any_local = false;
        for (int g = 0; g < group; ++g) {
            G.indptr[g] = out[g].indptr[h];
            G.nbr[g] = out[g].nbr[h];
            G.nbr_local[g] = out[g].nbr_local ? out[g].nbr_local[h] : nullptr;
            G.edges_out[g] = out[g].num_edges ? out[g].num_edges + h : nullptr;
            any_local = any_local || G.nbr_local[g];
        }
        const unsigned count_blocks = (unsigned)grid_for(fub_max[h], kChunk, 1ll << 30);
        if (rp64)
            k_hop_count<int64_t><<<count_blocks * ug, kChunk, 0, s>>>((const int64_t*)csr->row_ptr, G, S, h, fanouts[h]);
        else
            k_hop_count<int32_t><<<count_blocks * ug, kChunk, 0, s>>>((const int32_t*)csr->row_ptr, G, S, h, fanouts[h]);
        RG_LAUNCH_CHECK(ctx, "k_hop_count");
        // chunk sums -> exclusive offsets; total edge count -> indptr[n_h]
        k_scan_hop<<<ug, 1024, 0, s>>>(G, S, h);
        RG_LAUNCH_CHECK(ctx, "k_scan_hop");

        const int tok = rg_prof_begin(ctx, RG_K_SAMPLE, s);
        const int F = fanouts[h];
        if (F >= 1 && F <= 32 && csr->num_edges < (1ll << 32)) {
            const int kmax = F <= 8 ? 8 : (F <= 16 ? 16 : 32);
            const size_t lds = (size_t)kChunk * F * sizeof(uint32_t);
#define RG_LAUNCH_FAST(KM, FS)                                                                                        \
    k_hop_sample_thread<KM, FS><<<count_blocks * ug, kChunk, lds, s>>>(csr->col_idx, G, S, F, (uint32_t)h, k0, k1, epoch)
            if (first_seen) { if (kmax == 8) RG_LAUNCH_FAST(8, true); else if (kmax == 16) RG_LAUNCH_FAST(16, true); else RG_LAUNCH_FAST(32, true); }
            else { if (kmax == 8) RG_LAUNCH_FAST(8, false); else if (kmax == 16) RG_LAUNCH_FAST(16, false); else RG_LAUNCH_FAST(32, false); }
#undef RG_LAUNCH_FAST
        } else {
            const unsigned sample_blocks = (unsigned)grid_for(fub_max[h], 1, (int64_t)ctx->num_cus * 64);
            if (first_seen)
                k_hop_sample_wave<true><<<sample_blocks * ug, RG_WAVE, 0, s>>>(csr->col_idx, G, S, F, (uint32_t)h, k0, k1, epoch);
            else
                k_hop_sample_wave<false><<<sample_blocks * ug, RG_WAVE, 0, s>>>(csr->col_idx, G, S, F, (uint32_t)h, k0, k1, epoch);
        }
        rg_prof_end(ctx, tok, s);
        RG_LAUNCH_CHECK(ctx, "k_hop_sample");

        if (first_seen) {
            // new tier: edges that open a node, counted per block of the edge list, scanned, emitted in edge order
            const int fs_blocks = (int)rg_max64(1, rg_div_up(eub_max[h], kEdgesPerBlock));
            k_first_seen_count<<<(unsigned)(fs_blocks) * ug, 256, 0, s>>>(G, S, h);
            RG_LAUNCH_CHECK(ctx, "k_first_seen_count");
            k_scan_tier<<<ug, 1024, 0, s>>>(G, S, h, fs_blocks);
            RG_LAUNCH_CHECK(ctx, "k_scan_tier");
            k_first_seen_emit<<<(unsigned)(fs_blocks) * ug, 256, 0, s>>>(G, S, h);
            RG_LAUNCH_CHECK(ctx, "k_first_seen_emit");
        } else {
            // new tier: count fresh bits per block, scan, emit ascending
            k_tier_count<<<(unsigned)(tier_blocks) * ug, 256, 0, s>>>(S);
            RG_LAUNCH_CHECK(ctx, "k_tier_count");
            k_scan_tier<<<ug, 1024, 0, s>>>(G, S, h, tier_blocks);
            RG_LAUNCH_CHECK(ctx, "k_scan_tier");
            k_tier_emit<<<(unsigned)(tier_blocks) * ug, 256, 0, s>>>(G, S, h);
            RG_LAUNCH_CHECK(ctx, "k_tier_emit");
        }

        if (any_local && eub_max[h] > 0) {
            k_relabel<<<(unsigned)(grid_for(eub_max[h], 256, (int64_t)ctx->num_cus * 16)) * ug, 256, 0, s>>>(G, S, h);
            RG_LAUNCH_CHECK(ctx, "k_relabel");
        }
    }
    ctx->sampler_dirty = false;
    ctx->last_sample_group = group;
    ctx->last_sample_nodes = N;
    return RG_OK;
}

rg_status rg_access_histogram_sampled(rg_ctx* ctx, int32_t group, const int32_t* batch_index, uint32_t* counts,
                                      uint32_t* first_batch, int64_t num_nodes, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, group >= 1 && group <= RG_MAX_GROUP, "rg_access_histogram_sampled: group = %d not in [1,%d]", group, RG_MAX_GROUP);
    RG_REQUIRE(ctx, counts && (batch_index || !first_batch), "rg_access_histogram_sampled: null counts, or first_batch without batch_index");
    if (ctx->last_sample_group != group || ctx->last_sample_nodes != num_nodes)
        return rg_set_error(ctx, RG_ERR_STATE, "rg_access_histogram_sampled: the last sampling call of this context covered %d "
                            "batches on %lld nodes, not %d on %lld", ctx->last_sample_group, (long long)ctx->last_sample_nodes,
                            group, (long long)num_nodes);
    BatchIndices batch;
    for (int g = 0; g < kMaxGroup; ++g) {
        RG_REQUIRE(ctx, g >= group || !batch_index || batch_index[g] >= 0, "rg_access_histogram_sampled: negative batch index");
        batch.v[g] = g < group && batch_index ? (uint32_t)batch_index[g] : 0u;
    }
    if (num_nodes == 0) return RG_OK;
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int64_t words = rg_div_up(num_nodes, 32);
    const int tok = rg_prof_begin(ctx, RG_K_HISTOGRAM, s);
    k_histogram_bitmaps<<<grid_for(words, 256, (int64_t)ctx->num_cus * 16), 256, 0, s>>>((const uint32_t*)ctx->visited.p, words, group,
                                                                                         batch, counts, first_batch, num_nodes);
    rg_prof_end(ctx, tok, s);
    RG_LAUNCH_CHECK(ctx, "k_histogram_bitmaps");
    return RG_OK;
}

rg_status rg_sample_blocks(rg_ctx* ctx, const rg_csr* csr, const int32_t* seeds, int32_t num_seeds,
                           const int32_t* fanouts, int32_t num_hops, uint64_t seed, uint32_t epoch,
                           rg_blocks* out, void* stream) {
    return rg_sample_blocks_group(ctx, csr, 1, &seeds, &num_seeds, fanouts, num_hops, seed, epoch, RG_ORDER_ASCENDING, out, stream);
}

}  // extern "C"
