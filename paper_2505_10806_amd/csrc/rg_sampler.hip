// Epoch schedule and multi-hop neighbour sampling (Alg. 1 line 1; SAMPLE(eta(v), k) of Section II-B).
//
// Data layout in HBM: CSR (row_ptr int32/int64, col_idx int32) is read-only; the batch's cumulative
// frontier `nodes` grows tier by tier; membership lives in two N-bit bitmaps (`visited` = members of
// the cumulative frontier, `fresh` = ids first seen in the current hop) and `pos[v]` maps a member to
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

// ---------------------------------------------------------------------------- batch start
__global__ void __launch_bounds__(256) k_clear_words(uint32_t* __restrict__ w, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0u;
}

__global__ void __launch_bounds__(256) k_mark_seeds(const int32_t* __restrict__ seeds, int32_t num_seeds,
                                                    int32_t* __restrict__ nodes, int32_t* __restrict__ pos,
                                                    uint32_t* __restrict__ visited, int32_t* __restrict__ tier_off) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) { tier_off[0] = 0; tier_off[1] = num_seeds; }
    if (i >= num_seeds) return;
    const int32_t v = seeds[i];
    nodes[i] = v;
    pos[v] = i;
    atomicOr(&visited[(uint32_t)v >> 5], 1u << (v & 31));
}

// ---------------------------------------------------------------------------- per hop: sizes
// indptr[i] = exclusive prefix of m within the node's 256-node chunk; chunk_sum[b] = chunk total;
// row_start[i], row_deg[i] = the node's adjacency row.
template <typename RP>
__global__ void __launch_bounds__(kChunk) k_hop_count(const RP* __restrict__ row_ptr, const int32_t* __restrict__ nodes,
                                                      const int32_t* __restrict__ n_frontier_ptr, int fanout,
                                                      int32_t* __restrict__ indptr, int32_t* __restrict__ chunk_sum,
                                                      int64_t* __restrict__ row_start, int32_t* __restrict__ row_deg) {
    __shared__ int smem[kChunk / RG_WAVE + 1];
    const int n_h = *n_frontier_ptr;
    const int64_t first = (int64_t)blockIdx.x * kChunk;
    if (first >= n_h) return;                       // uniform per workgroup
    const int64_t i = first + threadIdx.x;
    int m = 0;
    if (i < n_h) {
        int64_t start, deg;
        rg_row_extent(row_ptr, nodes[i], start, deg);
        m = (fanout < 0 || deg <= fanout) ? (int)deg : fanout;
        row_start[i] = start;             // kept for the draw kernel: one coalesced read there instead of a second
        row_deg[i] = (int32_t)deg;        // random lookup of row_ptr
    }
    int total;
    const int excl = rg_block_excl_scan<kChunk / RG_WAVE>(m, smem, &total);
    if (i < n_h) indptr[i] = excl;
    if (threadIdx.x == 0) chunk_sum[blockIdx.x] = total;
}

// In-place exclusive scan of data[0..n) by one workgroup, n = ceil(count / per) with count = *count_ptr
// (or fixed_count when count_ptr is NULL).  The grand total plus *base_ptr (or 0) is stored to
// total_out[count] when total_at_count is set (the edge total behind the last indptr entry), else to
// total_out[0].
__global__ void __launch_bounds__(1024) k_scan_sums(int32_t* __restrict__ data, const int32_t* __restrict__ count_ptr,
                                                    int64_t fixed_count, int per, const int32_t* __restrict__ base_ptr,
                                                    int32_t* __restrict__ total_out, int total_at_count,
                                                    int32_t* __restrict__ total_copy) {
    __shared__ int smem[1024 / RG_WAVE + 1];
    __shared__ int carry_s;
    const int64_t count = count_ptr ? (int64_t)*count_ptr : fixed_count;
    const int64_t n = (count + per - 1) / per;
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
    if (threadIdx.x == 0) {
        const int b = base_ptr ? *base_ptr : 0;
        const int64_t slot = total_at_count ? count : 0;
        total_out[slot] = b + carry_s;
        if (total_copy) *total_copy = b + carry_s;
    }
}

// ---------------------------------------------------------------------------- per hop: draw + read
__device__ __forceinline__ void rg_mark_fresh(int32_t u, const uint32_t* __restrict__ visited, uint32_t* __restrict__ fresh) {
    const uint32_t w = (uint32_t)u >> 5, bit = 1u << (u & 31);
    if (visited[w] & bit) return;
    if (fresh[w] & bit) return;                       // a stale read only costs a redundant atomic
    atomicOr(&fresh[w], bit);
}

// General sampler: one wavefront (= one 64-thread workgroup) per frontier node, any fan-out up to
// RG_MAX_FANOUT.  The Floyd set lives in LDS; step i tests membership of t with all lanes.
__global__ void __launch_bounds__(RG_WAVE) k_hop_sample_wave(const int64_t* __restrict__ row_start, const int32_t* __restrict__ row_deg,
                                                            const int32_t* __restrict__ col_idx, const int32_t* __restrict__ nodes,
                                                            const int32_t* __restrict__ n_frontier_ptr, int fanout, uint32_t hop,
                                                            uint32_t k0, uint32_t k1, uint32_t epoch,
                                                            int32_t* __restrict__ indptr, const int32_t* __restrict__ chunk_sum,
                                                            int32_t* __restrict__ nbr, const uint32_t* __restrict__ visited,
                                                            uint32_t* __restrict__ fresh) {
    __shared__ uint32_t draws[RG_MAX_FANOUT];
    __shared__ uint32_t chosen[RG_MAX_FANOUT];
    const int n_h = *n_frontier_ptr;
    const int lane = threadIdx.x;
    for (int64_t i = blockIdx.x; i < n_h; i += gridDim.x) {
        const int32_t v = nodes[i];
        const int64_t start = row_start[i], deg = row_deg[i];
        const int base = indptr[i] + chunk_sum[i / kChunk];
        __syncthreads();                               // every lane has read indptr[i] before it is rewritten
        if (lane == 0) indptr[i] = base;
        if (fanout < 0 || deg <= fanout) {             // whole row, CSR order
            for (int64_t t = lane; t < deg; t += RG_WAVE) {
                const int32_t u = col_idx[start + t];
                nbr[base + t] = u;
                rg_mark_fresh(u, visited, fresh);
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
            rg_mark_fresh(u, visited, fresh);
        }
    }
}

// Fast sampler for fan-outs up to 32 on graphs with fewer than 2^32 edges: one thread per frontier node
// draws (Philox + Floyd entirely in registers), the 256 nodes of a workgroup stage the col_idx offsets
// of their picks in LDS in output order, then the whole workgroup reads col_idx and writes nbr with
// consecutive lanes on consecutive output slots.
template <int KMAX>
__global__ void __launch_bounds__(kChunk) k_hop_sample_thread(const int64_t* __restrict__ row_start, const int32_t* __restrict__ row_deg,
                                                              const int32_t* __restrict__ col_idx, const int32_t* __restrict__ nodes,
                                                              const int32_t* __restrict__ n_frontier_ptr, int fanout, uint32_t hop,
                                                              uint32_t k0, uint32_t k1, uint32_t epoch,
                                                              int32_t* __restrict__ indptr, const int32_t* __restrict__ chunk_sum,
                                                              int32_t* __restrict__ nbr, const uint32_t* __restrict__ visited,
                                                              uint32_t* __restrict__ fresh) {
    extern __shared__ uint32_t staged[];                 // kChunk * fanout col_idx offsets
    const int n_h = *n_frontier_ptr;
    const int64_t first = (int64_t)blockIdx.x * kChunk;
    if (first >= n_h) return;                            // uniform per workgroup
    const int64_t i = first + threadIdx.x;
    const int k = fanout;
    // chunk_sum[b] is the exclusive offset of chunk b; the chunk's edge count follows from its successor
    // (or from the hop total behind the last indptr entry for the last chunk)
    const int base = chunk_sum[blockIdx.x];
    const bool last_chunk = first + kChunk >= n_h;
    const int chunk_edges = (last_chunk ? indptr[n_h] : chunk_sum[blockIdx.x + 1]) - base;
    if (i < n_h) {
        const int32_t v = nodes[i];
        const int64_t start = row_start[i], deg = row_deg[i];
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
        rg_mark_fresh(u, visited, fresh);
    }
}

// ---------------------------------------------------------------------------- per hop: new tier
__global__ void __launch_bounds__(256) k_tier_count(const uint32_t* __restrict__ fresh, int64_t words,
                                                    int32_t* __restrict__ blk_sum) {
    const int64_t w0 = (int64_t)blockIdx.x * kWordsPerBlock + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (w0 + q < words) c += __popc(fresh[w0 + q]);
    c = rg_wave_sum(c);
    __shared__ int part[4];
    if (rg_lane() == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) blk_sum[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// Emit the ids of `fresh` in ascending order behind the current frontier, record their positions,
// fold `fresh` into `visited` and leave `fresh` all-zero.  blk_sum holds exclusive block offsets.
__global__ void __launch_bounds__(256) k_tier_emit(uint32_t* __restrict__ fresh, uint32_t* __restrict__ visited, int64_t words,
                                                   const int32_t* __restrict__ blk_sum, const int32_t* __restrict__ tier_start_ptr,
                                                   int32_t* __restrict__ nodes, int32_t* __restrict__ pos) {
    __shared__ int smem[256 / RG_WAVE + 1];
    const int64_t w0 = (int64_t)blockIdx.x * kWordsPerBlock + threadIdx.x * 4;
    uint32_t bits[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        bits[q] = (w0 + q < words) ? fresh[w0 + q] : 0u;
        c += __popc(bits[q]);
    }
    int total;
    const int excl = rg_block_excl_scan<256 / RG_WAVE>(c, smem, &total);
    if (total == 0) return;                          // uniform: nothing fresh in this block
    int out = *tier_start_ptr + blk_sum[blockIdx.x] + excl;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t b = bits[q];
        if (b == 0u) continue;
        visited[w0 + q] |= b;
        fresh[w0 + q] = 0u;
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

// nbr_local[e] = position of nbr[e] in the extended frontier; the hop's edge count is indptr[n_h].
__global__ void __launch_bounds__(256) k_relabel(const int32_t* __restrict__ nbr, const int32_t* __restrict__ indptr,
                                                 const int32_t* __restrict__ n_frontier_ptr, const int32_t* __restrict__ pos,
                                                 int32_t* __restrict__ nbr_local) {
    const int n = indptr[*n_frontier_ptr];
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
        nbr_local[e] = pos[nbr[e]];
}

int grid_for(int64_t work_items, int per_block, int64_t cap) {
    int64_t g = rg_div_up(work_items, per_block);
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

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

rg_status rg_sample_blocks(rg_ctx* ctx, const rg_csr* csr, const int32_t* seeds, int32_t num_seeds,
                           const int32_t* fanouts, int32_t num_hops, uint64_t seed, uint32_t epoch,
                           const rg_blocks* out, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, csr && out && fanouts, "rg_sample_blocks: null argument");
    RG_REQUIRE(ctx, num_hops >= 1 && num_hops <= RG_MAX_HOPS, "rg_sample_blocks: num_hops = %d not in [1,%d]", num_hops, RG_MAX_HOPS);
    RG_REQUIRE(ctx, num_seeds >= 0, "rg_sample_blocks: num_seeds is negative");
    RG_REQUIRE(ctx, csr->num_nodes >= 0 && csr->num_nodes <= (int64_t)RG_ROW_MASK + 1, "rg_sample_blocks: num_nodes out of range");
    RG_REQUIRE(ctx, csr->num_edges >= 0, "rg_sample_blocks: num_edges is negative");
    RG_REQUIRE(ctx, csr->row_ptr_bits == 32 || csr->row_ptr_bits == 64, "rg_sample_blocks: row_ptr_bits must be 32 or 64");
    RG_REQUIRE(ctx, csr->row_ptr_bits == 64 || csr->num_edges < (1ll << 31), "rg_sample_blocks: 32-bit row_ptr with >= 2^31 edges");
    RG_REQUIRE(ctx, csr->row_ptr && (csr->col_idx || csr->num_edges == 0), "rg_sample_blocks: null CSR array");
    RG_REQUIRE(ctx, num_seeds <= csr->num_nodes, "rg_sample_blocks: more seeds than nodes (seeds must be distinct)");
    RG_REQUIRE(ctx, seeds || num_seeds == 0, "rg_sample_blocks: seeds is NULL");
    RG_REQUIRE(ctx, out->nodes && out->tier_off && out->indptr && out->indptr_cap && out->nbr && out->nbr_cap,
               "rg_sample_blocks: null output pointer");
    for (int h = 0; h < num_hops; ++h)
        RG_REQUIRE(ctx, fanouts[h] == RG_FANOUT_ALL || (fanouts[h] >= 0 && fanouts[h] <= RG_MAX_FANOUT),
                   "rg_sample_blocks: fanouts[%d] = %d not in [0,%d] and not RG_FANOUT_ALL", h, fanouts[h], RG_MAX_FANOUT);
    int64_t fub[RG_MAX_HOPS + 1], eub[RG_MAX_HOPS];
    rg_blocks_bounds(csr->num_nodes, csr->num_edges, num_seeds, fanouts, num_hops, fub, eub);
    for (int h = 0; h < num_hops; ++h) {
        RG_REQUIRE(ctx, eub[h] < (1ll << 31), "rg_sample_blocks: hop %d may produce >= 2^31 edges", h);
        RG_REQUIRE(ctx, out->indptr[h] && (out->nbr[h] || eub[h] == 0), "rg_sample_blocks: null buffer for hop %d", h);
        if (out->indptr_cap[h] < fub[h] + 1)
            return rg_set_error(ctx, RG_ERR_CAPACITY, "rg_sample_blocks: indptr_cap[%d] = %lld < %lld", h,
                                (long long)out->indptr_cap[h], (long long)(fub[h] + 1));
        if (out->nbr_cap[h] < eub[h])
            return rg_set_error(ctx, RG_ERR_CAPACITY, "rg_sample_blocks: nbr_cap[%d] = %lld < %lld", h,
                                (long long)out->nbr_cap[h], (long long)eub[h]);
        RG_REQUIRE(ctx, !out->nbr_local || out->nbr_local[h] || eub[h] == 0, "rg_sample_blocks: nbr_local[%d] is NULL", h);
    }
    if (out->nodes_cap < fub[num_hops])
        return rg_set_error(ctx, RG_ERR_CAPACITY, "rg_sample_blocks: nodes_cap = %lld < %lld", (long long)out->nodes_cap,
                            (long long)fub[num_hops]);

    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int64_t N = csr->num_nodes;
    const int64_t words = rg_div_up(N, 32);
    rg_status st = rg_reserve(ctx, N, fub[num_hops], 0);
    if (st != RG_OK) return st;
    uint32_t* visited = (uint32_t*)ctx->visited.p;
    uint32_t* fresh = (uint32_t*)ctx->fresh.p;
    int32_t* pos = (int32_t*)ctx->pos.p;
    int32_t* chunk_sum = (int32_t*)ctx->chunk_sum.p;
    int64_t* row_start = (int64_t*)ctx->row_start.p;
    int32_t* row_deg = (int32_t*)ctx->row_deg.p;
    const uint32_t k0 = (uint32_t)(seed & 0xffffffffu), k1 = (uint32_t)(seed >> 32);
    const bool rp64 = csr->row_ptr_bits == 64;

    if (words > 0) {
        if (ctx->sampler_dirty) {        // an earlier call stopped between a draw kernel and its tier emit
            k_clear_words<<<(int)rg_div_up(words, 256), 256, 0, s>>>(fresh, words);
            RG_LAUNCH_CHECK(ctx, "k_clear_words");
        }
        ctx->sampler_dirty = true;       // cleared again when every launch of this call has been queued
        k_clear_words<<<(int)rg_div_up(words, 256), 256, 0, s>>>(visited, words);
        RG_LAUNCH_CHECK(ctx, "k_clear_words");
    }
    k_mark_seeds<<<grid_for(num_seeds, 256, 1 << 30), 256, 0, s>>>(seeds, num_seeds, out->nodes, pos, visited, out->tier_off);
    RG_LAUNCH_CHECK(ctx, "k_mark_seeds");

    const int tier_blocks = (int)rg_max64(1, rg_div_up(words, kWordsPerBlock));
    for (int h = 0; h < num_hops; ++h) {
        const int32_t* n_frontier = out->tier_off + h + 1;
        const int count_blocks = grid_for(fub[h], kChunk, 1ll << 30);
        int32_t* indptr = out->indptr[h];
        if (rp64)
            k_hop_count<int64_t><<<count_blocks, kChunk, 0, s>>>((const int64_t*)csr->row_ptr, out->nodes, n_frontier, fanouts[h], indptr, chunk_sum, row_start, row_deg);
        else
            k_hop_count<int32_t><<<count_blocks, kChunk, 0, s>>>((const int32_t*)csr->row_ptr, out->nodes, n_frontier, fanouts[h], indptr, chunk_sum, row_start, row_deg);
        RG_LAUNCH_CHECK(ctx, "k_hop_count");
        // chunk sums -> exclusive offsets; total edge count -> indptr[n_h]
        k_scan_sums<<<1, 1024, 0, s>>>(chunk_sum, n_frontier, 0, kChunk, nullptr, indptr, 1, out->num_edges ? out->num_edges + h : nullptr);
        RG_LAUNCH_CHECK(ctx, "k_scan_sums");

        const int tok = rg_prof_begin(ctx, RG_K_SAMPLE, s);
        const int F = fanouts[h];
        if (F >= 1 && F <= 32 && csr->num_edges < (1ll << 32)) {
            const int kmax = F <= 8 ? 8 : (F <= 16 ? 16 : 32);
            const size_t lds = (size_t)kChunk * F * sizeof(uint32_t);
#define RG_LAUNCH_FAST(KM)                                                                                            \
    k_hop_sample_thread<KM><<<count_blocks, kChunk, lds, s>>>(row_start, row_deg, csr->col_idx, out->nodes, n_frontier, F,   \
                                                              (uint32_t)h, k0, k1, epoch, indptr, chunk_sum, out->nbr[h],  \
                                                              visited, fresh)
            if (kmax == 8) RG_LAUNCH_FAST(8); else if (kmax == 16) RG_LAUNCH_FAST(16); else RG_LAUNCH_FAST(32);
#undef RG_LAUNCH_FAST
        } else {
            const int sample_blocks = grid_for(fub[h], 1, (int64_t)ctx->num_cus * 64);
            k_hop_sample_wave<<<sample_blocks, RG_WAVE, 0, s>>>(row_start, row_deg, csr->col_idx, out->nodes, n_frontier, F, (uint32_t)h,
                                                                k0, k1, epoch, indptr, chunk_sum, out->nbr[h], visited, fresh);
        }
        rg_prof_end(ctx, tok, s);
        RG_LAUNCH_CHECK(ctx, "k_hop_sample");

        // new tier: count fresh bits per block, scan, emit ascending
        k_tier_count<<<tier_blocks, 256, 0, s>>>(fresh, words, chunk_sum);
        RG_LAUNCH_CHECK(ctx, "k_tier_count");
        k_scan_sums<<<1, 1024, 0, s>>>(chunk_sum, nullptr, tier_blocks, 1, n_frontier, out->tier_off + h + 2, 0, nullptr);
        RG_LAUNCH_CHECK(ctx, "k_scan_sums");
        k_tier_emit<<<tier_blocks, 256, 0, s>>>(fresh, visited, words, chunk_sum, n_frontier, out->nodes, pos);
        RG_LAUNCH_CHECK(ctx, "k_tier_emit");

        if (out->nbr_local && eub[h] > 0) {
            k_relabel<<<grid_for(eub[h], 256, (int64_t)ctx->num_cus * 16), 256, 0, s>>>(out->nbr[h], indptr, n_frontier, pos,
                                                                                       out->nbr_local[h]);
            RG_LAUNCH_CHECK(ctx, "k_relabel");
        }
    }
    ctx->sampler_dirty = false;
    return RG_OK;
}

}  // extern "C"
