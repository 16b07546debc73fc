// Access-frequency histogram (Section IV, offline stage), TopHot selection (Alg. 1 line 3) and the
// bulk pull of the selected rows into the HBM cache (VectorPull, Alg. 1 line 4).
#include "rg_rowcopy.h"

namespace {

// ---------------------------------------------------------------------------- histogram
__global__ void __launch_bounds__(256) k_histogram(const int32_t* __restrict__ nodes, int64_t n, const int32_t* __restrict__ n_dev,
                                                   uint32_t* __restrict__ counts) {
    int64_t n_act = n;
    if (n_dev) { const int64_t d = *n_dev; n_act = d < n ? d : n; }
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_act; i += (int64_t)gridDim.x * blockDim.x)
        atomicAdd(&counts[nodes[i]], 1u);
}

// ---------------------------------------------------------------------------- radix select
// Finds the count threshold T of the K_eff-th best candidate, most significant byte first.
struct TopkCtl {
    uint32_t prefix;     // resolved high bytes of T
    uint32_t need;       // how many of the candidates matching the prefix are still to be taken
    uint32_t k_eff;
    uint32_t pad;
    uint32_t hist[4][256];
};

__device__ __forceinline__ bool rg_is_candidate(uint32_t home_word, uint32_t count) {
    return (home_word >> RG_TAG_SHIFT) == RG_TAG_REMOTE && count >= 1u;
}

__global__ void __launch_bounds__(256) k_topk_init(TopkCtl* __restrict__ ctl) {
    for (int i = threadIdx.x; i < 4 * 256; i += 256) (&ctl->hist[0][0])[i] = 0u;
    if (threadIdx.x == 0) { ctl->prefix = 0u; ctl->need = 0u; ctl->k_eff = 0u; ctl->pad = 0u; }
}

// Histogram of byte `pass` (0 = most significant) of the counts of candidates that match the prefix.
__global__ void __launch_bounds__(256) k_topk_hist(const uint32_t* __restrict__ counts, const int32_t* __restrict__ home, int64_t n,
                                                   int pass, TopkCtl* __restrict__ ctl) {
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0u;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    const uint32_t prefix = ctl->prefix;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t c = counts[v];
        if (!rg_is_candidate((uint32_t)home[v], c)) continue;
        if (pass > 0 && (c >> (shift + 8)) != (prefix >> (shift + 8))) continue;
        atomicAdd(&h[(c >> shift) & 255u], 1u);
    }
    __syncthreads();
    const uint32_t mine = h[threadIdx.x];
    if (mine) atomicAdd(&ctl->hist[pass][threadIdx.x], mine);
}

// One workgroup: pick the byte value holding the need-th largest remaining candidate.
__global__ void __launch_bounds__(256) k_topk_pick(TopkCtl* __restrict__ ctl, int pass, int64_t capacity, int64_t* __restrict__ num_cached) {
    __shared__ uint32_t h[256];
    __shared__ uint32_t above[256];      // candidates in strictly larger byte values
    __shared__ uint32_t need_s;
    h[threadIdx.x] = ctl->hist[pass][threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int d = 255; d >= 0; --d) { above[d] = run; run += h[d]; }
        uint32_t need0 = ctl->need;
        if (pass == 0) {                 // run = number of candidates
            const uint64_t k = (uint64_t)capacity < (uint64_t)run ? (uint64_t)capacity : (uint64_t)run;
            ctl->k_eff = (uint32_t)k;
            ctl->need = (uint32_t)k;
            *num_cached = (int64_t)k;
            need0 = (uint32_t)k;
        }
        need_s = need0;
    }
    __syncthreads();
    const uint32_t need = need_s;
    const int shift = 24 - 8 * pass;
    if (need == 0u) {
        // nothing to select: a threshold no count can exceed or tie with a positive quota
        if (threadIdx.x == 0 && pass == 3) ctl->prefix = 0xFFFFFFFFu;
        return;
    }
    const int d = threadIdx.x;
    if (above[d] < need && need <= above[d] + h[d]) {     // exactly one byte value satisfies this
        ctl->prefix |= (uint32_t)d << shift;
        ctl->need = need - above[d];
    }
}

constexpr int kNodesPerBlock = 1024;   // 256 threads x 4 consecutive nodes

// Per block: number of candidates above the threshold and number tied with it.
__global__ void __launch_bounds__(256) k_topk_count(const uint32_t* __restrict__ counts, const int32_t* __restrict__ home, int64_t n,
                                                    const TopkCtl* __restrict__ ctl, int32_t* __restrict__ blk_gt, int32_t* __restrict__ blk_eq) {
    const uint32_t T = ctl->prefix;
    const int64_t v0 = (int64_t)blockIdx.x * kNodesPerBlock + threadIdx.x * 4;
    int gt = 0, eq = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t v = v0 + q;
        if (v < n) {
            const uint32_t c = counts[v];
            if (rg_is_candidate((uint32_t)home[v], c)) { gt += c > T; eq += c == T; }
        }
    }
    gt = rg_wave_sum(gt);
    eq = rg_wave_sum(eq);
    __shared__ int pg[4], pe[4];
    if (rg_lane() == 0) { pg[threadIdx.x >> 6] = gt; pe[threadIdx.x >> 6] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_gt[blockIdx.x] = pg[0] + pg[1] + pg[2] + pg[3];
        blk_eq[blockIdx.x] = pe[0] + pe[1] + pe[2] + pe[3];
    }
}

// One workgroup: exclusive scans of both per-block arrays, in place.
__global__ void __launch_bounds__(1024) k_topk_scan(int32_t* __restrict__ blk_gt, int32_t* __restrict__ blk_eq, int64_t nblocks) {
    __shared__ int smem[1024 / RG_WAVE + 1];
    __shared__ int carry_g, carry_e;
    if (threadIdx.x == 0) { carry_g = 0; carry_e = 0; }
    __syncthreads();
    for (int64_t base = 0; base < nblocks; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int g = i < nblocks ? blk_gt[i] : 0;
        const int e = i < nblocks ? blk_eq[i] : 0;
        int tg, te;
        const int xg = rg_block_excl_scan<1024 / RG_WAVE>(g, smem, &tg);
        const int xe = rg_block_excl_scan<1024 / RG_WAVE>(e, smem, &te);
        const int cg = carry_g, ce = carry_e;
        if (i < nblocks) { blk_gt[i] = cg + xg; blk_eq[i] = ce + xe; }
        __syncthreads();
        if (threadIdx.x == 0) { carry_g = cg + tg; carry_e = ce + te; }
        __syncthreads();
    }
}

// Selected = above the threshold, or tied with it and among the first `need` ties in id order.
// Slots are handed out in ascending id, so cache_ids comes out sorted.
__global__ void __launch_bounds__(256) k_topk_emit(const uint32_t* __restrict__ counts, const int32_t* __restrict__ home, int64_t n,
                                                   const TopkCtl* __restrict__ ctl, const int32_t* __restrict__ blk_gt,
                                                   const int32_t* __restrict__ blk_eq, int32_t* __restrict__ cache_ids,
                                                   int32_t* __restrict__ loc) {
    __shared__ int smem[256 / RG_WAVE + 1];
    const uint32_t T = ctl->prefix;
    const int need = (int)ctl->need;
    const int gt_before = blk_gt[blockIdx.x];
    const int eq_before = blk_eq[blockIdx.x];
    const int64_t v0 = (int64_t)blockIdx.x * kNodesPerBlock + threadIdx.x * 4;
    uint32_t hw[4];
    bool is_gt[4], is_eq[4];
    int eq_cnt = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t v = v0 + q;
        is_gt[q] = is_eq[q] = false;
        hw[q] = 0u;
        if (v < n) {
            const uint32_t c = counts[v];
            hw[q] = (uint32_t)home[v];
            if (rg_is_candidate(hw[q], c)) { is_gt[q] = c > T; is_eq[q] = c == T; }
        }
        eq_cnt += is_eq[q];
    }
    int tot;
    int eq_rank = eq_before + rg_block_excl_scan<256 / RG_WAVE>(eq_cnt, smem, &tot);
    bool sel[4];
    int sel_cnt = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        sel[q] = is_gt[q] || (is_eq[q] && eq_rank < need);
        eq_rank += is_eq[q];
        sel_cnt += sel[q];
    }
    int slot = gt_before + (eq_before < need ? eq_before : need) + rg_block_excl_scan<256 / RG_WAVE>(sel_cnt, smem, &tot);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t v = v0 + q;
        if (v >= n) break;
        if (sel[q]) {
            cache_ids[slot] = (int32_t)v;
            loc[v] = (int32_t)((RG_TAG_CACHE << RG_TAG_SHIFT) | (uint32_t)slot);
            ++slot;
        } else {
            loc[v] = (int32_t)hw[q];
        }
    }
}

// ---------------------------------------------------------------------------- VectorPull
// cache_rows[slot] = remote_store[row(home[cache_ids[slot]])] for slot < *num_cached.
template <int VEC>
__global__ void __launch_bounds__(256) k_cache_fill(const int32_t* __restrict__ cache_ids, const int32_t* __restrict__ home,
                                                    const int64_t* __restrict__ num_cached, const float* __restrict__ remote_store,
                                                    int64_t remote_stride, float* __restrict__ cache_rows, int64_t cache_stride,
                                                    int cpr, int log2L) {
    typedef typename RgVec<VEC>::type V;
    constexpr int U = 4;
    const int64_t n = *num_cached;
    const int lane = rg_lane();
    const int L = 1 << log2L;
    const int R = RG_WAVE >> log2L;            // rows per wave step
    const int sub = lane >> log2L;
    const int c0 = lane & (L - 1);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t row0 = wave * (R * U); row0 < n; row0 += nwaves * (R * U)) {
        const V* src[U];
        V* dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t slot = row0 + u * R + sub;
            src[u] = nullptr;
            dst[u] = nullptr;
            if (slot < n) {
                const uint32_t hw = (uint32_t)home[cache_ids[slot]];
                src[u] = (const V*)(remote_store + (int64_t)(hw & RG_ROW_MASK) * remote_stride);
                dst[u] = (V*)(cache_rows + slot * cache_stride);
            }
        }
        for (int c = c0; c < cpr; c += L) {
            V val[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (src[u]) val[u] = src[u][c];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u]) dst[u][c] = val[u];
        }
    }
}

}  // namespace

extern "C" {

rg_status rg_access_histogram(rg_ctx* ctx, const int32_t* nodes, int64_t n, const int32_t* n_dev, uint32_t* counts,
                              int64_t num_nodes, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, n >= 0 && num_nodes >= 0, "rg_access_histogram: negative size");
    if (n == 0) return RG_OK;
    RG_REQUIRE(ctx, nodes && counts, "rg_access_histogram: null pointer");
    RG_REQUIRE(ctx, num_nodes > 0, "rg_access_histogram: entries given but num_nodes is 0");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int grid = (int)rg_min64(rg_div_up(n, 256), (int64_t)ctx->num_cus * 32);
    const int tok = rg_prof_begin(ctx, RG_K_HISTOGRAM, s);
    k_histogram<<<grid, 256, 0, s>>>(nodes, n, n_dev, counts);
    rg_prof_end(ctx, tok, s);
    RG_LAUNCH_CHECK(ctx, "k_histogram");
    return RG_OK;
}

rg_status rg_build_cache(rg_ctx* ctx, const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                         const float* remote_store, int64_t remote_stride, int32_t dim, const rg_cache* cache,
                         void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, cache, "rg_build_cache: cache is NULL");
    RG_REQUIRE(ctx, num_nodes >= 0 && num_nodes <= (int64_t)RG_ROW_MASK + 1, "rg_build_cache: num_nodes out of range");
    RG_REQUIRE(ctx, cache->capacity_rows >= 0 && cache->capacity_rows <= (int64_t)RG_ROW_MASK + 1,
               "rg_build_cache: capacity_rows = %lld out of range", (long long)cache->capacity_rows);
    RG_REQUIRE(ctx, dim >= 1, "rg_build_cache: dim = %d must be positive", dim);
    RG_REQUIRE(ctx, cache->row_stride >= dim && remote_stride >= dim, "rg_build_cache: row stride smaller than dim");
    RG_REQUIRE(ctx, cache->num_cached, "rg_build_cache: num_cached is NULL");
    RG_REQUIRE(ctx, num_nodes == 0 || (counts && home && cache->loc), "rg_build_cache: null node array");
    const bool may_select = cache->capacity_rows > 0 && num_nodes > 0;
    RG_REQUIRE(ctx, !may_select || (cache->cache_ids && cache->cache_rows && remote_store), "rg_build_cache: null cache buffer");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;

    const int64_t nblocks = rg_max64(1, rg_div_up(num_nodes, kNodesPerBlock));
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->topk_ctl, sizeof(TopkCtl))) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->topk_blk, (size_t)nblocks * 8)) != RG_OK) return st;
    TopkCtl* ctl = (TopkCtl*)ctx->topk_ctl.p;
    int32_t* blk_gt = (int32_t*)ctx->topk_blk.p;
    int32_t* blk_eq = blk_gt + nblocks;

    k_topk_init<<<1, 256, 0, s>>>(ctl);
    RG_LAUNCH_CHECK(ctx, "k_topk_init");
    const int hist_grid = (int)rg_max64(1, rg_min64(rg_div_up(num_nodes, 256 * 8), (int64_t)ctx->num_cus * 8));
    for (int pass = 0; pass < 4; ++pass) {
        k_topk_hist<<<hist_grid, 256, 0, s>>>(counts, home, num_nodes, pass, ctl);
        RG_LAUNCH_CHECK(ctx, "k_topk_hist");
        k_topk_pick<<<1, 256, 0, s>>>(ctl, pass, cache->capacity_rows, cache->num_cached);
        RG_LAUNCH_CHECK(ctx, "k_topk_pick");
    }
    k_topk_count<<<(int)nblocks, 256, 0, s>>>(counts, home, num_nodes, ctl, blk_gt, blk_eq);
    RG_LAUNCH_CHECK(ctx, "k_topk_count");
    k_topk_scan<<<1, 1024, 0, s>>>(blk_gt, blk_eq, nblocks);
    RG_LAUNCH_CHECK(ctx, "k_topk_scan");
    k_topk_emit<<<(int)nblocks, 256, 0, s>>>(counts, home, num_nodes, ctl, blk_gt, blk_eq, cache->cache_ids, cache->loc);
    RG_LAUNCH_CHECK(ctx, "k_topk_emit");

    if (may_select) {
        const void* ptrs[2] = {remote_store, cache->cache_rows};
        const int64_t strides[2] = {remote_stride, cache->row_stride};
        const int vec = rg_pick_vec(dim, ptrs, 2, strides, 2);
        const RgRowShape shp = rg_row_shape(dim, vec);
        const int64_t rows_ub = rg_min64(cache->capacity_rows, num_nodes);
        const int rows_per_block = 4 * (RG_WAVE >> shp.log2L) * 4;
        const int grid = (int)rg_max64(1, rg_min64(rg_div_up(rows_ub, rows_per_block), (int64_t)ctx->num_cus * 16));
        const int tok = rg_prof_begin(ctx, RG_K_CACHE_FILL, s);
        if (vec == 4)
            k_cache_fill<4><<<grid, 256, 0, s>>>(cache->cache_ids, home, cache->num_cached, remote_store, remote_stride, cache->cache_rows, cache->row_stride, shp.cpr, shp.log2L);
        else if (vec == 2)
            k_cache_fill<2><<<grid, 256, 0, s>>>(cache->cache_ids, home, cache->num_cached, remote_store, remote_stride, cache->cache_rows, cache->row_stride, shp.cpr, shp.log2L);
        else
            k_cache_fill<1><<<grid, 256, 0, s>>>(cache->cache_ids, home, cache->num_cached, remote_store, remote_stride, cache->cache_rows, cache->row_stride, shp.cpr, shp.log2L);
        rg_prof_end(ctx, tok, s);
        RG_LAUNCH_CHECK(ctx, "k_cache_fill");
    }
    return RG_OK;
}

}  // extern "C"
