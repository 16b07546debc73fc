// Per-batch feature assembly (Alg. 1 lines 12-14): rows of the batch's input nodes are copied from the
// local store (HBM), the steady cache (HBM) or, for misses only, the remote store (pinned host memory).
//
// Three kernels: classify resolves every output row to a location word (one random 4-byte read of loc[]
// per row), counts the three classes and compacts the indices of the miss rows; the HBM kernel copies
// local and cached rows; the miss kernel copies the remote rows and may run on a second stream so the
// host-link transfers overlap the HBM copies.
#include <stdlib.h>

#include "rg_rowcopy.h"

namespace {

__device__ __forceinline__ int64_t rg_actual_n(int64_t n, const int32_t* __restrict__ n_dev) {
    if (!n_dev) return n;
    const int64_t d = *n_dev;
    return d < n ? d : n;
}

// Batches classified by one launch: blockIdx.y selects the batch (its ticket's scratch slices).
struct ClassifyGroup {
    const int32_t* nodes[RG_GATHER_TICKETS];
    const int32_t* n_dev[RG_GATHER_TICKETS];
    int64_t n[RG_GATHER_TICKETS];
    uint32_t* src[RG_GATHER_TICKETS];
    int32_t* miss_list[RG_GATHER_TICKETS];
    uint32_t* gctl[RG_GATHER_TICKETS];
    unsigned long long* stats[RG_GATHER_TICKETS];
};

__global__ void k_gather_reset(const ClassifyGroup C) {
    const int k = blockIdx.x;
    if (threadIdx.x == 0) C.gctl[k][0] = 0u;
    if (threadIdx.x < 3) C.stats[k][threadIdx.x] = 0ull;
}

// Four rows per thread (row i0 + k*256 + threadIdx.x, k = 0..3) so that each thread has four independent
// loc[] lookups in flight; the miss pairs of a workgroup are appended in that visiting order (any order is valid).
constexpr int kClassifyRows = 4;

__global__ void __launch_bounds__(256) k_classify(const ClassifyGroup C, const int32_t* __restrict__ loc) {
    __shared__ int smem[256 / RG_WAVE + 1];
    __shared__ int cls[3][4];
    __shared__ uint32_t miss_base;
    const int b = blockIdx.y;
    const int32_t* __restrict__ nodes = C.nodes[b];
    uint32_t* __restrict__ src = C.src[b];
    int32_t* __restrict__ miss_list = C.miss_list[b];
    uint32_t* __restrict__ gctl = C.gctl[b];
    unsigned long long* __restrict__ stats = C.stats[b];
    const int64_t n_act = rg_actual_n(C.n[b], C.n_dev[b]);
    const int64_t i0 = (int64_t)blockIdx.x * (256 * kClassifyRows);
    if (i0 >= n_act) return;                                       // uniform per workgroup
    uint32_t w[kClassifyRows];
    int32_t v[kClassifyRows];
#pragma unroll
    for (int k = 0; k < kClassifyRows; ++k) {
        const int64_t i = i0 + k * 256 + threadIdx.x;
        v[k] = i < n_act ? nodes[i] : -1;
    }
#pragma unroll
    for (int k = 0; k < kClassifyRows; ++k) w[k] = v[k] >= 0 ? (uint32_t)loc[v[k]] : 0xFFFFFFFFu;   // tag 3 = no row
    int c_local = 0, c_hit = 0, n_miss = 0;
#pragma unroll
    for (int k = 0; k < kClassifyRows; ++k) {
        const int64_t i = i0 + k * 256 + threadIdx.x;
        const uint32_t tag = w[k] >> RG_TAG_SHIFT;
        if (i < n_act) src[i] = w[k];
        c_local += tag == RG_TAG_LOCAL;
        c_hit += tag == RG_TAG_CACHE;
        n_miss += tag == RG_TAG_REMOTE;
    }
    const int wave = threadIdx.x >> 6;
    c_local = rg_wave_sum(c_local);
    c_hit = rg_wave_sum(c_hit);
    const int c_miss = rg_wave_sum(n_miss);
    if (rg_lane() == 0) { cls[0][wave] = c_local; cls[1][wave] = c_hit; cls[2][wave] = c_miss; }
    int total_miss;
    int excl = rg_block_excl_scan<256 / RG_WAVE>(n_miss, smem, &total_miss);          // barriers inside publish cls[]
    if (threadIdx.x < 3) {
        const int t = cls[threadIdx.x][0] + cls[threadIdx.x][1] + cls[threadIdx.x][2] + cls[threadIdx.x][3];
        if (t) atomicAdd(&stats[threadIdx.x], (unsigned long long)t);
    }
    if (total_miss == 0) return;                                   // uniform
    if (threadIdx.x == 0) miss_base = atomicAdd(&gctl[0], (uint32_t)total_miss);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kClassifyRows; ++k)
        if ((w[k] >> RG_TAG_SHIFT) == RG_TAG_REMOTE) {   // (output row, remote row) pairs: the miss kernel needs no further lookup
            const int64_t j = (int64_t)miss_base + excl++;
            miss_list[2 * j] = (int32_t)(i0 + k * 256 + threadIdx.x);
            miss_list[2 * j + 1] = (int32_t)(w[k] & RG_ROW_MASK);
        }
}

// Rows whose source is in HBM, with a flat work split: the batch is one stream of 16-byte chunks (row-major over
// the output), every wavefront takes 64*T consecutive chunks and every lane T of them, whatever the row length,
// so all lanes carry T loads in flight for 400-byte and 2408-byte rows as well as for power-of-two ones, and
// the stores of a wavefront are contiguous when the output stride equals the padded row length.
template <int VEC, int T>
__global__ void __launch_bounds__(256) k_gather_hbm(const uint32_t* __restrict__ src, int64_t n, const int32_t* __restrict__ n_dev,
                                                         const float* __restrict__ local_store, int64_t local_stride,
                                                         const float* __restrict__ cache_rows, int64_t cache_stride,
                                                         float* __restrict__ out, int64_t out_stride, int cpr, float inv_cpr) {
    typedef typename RgVec<VEC>::type V;
    const int64_t n_act = rg_actual_n(n, n_dev);
    const int lane = rg_lane();
    constexpr int CW = RG_WAVE * T;                    // chunks per wavefront step
    const int64_t total = n_act * cpr;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t q0 = wave * CW; q0 < total; q0 += nwaves * CW) {
        const int64_t row0 = q0 / cpr;
        const int off0 = (int)(q0 - row0 * cpr);
        const V* sp[T];
        V* dp[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int ql = off0 + lane + RG_WAVE * t;           // < cpr + 64*T: exact in fp32
            int r = (int)((float)ql * inv_cpr);
            if (r * cpr > ql) --r; else if ((r + 1) * cpr <= ql) ++r;
            const int c = ql - r * cpr;
            const int64_t i = row0 + r;
            sp[t] = nullptr;
            dp[t] = nullptr;
            if (i < n_act) {
                const uint32_t w = src[i];
                const uint32_t tag = w >> RG_TAG_SHIFT;
                const int64_t row = (int64_t)(w & RG_ROW_MASK);
                if (tag != RG_TAG_REMOTE) {
                    sp[t] = (const V*)(tag == RG_TAG_LOCAL ? local_store + row * local_stride : cache_rows + row * cache_stride) + c;
                    dp[t] = (V*)(out + i * out_stride) + c;
                }
            }
        }
        V val[T];
#pragma unroll
        for (int t = 0; t < T; ++t)
            if (sp[t]) val[t] = *sp[t];
#pragma unroll
        for (int t = 0; t < T; ++t)
            if (dp[t]) __builtin_nontemporal_store(val[t], dp[t]);
    }
}

// Rows whose source is the remote store: walks the compacted miss list.
template <int VEC, int U>
__global__ void __launch_bounds__(1024) k_gather_miss(const int32_t* __restrict__ miss_list,
                                                     const uint32_t* __restrict__ gctl, const float* __restrict__ remote_store,
                                                     int64_t remote_stride, float* __restrict__ out, int64_t out_stride,
                                                     int cpr, int log2L) {
    typedef typename RgVec<VEC>::type V;
    const int64_t n_miss = gctl[0];
    const int lane = rg_lane();
    const int L = 1 << log2L;
    const int R = RG_WAVE >> log2L;
    const int sub = lane >> log2L;
    const int c0 = lane & (L - 1);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t j0 = wave * (R * U); j0 < n_miss; j0 += nwaves * (R * U)) {
        const V* sp[U];
        V* dp[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // loads are unconditional (a lane group without a row reads output row 0, which is in HBM; the value is
            // discarded) so that every wavefront keeps U row loads in flight on the link; only the stores are predicated
            const int64_t j = j0 + u * R + sub;
            sp[u] = (const V*)out;
            dp[u] = nullptr;
            if (j < n_miss) {
                const int64_t i = miss_list[2 * j];
                const int64_t row = miss_list[2 * j + 1];
                sp[u] = (const V*)(remote_store + row * remote_stride);
                dp[u] = (V*)(out + i * out_stride);
            }
        }
        for (int c = c0; c < cpr; c += L) {
            V val[U];
#pragma unroll
            for (int u = 0; u < U; ++u) val[u] = sp[u][c];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dp[u]) __builtin_nontemporal_store(val[u], &dp[u][c]);
        }
    }
}

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    const int x = atoi(v);
    return x > 0 ? x : dflt;
}

}  // namespace

extern "C" {

rg_status rg_gather_prepare(rg_ctx* ctx, int32_t first_ticket, int32_t count, const int32_t* const* input_nodes,
                            const int64_t* n, const int32_t* const* n_dev, const rg_cache* cache,
                            rg_gather_stats* const* stats, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, first_ticket >= 0 && count >= 0 && first_ticket + count <= RG_GATHER_TICKETS,
               "rg_gather_prepare: tickets %d..%d not in [0,%d)", first_ticket, first_ticket + count - 1, RG_GATHER_TICKETS);
    if (count == 0) return RG_OK;
    RG_REQUIRE(ctx, input_nodes && n && stats, "rg_gather_prepare: null argument array");
    RG_REQUIRE(ctx, cache && cache->loc, "rg_gather_prepare: cache / cache->loc is NULL");
    int64_t n_max = 0;
    for (int k = 0; k < count; ++k) {
        RG_REQUIRE(ctx, n[k] >= 0 && n[k] <= (1ll << 31) - 1, "rg_gather_prepare: n = %lld out of range (batch %d)", (long long)n[k], k);
        RG_REQUIRE(ctx, stats[k], "rg_gather_prepare: stats is NULL (batch %d)", k);
        RG_REQUIRE(ctx, n[k] == 0 || input_nodes[k], "rg_gather_prepare: input_nodes is NULL (batch %d)", k);
        n_max = rg_max64(n_max, n[k]);
    }
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    rg_status st = rg_gather_reserve(ctx, rg_max64(n_max, 1));
    if (st != RG_OK) return st;
    ClassifyGroup C;
    for (int k = 0; k < RG_GATHER_TICKETS; ++k) {
        const bool live = k < count;
        const int t = first_ticket + (live ? k : 0);
        C.nodes[k] = live ? input_nodes[k] : nullptr;
        C.n_dev[k] = live && n_dev ? n_dev[k] : nullptr;
        C.n[k] = live ? n[k] : 0;
        C.src[k] = (uint32_t*)ctx->gather_src.p + (int64_t)t * ctx->gather_cap;
        C.miss_list[k] = (int32_t*)ctx->miss_list.p + (int64_t)t * 2 * ctx->gather_cap;
        C.gctl[k] = (uint32_t*)ctx->gather_ctl.p + t * 16;
        C.stats[k] = live ? (unsigned long long*)stats[k] : nullptr;
        if (live) ctx->gather_rows[t] = -1;
    }
    k_gather_reset<<<count, 64, 0, s>>>(C);
    RG_LAUNCH_CHECK(ctx, "k_gather_reset");
    if (n_max > 0) {
        k_classify<<<dim3((unsigned)rg_div_up(n_max, 256 * kClassifyRows), (unsigned)count), 256, 0, s>>>(C, cache->loc);
        RG_LAUNCH_CHECK(ctx, "k_classify");
    }
    for (int k = 0; k < count; ++k) ctx->gather_rows[first_ticket + k] = n[k];
    return RG_OK;
}

rg_status rg_gather_run(rg_ctx* ctx, int32_t ticket, int64_t n, const int32_t* n_dev, const rg_cache* cache,
                        const float* local_store, int64_t local_stride, const float* remote_store, int64_t remote_stride,
                        int32_t dim, float* out, int64_t out_stride, void* hit_stream, void* miss_stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, ticket >= 0 && ticket < RG_GATHER_TICKETS, "rg_gather_run: ticket = %d not in [0,%d)", ticket, RG_GATHER_TICKETS);
    RG_REQUIRE(ctx, n >= 0 && n <= (1ll << 31) - 1, "rg_gather_run: n = %lld out of range", (long long)n);
    RG_REQUIRE(ctx, dim >= 1, "rg_gather_run: dim = %d must be positive", dim);
    RG_REQUIRE(ctx, cache && cache->loc, "rg_gather_run: cache / cache->loc is NULL");
    RG_REQUIRE(ctx, out_stride >= dim, "rg_gather_run: out_stride < dim");
    RG_REQUIRE(ctx, !local_store || local_stride >= dim, "rg_gather_run: local_stride < dim");
    RG_REQUIRE(ctx, !remote_store || remote_stride >= dim, "rg_gather_run: remote_stride < dim");
    RG_REQUIRE(ctx, !cache->cache_rows || cache->row_stride >= dim, "rg_gather_run: cache row_stride < dim");
    RG_REQUIRE(ctx, n == 0 || out, "rg_gather_run: out is NULL");
    // A store may be absent only if no location word can point into it; that cannot be verified on the
    // host, so all three are required whenever rows are requested.
    RG_REQUIRE(ctx, n == 0 || (local_store && remote_store), "rg_gather_run: null feature store");
    RG_REQUIRE(ctx, n == 0 || cache->cache_rows || cache->capacity_rows == 0, "rg_gather_run: cache_rows is NULL");
    if (ctx->gather_rows[ticket] != n)
        return rg_set_error(ctx, RG_ERR_STATE, "rg_gather_run: ticket %d was prepared for %lld rows, not %lld", ticket,
                            (long long)ctx->gather_rows[ticket], (long long)n);
    if (n == 0) return RG_OK;
    RG_HIP(ctx, hipSetDevice(ctx->device));
    {
        const rg_status chk = rg_check_device_readable(ctx, remote_store, "rg_gather_run: remote_store");
        if (chk != RG_OK) return chk;
    }
    hipStream_t sh = (hipStream_t)hit_stream;
    hipStream_t sm = miss_stream ? (hipStream_t)miss_stream : sh;
    const bool two_streams = sm != sh;
    uint32_t* gctl = (uint32_t*)ctx->gather_ctl.p + ticket * 16;
    uint32_t* src = (uint32_t*)ctx->gather_src.p + (int64_t)ticket * ctx->gather_cap;
    int32_t* miss_list = (int32_t*)ctx->miss_list.p + (int64_t)ticket * 2 * ctx->gather_cap;
    if (two_streams) {
        RG_HIP(ctx, hipEventRecord(ctx->ev_classified, sh));
        RG_HIP(ctx, hipStreamWaitEvent(sm, ctx->ev_classified, 0));
    }

    const void* ptrs[4] = {local_store, remote_store, cache->cache_rows, out};
    const int64_t strides[4] = {local_stride, remote_stride, cache->cache_rows ? cache->row_stride : 0, out_stride};
    const int vec = rg_pick_vec(dim, ptrs, 4, strides, 4);
    const RgRowShape shp = rg_row_shape(dim, vec);
    constexpr int U = 4;                                    // rows in flight per lane group in the miss kernel
    // T chunks in flight per lane; swept on the box: 2 is best (T = 4: -2 %, T = 8: -12 %), an uncapped grid
    // (one step per wavefront) beats a persistent one, and non-temporal stores make no difference.
    int T = env_int("RG_GATHER_UNROLL", 2);
    if (vec != 4 || (T != 2 && T != 4 && T != 8)) T = (vec == 4) ? 2 : 4;
    const int per_cu = env_int("RG_GATHER_BLOCKS_PER_CU", 4096);
    const int64_t chunks_per_block = 4ll * RG_WAVE * T;
    const int grid = (int)rg_max64(1, rg_min64(rg_div_up(n * (int64_t)shp.cpr, chunks_per_block), (int64_t)ctx->num_cus * per_cu));
    const float inv_cpr = 1.0f / (float)shp.cpr;
    const float* cache_rows = cache->cache_rows ? cache->cache_rows : local_store;   // never dereferenced without cache words

    int tok = rg_prof_begin(ctx, RG_K_GATHER_HBM, sh);
#define RG_LAUNCH_HBM(V, TT)                                                                                     \
    k_gather_hbm<V, TT><<<grid, 256, 0, sh>>>(src, n, n_dev, local_store, local_stride, cache_rows, cache->row_stride, \
                                              out, out_stride, shp.cpr, inv_cpr)
    if (vec == 4) { if (T == 2) RG_LAUNCH_HBM(4, 2); else if (T == 8) RG_LAUNCH_HBM(4, 8); else RG_LAUNCH_HBM(4, 4); }
    else if (vec == 2) RG_LAUNCH_HBM(2, 4);
    else RG_LAUNCH_HBM(1, 4);
#undef RG_LAUNCH_HBM
    rg_prof_end(ctx, tok, sh);
    RG_LAUNCH_CHECK(ctx, "k_gather_hbm");

    int64_t miss_blocks;
    int miss_threads;
    rg_hostlink_launch_shape(&miss_blocks, &miss_threads, true);
    const int miss_rows_per_block = (miss_threads / RG_WAVE) * (RG_WAVE >> shp.log2L) * U;
    const int miss_grid = (int)rg_max64(1, rg_min64(rg_div_up(n, miss_rows_per_block), miss_blocks));
    tok = rg_prof_begin(ctx, RG_K_GATHER_MISS, sm);
    if (vec == 4)
        k_gather_miss<4, U><<<miss_grid, miss_threads, 0, sm>>>(miss_list, gctl, remote_store, remote_stride, out, out_stride, shp.cpr, shp.log2L);
    else if (vec == 2)
        k_gather_miss<2, U><<<miss_grid, miss_threads, 0, sm>>>(miss_list, gctl, remote_store, remote_stride, out, out_stride, shp.cpr, shp.log2L);
    else
        k_gather_miss<1, U><<<miss_grid, miss_threads, 0, sm>>>(miss_list, gctl, remote_store, remote_stride, out, out_stride, shp.cpr, shp.log2L);
    rg_prof_end(ctx, tok, sm);
    RG_LAUNCH_CHECK(ctx, "k_gather_miss");
    if (two_streams) {
        RG_HIP(ctx, hipEventRecord(ctx->ev_miss_done, sm));
        RG_HIP(ctx, hipStreamWaitEvent(sh, ctx->ev_miss_done, 0));
    }
    return RG_OK;
}

rg_status rg_gather_features(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                             const rg_cache* cache, const float* local_store, int64_t local_stride,
                             const float* remote_store, int64_t remote_stride, int32_t dim, float* out,
                             int64_t out_stride, rg_gather_stats* stats, void* hit_stream, void* miss_stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, stats, "rg_gather_features: stats is NULL");
    // argument errors of the copy step are reported before anything is queued
    RG_REQUIRE(ctx, n >= 0 && n <= (1ll << 31) - 1, "rg_gather_features: n = %lld out of range", (long long)n);
    RG_REQUIRE(ctx, dim >= 1, "rg_gather_features: dim = %d must be positive", dim);
    RG_REQUIRE(ctx, cache && cache->loc, "rg_gather_features: cache / cache->loc is NULL");
    RG_REQUIRE(ctx, out_stride >= dim && (!local_store || local_stride >= dim) && (!remote_store || remote_stride >= dim) &&
                        (!cache->cache_rows || cache->row_stride >= dim), "rg_gather_features: a row stride is smaller than dim");
    RG_REQUIRE(ctx, n == 0 || (input_nodes && out && local_store && remote_store), "rg_gather_features: null pointer");
    RG_REQUIRE(ctx, n == 0 || cache->cache_rows || cache->capacity_rows == 0, "rg_gather_features: cache_rows is NULL");
    if (n > 0) {
        RG_HIP(ctx, hipSetDevice(ctx->device));
        const rg_status chk = rg_check_device_readable(ctx, remote_store, "rg_gather_features: remote_store");
        if (chk != RG_OK) return chk;
    }
    rg_status st = rg_gather_prepare(ctx, 0, 1, &input_nodes, &n, &n_dev, cache, &stats, hit_stream);
    if (st != RG_OK) return st;
    return rg_gather_run(ctx, 0, n, n_dev, cache, local_store, local_stride, remote_store, remote_stride, dim, out, out_stride,
                         hit_stream, miss_stream);
}

}  // extern "C"
