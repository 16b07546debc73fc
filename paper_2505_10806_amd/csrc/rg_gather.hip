// Per-batch feature assembly (Alg. 1 lines 12-14): rows of the batch's input nodes are copied from the
// local store (HBM), the steady cache (HBM) or, for misses only, the remote store (pinned host memory).
//
// Three kernels: classify resolves every output row to a location word (one random 4-byte read of loc[]
// per row), counts the three classes and compacts the indices of the miss rows; the HBM kernel copies
// local and cached rows; the miss kernel copies the remote rows and may run on a second stream so the
// host-link transfers overlap the HBM copies.
#include "rg_rowcopy.h"

// Scratch of rg_gather_features_static: one control block, the resolved location word of every output row and
// the (output row, remote row) pairs of the miss rows, for up to RG_STATIC_GATHER_MAX_ROWS rows.  Every GPU the
// library runs on holds its own copy of this array until the process ends.  Host code must not use the array's
// name as an address: rg_gather_static_init resolves the device address once per context.
constexpr size_t kStaticCtlBytes = 256;
constexpr size_t kStaticSrcBytes = (size_t)RG_STATIC_GATHER_MAX_ROWS * 4;
constexpr size_t kStaticMissBytes = (size_t)RG_STATIC_GATHER_MAX_ROWS * 8;
static __device__ __align__(256) unsigned char scratch[kStaticCtlBytes + kStaticSrcBytes + kStaticMissBytes];

rg_status rg_gather_static_init(rg_ctx* ctx) {
    void* ptr = nullptr;
    RG_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return rg_set_error(ctx, RG_ERR_HIP, "hipGetSymbolAddress returned a null address for the gather scratch");
    ctx->static_scratch = ptr;
    return RG_OK;
}

namespace {

// Where one batch's lookup results live: a ticket's slices of the context scratch, or the static scratch.
struct GatherScratch {
    uint32_t* src;        // [rows] resolved location word per output row
    int32_t* miss_list;   // [2 * rows] (output row, remote row) pairs
    uint32_t* gctl;       // [0] = number of misses
};

GatherScratch ticket_scratch(rg_ctx* ctx, int t) {
    GatherScratch g;
    g.src = (uint32_t*)ctx->gather_src.p + (int64_t)t * ctx->gather_cap;
    g.miss_list = (int32_t*)ctx->miss_list.p + (int64_t)t * 2 * ctx->gather_cap;
    g.gctl = (uint32_t*)ctx->gather_ctl.p + t * 16;
    return g;
}

GatherScratch static_scratch(rg_ctx* ctx) {
    unsigned char* base = (unsigned char*)ctx->static_scratch;
    GatherScratch g;
    g.gctl = (uint32_t*)base;
    g.src = (uint32_t*)(base + kStaticCtlBytes);
    g.miss_list = (int32_t*)(base + kStaticCtlBytes + kStaticSrcBytes);
    return g;
}


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

// mirror_home != NULL: the cache is laid out as a mirror of the remote store, so a cached node's row is found at its
// remote-store row (from its home word) instead of at its slot.
__global__ void __launch_bounds__(256) k_classify(const ClassifyGroup C, const int32_t* __restrict__ loc,
                                                  const int32_t* __restrict__ mirror_home) {
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
    if (mirror_home) {
#pragma unroll
        for (int k = 0; k < kClassifyRows; ++k)
            if ((w[k] >> RG_TAG_SHIFT) == RG_TAG_CACHE)
                w[k] = (RG_TAG_CACHE << RG_TAG_SHIFT) | ((uint32_t)mirror_home[v[k]] & RG_ROW_MASK);
    }
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
                                                         float* __restrict__ out, int64_t out_stride, int cpr, float inv_cpr,
                                                         int tail) {
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
        bool last[T];                                           // the row's last chunk, of which only `tail` floats are stored
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int ql = off0 + lane + RG_WAVE * t;           // < cpr + 64*T: exact in fp32
            int r = (int)((float)ql * inv_cpr);
            if (r * cpr > ql) --r; else if ((r + 1) * cpr <= ql) ++r;
            const int c = ql - r * cpr;
            last[t] = tail < VEC && c == cpr - 1;
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
            if (dp[t]) {
                if (last[t]) rg_store_head(dp[t], val[t], tail);
                else __builtin_nontemporal_store(val[t], dp[t]);
            }
    }
}

// Rows whose source is the remote store: walks the compacted miss list.
template <int VEC, int U>
__global__ void __launch_bounds__(1024) k_gather_miss(const int32_t* __restrict__ miss_list,
                                                    const uint32_t* __restrict__ gctl, const float* __restrict__ remote_store,
                                                    int64_t remote_stride, float* __restrict__ out, int64_t out_stride,
                                                    int cpr, int log2L, int tail) {
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
            const bool head_only = tail < VEC && c == cpr - 1;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dp[u]) {
                    if (head_only) rg_store_head(&dp[u][c], val[u], tail);
                    else __builtin_nontemporal_store(val[u], &dp[u][c]);
                }
        }
    }
}

// Lookups of `count` batches in one launch; scr[k] receives batch k's results.
rg_status launch_classify(rg_ctx* ctx, int count, const int32_t* const* input_nodes, const int64_t* n, const int32_t* const* n_dev,
                          const rg_cache* cache, rg_gather_stats* const* stats, const GatherScratch* scr, hipStream_t s) {
    ClassifyGroup C;
    int64_t n_max = 0;
    for (int k = 0; k < RG_GATHER_TICKETS; ++k) {
        const bool live = k < count;
        const GatherScratch& g = scr[live ? k : 0];
        C.nodes[k] = live ? input_nodes[k] : nullptr;
        C.n_dev[k] = live && n_dev ? n_dev[k] : nullptr;
        C.n[k] = live ? n[k] : 0;
        C.src[k] = g.src;
        C.miss_list[k] = g.miss_list;
        C.gctl[k] = g.gctl;
        C.stats[k] = live ? (unsigned long long*)stats[k] : nullptr;
        if (live) n_max = rg_max64(n_max, n[k]);
    }
    k_gather_reset<<<count, 64, 0, s>>>(C);
    RG_LAUNCH_CHECK(ctx, "k_gather_reset");
    if (n_max > 0) {
        k_classify<<<dim3((unsigned)rg_div_up(n_max, 256 * kClassifyRows), (unsigned)count), 256, 0, s>>>(
            C, cache->loc, cache->mirror_rows > 0 ? cache->home : nullptr);
        RG_LAUNCH_CHECK(ctx, "k_classify");
    }
    return RG_OK;
}

// Copies the rows of one classified batch: HBM rows on sh, miss rows on sm (joined back into sh when they differ).
// Every argument has been validated by the caller; `timed` brackets the kernels for rg_profile_read.
rg_status launch_copies(rg_ctx* ctx, const GatherScratch& scr, int64_t n, const int32_t* n_dev, const rg_cache* cache,
                        const float* local_store, int64_t local_stride, const float* remote_store, int64_t remote_stride,
                        int32_t dim, float* out, int64_t out_stride, hipStream_t sh, hipStream_t sm, bool timed,
                        int parts = RG_GATHER_PART_HBM | RG_GATHER_PART_MISS) {
    const bool do_hbm = parts & RG_GATHER_PART_HBM, do_miss = parts & RG_GATHER_PART_MISS;
    const bool two_streams = sm != sh && do_hbm && do_miss;      // one part alone: no fork, no join, the caller orders the streams
    if (two_streams) {
        RG_HIP(ctx, hipEventRecord(ctx->ev_classified, sh));
        RG_HIP(ctx, hipStreamWaitEvent(sm, ctx->ev_classified, 0));
    }
    const void* ptrs[4] = {local_store, remote_store, cache->cache_rows, out};
    const int64_t strides[4] = {local_stride, remote_stride, cache->cache_rows ? cache->row_stride : 0, out_stride};
    const int vec = rg_pick_vec(dim, ptrs, 4, strides, 4);
    const RgRowShape shp = rg_row_shape(dim, vec);
    constexpr int U = 4;                                    // rows in flight per lane group in the miss kernel
    // T chunks in flight per lane; swept on the device: 2 is best (T = 4: -2 %, T = 8: -12 %), and non-temporal
    // stores make no difference.
    const int T = vec == 4 ? ctx->knobs.gather_unroll : 4;
    const int64_t chunks_per_block = 4ll * RG_WAVE * T;
    int64_t grid64 = rg_div_up(n * (int64_t)shp.cpr, chunks_per_block);
    if (ctx->knobs.gather_blocks_per_cu > 0) grid64 = rg_min64(grid64, (int64_t)ctx->num_cus * ctx->knobs.gather_blocks_per_cu);
    const int grid = (int)rg_max64(1, grid64);
    const float inv_cpr = 1.0f / (float)shp.cpr;
    const float* cache_rows = cache->cache_rows ? cache->cache_rows : local_store;   // never dereferenced without cache words

    int tok = -1;
    if (do_hbm) {
        tok = timed ? rg_prof_begin(ctx, RG_K_GATHER_HBM, sh) : -1;
#define RG_LAUNCH_HBM(V, TT)                                                                                            \
        k_gather_hbm<V, TT><<<grid, 256, 0, sh>>>(scr.src, n, n_dev, local_store, local_stride, cache_rows, cache->row_stride, \
                                                  out, out_stride, shp.cpr, inv_cpr, shp.tail)
        if (vec == 4) { if (T == 2) RG_LAUNCH_HBM(4, 2); else if (T == 8) RG_LAUNCH_HBM(4, 8); else RG_LAUNCH_HBM(4, 4); }
        else if (vec == 2) RG_LAUNCH_HBM(2, 4);
        else RG_LAUNCH_HBM(1, 4);
#undef RG_LAUNCH_HBM
        rg_prof_end(ctx, tok, sh);
        RG_LAUNCH_CHECK(ctx, "k_gather_hbm");
    }

    if (do_miss) {
        const int miss_threads = ctx->knobs.miss_threads;
        const int miss_rows_per_block = (miss_threads / RG_WAVE) * (RG_WAVE >> shp.log2L) * U;
        const int miss_grid = (int)rg_max64(1, rg_min64(rg_div_up(n, miss_rows_per_block), ctx->knobs.miss_blocks));
        tok = timed ? rg_prof_begin(ctx, RG_K_GATHER_MISS, sm) : -1;
#define RG_LAUNCH_MISS(V)                                                                                               \
        k_gather_miss<V, U><<<miss_grid, miss_threads, 0, sm>>>(scr.miss_list, scr.gctl, remote_store, remote_stride, out, out_stride, \
                                                                shp.cpr, shp.log2L, shp.tail)
        if (vec == 4) RG_LAUNCH_MISS(4); else if (vec == 2) RG_LAUNCH_MISS(2); else RG_LAUNCH_MISS(1);
#undef RG_LAUNCH_MISS
        rg_prof_end(ctx, tok, sm);
        RG_LAUNCH_CHECK(ctx, "k_gather_miss");
    }
    if (two_streams) {
        RG_HIP(ctx, hipEventRecord(ctx->ev_miss_done, sm));
        RG_HIP(ctx, hipStreamWaitEvent(sh, ctx->ev_miss_done, 0));
    }
    return RG_OK;
}

// Argument checks shared by the entry points that copy rows.
rg_status check_copy_args(rg_ctx* ctx, const char* fn, int64_t n, int32_t dim, const rg_cache* cache, const float* local_store,
                          int64_t local_stride, const float* remote_store, int64_t remote_stride, const float* out,
                          int64_t out_stride) {
    RG_REQUIRE(ctx, n >= 0 && n <= (1ll << 31) - 1, "%s: n = %lld out of range", fn, (long long)n);
    RG_REQUIRE(ctx, dim >= 1, "%s: dim = %d must be positive", fn, dim);
    RG_REQUIRE(ctx, cache && cache->loc, "%s: cache / cache->loc is NULL", fn);
    RG_REQUIRE(ctx, cache->mirror_rows == 0 || (cache->home && cache->mirror_rows <= cache->capacity_rows),
               "%s: a mirrored cache needs cache->home and mirror_rows <= capacity_rows", fn);
    RG_REQUIRE(ctx, out_stride >= dim, "%s: out_stride < dim", fn);
    RG_REQUIRE(ctx, !local_store || local_stride >= dim, "%s: local_stride < dim", fn);
    RG_REQUIRE(ctx, !remote_store || remote_stride >= dim, "%s: remote_stride < dim", fn);
    RG_REQUIRE(ctx, !cache->cache_rows || cache->row_stride >= dim, "%s: cache row_stride < dim", fn);
    RG_REQUIRE(ctx, n == 0 || out, "%s: out is NULL", fn);
    // A store may be absent only if no location word can point into it; that cannot be verified on the
    // host, so all three are required whenever rows are requested.
    RG_REQUIRE(ctx, n == 0 || (local_store && remote_store), "%s: null feature store", fn);
    RG_REQUIRE(ctx, n == 0 || cache->cache_rows || cache->capacity_rows == 0, "%s: cache_rows is NULL", fn);
    return RG_OK;
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
    RG_REQUIRE(ctx, cache->mirror_rows == 0 || cache->home, "rg_gather_prepare: a mirrored cache needs cache->home");
    int64_t n_max = 0;
    for (int k = 0; k < count; ++k) {
        RG_REQUIRE(ctx, n[k] >= 0 && n[k] <= (1ll << 31) - 1, "rg_gather_prepare: n = %lld out of range (batch %d)", (long long)n[k], k);
        RG_REQUIRE(ctx, stats[k], "rg_gather_prepare: stats is NULL (batch %d)", k);
        RG_REQUIRE(ctx, n[k] == 0 || input_nodes[k], "rg_gather_prepare: input_nodes is NULL (batch %d)", k);
        n_max = rg_max64(n_max, n[k]);
    }
    RG_HIP(ctx, hipSetDevice(ctx->device));
    rg_status st = rg_gather_reserve(ctx, rg_max64(n_max, 1));
    if (st != RG_OK) return st;
    GatherScratch scr[RG_GATHER_TICKETS];
    for (int k = 0; k < count; ++k) {
        scr[k] = ticket_scratch(ctx, first_ticket + k);
        ctx->gather_rows[first_ticket + k] = -1;
    }
    if ((st = launch_classify(ctx, count, input_nodes, n, n_dev, cache, stats, scr, (hipStream_t)stream)) != RG_OK) return st;
    for (int k = 0; k < count; ++k) ctx->gather_rows[first_ticket + k] = n[k];
    return RG_OK;
}

rg_status rg_gather_run(rg_ctx* ctx, int32_t ticket, int64_t n, const int32_t* n_dev, const rg_cache* cache,
                        const float* local_store, int64_t local_stride, const float* remote_store, int64_t remote_stride,
                        int32_t dim, float* out, int64_t out_stride, void* hit_stream, void* miss_stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, ticket >= 0 && ticket < RG_GATHER_TICKETS, "rg_gather_run: ticket = %d not in [0,%d)", ticket, RG_GATHER_TICKETS);
    rg_status st = check_copy_args(ctx, "rg_gather_run", n, dim, cache, local_store, local_stride, remote_store, remote_stride, out, out_stride);
    if (st != RG_OK) return st;
    if (ctx->gather_rows[ticket] != n)
        return rg_set_error(ctx, RG_ERR_STATE, "rg_gather_run: ticket %d was prepared for %lld rows, not %lld", ticket,
                            (long long)ctx->gather_rows[ticket], (long long)n);
    if (n == 0) return RG_OK;
    RG_HIP(ctx, hipSetDevice(ctx->device));
    if ((st = rg_check_device_readable(ctx, remote_store, "rg_gather_run: remote_store")) != RG_OK) return st;
    hipStream_t sh = (hipStream_t)hit_stream;
    hipStream_t sm = miss_stream ? (hipStream_t)miss_stream : sh;
    return launch_copies(ctx, ticket_scratch(ctx, ticket), n, n_dev, cache, local_store, local_stride, remote_store, remote_stride,
                         dim, out, out_stride, sh, sm, true);
}

rg_status rg_gather_features(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                             const rg_cache* cache, const float* local_store, int64_t local_stride,
                             const float* remote_store, int64_t remote_stride, int32_t dim, float* out,
                             int64_t out_stride, rg_gather_stats* stats, void* hit_stream, void* miss_stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, stats, "rg_gather_features: stats is NULL");
    // argument errors of the copy step are reported before anything is queued
    rg_status st = check_copy_args(ctx, "rg_gather_features", n, dim, cache, local_store, local_stride, remote_store, remote_stride, out,
                                   out_stride);
    if (st != RG_OK) return st;
    RG_REQUIRE(ctx, n == 0 || input_nodes, "rg_gather_features: input_nodes is NULL");
    if (n > 0) {
        RG_HIP(ctx, hipSetDevice(ctx->device));
        if ((st = rg_check_device_readable(ctx, remote_store, "rg_gather_features: remote_store")) != RG_OK) return st;
    }
    st = rg_gather_prepare(ctx, 0, 1, &input_nodes, &n, &n_dev, cache, &stats, hit_stream);
    if (st != RG_OK) return st;
    return rg_gather_run(ctx, 0, n, n_dev, cache, local_store, local_stride, remote_store, remote_stride, dim, out, out_stride,
                         hit_stream, miss_stream);
}

rg_status rg_gather_run_part(rg_ctx* ctx, int32_t ticket, int32_t part, int64_t n, const int32_t* n_dev, const rg_cache* cache,
                             const float* local_store, int64_t local_stride, const float* remote_store, int64_t remote_stride,
                             int32_t dim, float* out, int64_t out_stride, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, ticket >= 0 && ticket < RG_GATHER_TICKETS, "rg_gather_run_part: ticket = %d not in [0,%d)", ticket, RG_GATHER_TICKETS);
    RG_REQUIRE(ctx, part == RG_GATHER_PART_HBM || part == RG_GATHER_PART_MISS, "rg_gather_run_part: part = %d is neither "
               "RG_GATHER_PART_HBM nor RG_GATHER_PART_MISS", part);
    rg_status st = check_copy_args(ctx, "rg_gather_run_part", n, dim, cache, local_store, local_stride, remote_store, remote_stride, out, out_stride);
    if (st != RG_OK) return st;
    if (ctx->gather_rows[ticket] != n)
        return rg_set_error(ctx, RG_ERR_STATE, "rg_gather_run_part: ticket %d was prepared for %lld rows, not %lld", ticket,
                            (long long)ctx->gather_rows[ticket], (long long)n);
    if (n == 0) return RG_OK;
    RG_HIP(ctx, hipSetDevice(ctx->device));
    if ((st = rg_check_device_readable(ctx, remote_store, "rg_gather_run_part: remote_store")) != RG_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    return launch_copies(ctx, ticket_scratch(ctx, ticket), n, n_dev, cache, local_store, local_stride, remote_store, remote_stride,
                         dim, out, out_stride, s, s, true, part);
}

rg_status rg_gather_features_static(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                                    const rg_cache* cache, const float* local_store, int64_t local_stride,
                                    const float* remote_store, int64_t remote_stride, int32_t dim, float* out,
                                    int64_t out_stride, rg_gather_stats* stats, void* hit_stream, void* miss_stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, stats, "rg_gather_features_static: stats is NULL");
    rg_status st = check_copy_args(ctx, "rg_gather_features_static", n, dim, cache, local_store, local_stride, remote_store,
                                   remote_stride, out, out_stride);
    if (st != RG_OK) return st;
    RG_REQUIRE(ctx, n == 0 || input_nodes, "rg_gather_features_static: input_nodes is NULL");
    if (n > RG_STATIC_GATHER_MAX_ROWS)
        return rg_set_error(ctx, RG_ERR_CAPACITY, "rg_gather_features_static: n = %lld exceeds the static scratch of %d rows "
                            "(use rg_gather_features)", (long long)n, RG_STATIC_GATHER_MAX_ROWS);
    RG_REQUIRE(ctx, ctx->static_scratch, "rg_gather_features_static: the static scratch was not resolved for this device");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    if (n > 0 && (st = rg_check_device_readable(ctx, remote_store, "rg_gather_features_static: remote_store")) != RG_OK) return st;
    hipStream_t sh = (hipStream_t)hit_stream;
    hipStream_t sm = miss_stream ? (hipStream_t)miss_stream : sh;
    // the reset kernel zeroes the miss counter and the statistics the previous call left behind
    const GatherScratch scr = static_scratch(ctx);
    if ((st = launch_classify(ctx, 1, &input_nodes, &n, &n_dev, cache, &stats, &scr, sh)) != RG_OK) return st;
    if (n == 0) return RG_OK;
    return launch_copies(ctx, scr, n, n_dev, cache, local_store, local_stride, remote_store, remote_stride, dim, out, out_stride,
                         sh, sm, false);
}

}  // extern "C"
