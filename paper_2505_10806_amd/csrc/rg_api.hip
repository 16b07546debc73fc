// Context, error reporting, scratch management and kernel timing of librapidgnn.
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include "rg_internal.h"
#include <algorithm>
#include <vector>

static char g_create_error[512];

rg_status rg_set_error(rg_ctx* ctx, rg_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    memcpy(ctx ? ctx->err : g_create_error, buf, sizeof(buf));
    return code;
}

rg_status rg_ensure(rg_ctx* ctx, RgBuf& buf, size_t bytes, bool zero_new) {
    if (bytes <= buf.bytes) return RG_OK;
    // Grow geometrically so repeated small increases do not reallocate every call.
    size_t want = bytes > buf.bytes + buf.bytes / 2 ? bytes : buf.bytes + buf.bytes / 2;
    want = (want + 255) & ~size_t(255);
    if (buf.p) {
        // Earlier work may still be reading the old allocation.
        RG_HIP(ctx, hipDeviceSynchronize());
        RG_HIP(ctx, hipFree(buf.p));
        buf.p = nullptr;
        buf.bytes = 0;
    }
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return rg_set_error(ctx, RG_ERR_OOM, "scratch allocation of %zu bytes failed: %s", want,
                            hipGetErrorString(e));
    }
    if (zero_new) {
        // the fill runs on the null stream, which streams created as non-blocking do not wait for: finish it here,
        // before a kernel on such a stream can touch the buffer
        RG_HIP(ctx, hipMemset(p, 0, want));
        RG_HIP(ctx, hipDeviceSynchronize());
    }
    buf.p = p;
    buf.bytes = want;
    return RG_OK;
}

rg_status rg_check_device_readable(rg_ctx* ctx, const void* p, const char* what) {
    hipPointerAttribute_t attr;
    const hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();          // an ordinary (pageable) host pointer is reported as an error
        return rg_set_error(ctx, RG_ERR_INVALID_ARG,
                            "%s = %p is not device-accessible memory (allocate it on the device or as pinned host memory)", what, p);
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeHost && attr.type != hipMemoryTypeManaged &&
        attr.type != hipMemoryTypeArray)
        return rg_set_error(ctx, RG_ERR_INVALID_ARG,
                            "%s = %p is not device-accessible memory (allocate it on the device or as pinned host memory)", what, p);
    return RG_OK;
}

rg_status rg_gather_reserve(rg_ctx* ctx, int64_t rows) {
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->gather_ctl, (size_t)RG_GATHER_TICKETS * 64)) != RG_OK) return st;
    if (rows <= ctx->gather_cap) return RG_OK;
    // a larger per-ticket stride moves every ticket's slice: nothing prepared earlier stays valid
    for (int t = 0; t < RG_GATHER_TICKETS; ++t) ctx->gather_rows[t] = -1;
    const int64_t cap = rg_max64(rows, ctx->gather_cap + ctx->gather_cap / 2);
    if ((st = rg_ensure(ctx, ctx->gather_src, (size_t)RG_GATHER_TICKETS * cap * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->miss_list, (size_t)RG_GATHER_TICKETS * cap * 8)) != RG_OK) return st;
    ctx->gather_cap = cap;
    return RG_OK;
}

static int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    const int x = atoi(v);
    return x > 0 ? x : dflt;
}

extern "C" {

const char* rg_version(void) { return "rapidgnn-mi355x 0.1 (gfx950)"; }

rg_status rg_create(int device, rg_ctx** out) {
    if (!out) return rg_set_error(nullptr, RG_ERR_INVALID_ARG, "rg_create: out is NULL");
    *out = nullptr;
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || count <= 0) {
        (void)hipGetLastError();
        return rg_set_error(nullptr, RG_ERR_HIP, "rg_create: no HIP device available (%s)",
                            e == hipSuccess ? "device count is 0" : hipGetErrorString(e));
    }
    if (device < 0 || device >= count)
        return rg_set_error(nullptr, RG_ERR_INVALID_ARG, "rg_create: device %d out of range [0,%d)", device, count);
    e = hipSetDevice(device);
    if (e != hipSuccess) return rg_set_error(nullptr, RG_ERR_HIP, "hipSetDevice: %s", hipGetErrorString(e));
    rg_ctx* ctx = new rg_ctx();
    ctx->device = device;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->num_cus = prop.multiProcessorCount;
    if (hipEventCreateWithFlags(&ctx->ev_classified, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->ev_miss_done, hipEventDisableTiming) != hipSuccess) {
        delete ctx;
        return rg_set_error(nullptr, RG_ERR_HIP, "rg_create: hipEventCreate failed");
    }
    if (rg_gather_static_init(ctx) != RG_OK) {
        memcpy(g_create_error, ctx->err, sizeof(g_create_error));
        rg_destroy(ctx);
        return RG_ERR_HIP;
    }
    // launch-shape knobs: read here once, never on the call paths
    RgKnobs& k = ctx->knobs;
    const int unroll = env_int("RG_GATHER_UNROLL", k.gather_unroll);
    if (unroll == 2 || unroll == 4 || unroll == 8) k.gather_unroll = unroll;
    k.gather_blocks_per_cu = env_int("RG_GATHER_BLOCKS_PER_CU", k.gather_blocks_per_cu);
    k.pull_blocks = env_int("RG_PULL_BLOCKS", k.pull_blocks);
    const int threads = env_int("RG_PULL_THREADS", k.pull_threads);
    if (threads == 64 || threads == 256 || threads == 1024) k.pull_threads = threads;
    k.miss_blocks = env_int("RG_MISS_BLOCKS", k.miss_blocks);
    { const char* v = getenv("RG_XCD_MAP"); if (v && *v == '0') k.xcd_map = 0; }
    const int mthreads = env_int("RG_MISS_THREADS", k.miss_threads);
    if (mthreads == 64 || mthreads == 256 || mthreads == 1024) k.miss_threads = mthreads;
    if (env_int("RG_PULL_ROWS", k.pull_rows) == 8) k.pull_rows = 8;
    *out = ctx;
    return RG_OK;
}

void rg_destroy(rg_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    RgBuf* bufs[] = {&ctx->visited, &ctx->marked, &ctx->pos, &ctx->chunk_sum, &ctx->row_start, &ctx->row_deg, &ctx->first_key, &ctx->sched_keys, &ctx->sched_ids,
                     &ctx->topk_ctl, &ctx->topk_blk, &ctx->topk_caps, &ctx->pf_list, &ctx->pf_ctl, &ctx->plan_cursor, &ctx->claim_bits, &ctx->claim_blk, &ctx->gather_src, &ctx->miss_list,
                     &ctx->gather_ctl};
    for (RgBuf* b : bufs)
        if (b->p) (void)hipFree(b->p);
    for (auto& s : ctx->spans) { (void)hipEventDestroy(s.start); (void)hipEventDestroy(s.stop); }
    for (auto& p : ctx->free_events) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
    if (ctx->ev_classified) (void)hipEventDestroy(ctx->ev_classified);
    if (ctx->ev_miss_done) (void)hipEventDestroy(ctx->ev_miss_done);
    for (hipStream_t s : ctx->streams) (void)hipStreamDestroy(s);       // after the events that may have been recorded on them
    delete ctx;
}

const char* rg_last_error(const rg_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

rg_status rg_reserve(rg_ctx* ctx, int64_t num_nodes, int64_t max_frontier, int64_t max_rows, int32_t sample_group) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, num_nodes >= 0 && max_frontier >= 0 && max_rows >= 0, "rg_reserve: negative size");
    RG_REQUIRE(ctx, num_nodes <= (int64_t)RG_ROW_MASK + 1, "rg_reserve: num_nodes exceeds 2^30");
    RG_REQUIRE(ctx, sample_group >= 1 && sample_group <= RG_MAX_GROUP, "rg_reserve: sample_group = %d not in [1,%d]", sample_group, RG_MAX_GROUP);
    RG_HIP(ctx, hipSetDevice(ctx->device));
    rg_status st;
    if ((st = rg_sampler_reserve(ctx, num_nodes, max_frontier, sample_group)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->topk_blk, ((size_t)rg_div_up(num_nodes, 1024) + 2) * 8)) != RG_OK) return st;
    if ((st = rg_gather_reserve(ctx, max_rows)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->pf_list, (size_t)max_rows * 8)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->pf_ctl, 64)) != RG_OK) return st;
    // rg_plan_sampled: one word of new-node bits per 32 nodes, one pair count per 1024 words
    const int64_t words = rg_max64(1, rg_div_up(num_nodes, 32));
    if ((st = rg_ensure(ctx, ctx->claim_bits, (size_t)words * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->claim_blk, (size_t)rg_max64(1, rg_div_up(words, 1024)) * 4)) != RG_OK) return st;
    return RG_OK;
}

rg_status rg_blocks_bounds(int64_t num_nodes, int64_t num_edges, int64_t num_seeds, const int32_t* fanouts,
                           int32_t num_hops, int64_t* frontier_ub, int64_t* edges_ub) {
    if (!fanouts || !frontier_ub || !edges_ub || num_hops < 1 || num_hops > RG_MAX_HOPS || num_nodes < 0 ||
        num_edges < 0 || num_seeds < 0)
        return RG_ERR_INVALID_ARG;
    for (int h = 0; h < num_hops; ++h)
        if (fanouts[h] != RG_FANOUT_ALL && (fanouts[h] < 0 || fanouts[h] > RG_MAX_FANOUT)) return RG_ERR_INVALID_ARG;
    frontier_ub[0] = rg_min64(num_seeds, num_nodes);
    for (int h = 0; h < num_hops; ++h) {
        const int64_t f = fanouts[h];
        // |nbr[h]| <= sum over distinct frontier nodes of min(F, deg) <= min(nnz, n_h * F)
        const int64_t e = (f == RG_FANOUT_ALL) ? num_edges : rg_min64(num_edges, frontier_ub[h] * f);
        edges_ub[h] = e;
        frontier_ub[h + 1] = rg_min64(num_nodes, frontier_ub[h] + e);
    }
    return RG_OK;
}

// ------------------------------------------------------------------ kernel timing
rg_status rg_profile_enable(rg_ctx* ctx, int on) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    ctx->profiling = on != 0;
    return RG_OK;
}

static rg_status rg_prof_collect(rg_ctx* ctx) {
    for (auto& s : ctx->spans) {
        RG_HIP(ctx, hipEventSynchronize(s.stop));
        float ms = 0.f;
        RG_HIP(ctx, hipEventElapsedTime(&ms, s.start, s.stop));
        ctx->prof_ms[s.kernel] += ms;
        ctx->prof_launches[s.kernel] += 1;
        ctx->free_events.emplace_back(s.start, s.stop);
    }
    ctx->spans.clear();
    return RG_OK;
}

rg_status rg_profile_reset(rg_ctx* ctx) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    rg_status st = rg_prof_collect(ctx);
    if (st != RG_OK) return st;
    for (int k = 0; k < RG_K_COUNT_; ++k) { ctx->prof_ms[k] = 0; ctx->prof_launches[k] = 0; }
    return RG_OK;
}

rg_status rg_profile_select(rg_ctx* ctx, uint32_t kernel_mask) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    ctx->prof_mask = kernel_mask;
    return RG_OK;
}

rg_status rg_profile_read(rg_ctx* ctx, int kernel_id, double* total_ms, int64_t* launches) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, kernel_id >= 0 && kernel_id < RG_K_COUNT_ && total_ms && launches, "rg_profile_read: bad argument");
    rg_status st = rg_prof_collect(ctx);
    if (st != RG_OK) return st;
    *total_ms = ctx->prof_ms[kernel_id];
    *launches = ctx->prof_launches[kernel_id];
    return RG_OK;
}

rg_status rg_stream_create(rg_ctx* ctx, int32_t first_cu, int32_t num_cus, void** stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, stream, "rg_stream_create: stream is NULL");
    RG_REQUIRE(ctx, first_cu >= 0 && num_cus >= 1 && first_cu + num_cus <= ctx->num_cus,
               "rg_stream_create: compute units [%d, %d) are not within the device's %d", first_cu, first_cu + num_cus, ctx->num_cus);
    RG_HIP(ctx, hipSetDevice(ctx->device));
    const int words = (ctx->num_cus + 31) / 32;
    std::vector<uint32_t> mask((size_t)words, 0u);
    for (int cu = first_cu; cu < first_cu + num_cus; ++cu) mask[(size_t)(cu >> 5)] |= 1u << (cu & 31);
    hipStream_t s = nullptr;
    RG_HIP(ctx, hipExtStreamCreateWithCUMask(&s, (uint32_t)words, mask.data()));
    ctx->streams.push_back(s);
    *stream = (void*)s;
    return RG_OK;
}

rg_status rg_stream_destroy(rg_ctx* ctx, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    auto it = std::find(ctx->streams.begin(), ctx->streams.end(), (hipStream_t)stream);
    RG_REQUIRE(ctx, it != ctx->streams.end(), "rg_stream_destroy: not a stream of this context's rg_stream_create");
    ctx->streams.erase(it);
    RG_HIP(ctx, hipSetDevice(ctx->device));
    RG_HIP(ctx, hipStreamSynchronize((hipStream_t)stream));
    RG_HIP(ctx, hipStreamDestroy((hipStream_t)stream));
    return RG_OK;
}

}  // extern "C"

int rg_prof_begin(rg_ctx* ctx, int kernel, hipStream_t s) {
    if (!ctx->profiling || !((ctx->prof_mask >> kernel) & 1u)) return -1;
    RgProfSpan span;
    span.kernel = kernel;
    if (!ctx->free_events.empty()) {
        span.start = ctx->free_events.back().first;
        span.stop = ctx->free_events.back().second;
        ctx->free_events.pop_back();
    } else {
        if (hipEventCreate(&span.start) != hipSuccess) return -1;
        if (hipEventCreate(&span.stop) != hipSuccess) { (void)hipEventDestroy(span.start); return -1; }
    }
    (void)hipEventRecord(span.start, s);
    ctx->spans.push_back(span);
    return (int)ctx->spans.size() - 1;
}

void rg_prof_end(rg_ctx* ctx, int token, hipStream_t s) {
    if (token < 0) return;
    (void)hipEventRecord(ctx->spans[token].stop, s);
}
