// Internal declarations shared by the HIP translation units of librapidgnn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string>
#include <vector>

#include "rapidgnn.h"

// A growable device allocation owned by the context.
struct RgBuf {
    void* p = nullptr;
    size_t bytes = 0;
};

struct RgProfSpan {
    hipEvent_t start, stop;
    int kernel;
};

// Launch-shape knobs, read from the environment once per context (rg_create); the defaults are the swept optima.
struct RgKnobs {
    int gather_unroll = 2;            // RG_GATHER_UNROLL: 16-byte chunks in flight per lane of the HBM gather (2, 4 or 8)
    int gather_blocks_per_cu = 0;     // RG_GATHER_BLOCKS_PER_CU: grid cap of the HBM gather (0 = one step per wavefront)
    int pull_blocks = 16;             // RG_PULL_BLOCKS / RG_PULL_THREADS: grid of the host-link pull kernels
    int pull_threads = 1024;
    int pull_rows = 4;                // RG_PULL_ROWS: rows in flight per lane group of the pull kernel (4 or 8)
    int miss_blocks = 192;            // RG_MISS_BLOCKS / RG_MISS_THREADS: grid of the miss-row kernel
    int miss_threads = 256;
    int xcd_map = 1;                  // RG_XCD_MAP=0: batch-major workgroup order in the sampler instead of one batch per XCD
};

struct rg_ctx {
    int device = 0;
    int num_cus = 256;
    char err[512] = {0};
    RgKnobs knobs;

    // sampler scratch
    RgBuf visited;      // uint32[ceil(N/32)] bitmap of cumulative-frontier members
    RgBuf marked;       // uint32[ceil(N/32)] bitmap of every id a batch has met: frontier members and the current hop's picks
    RgBuf pos;          // int32[N] position of a node in the cumulative frontier (valid for members only)
    RgBuf chunk_sum;    // int32[] per-256-node chunk edge counts / bitmap block counts
    RgBuf row_start;    // int64[max_frontier] adjacency row start of every frontier node (current hop)
    RgBuf row_deg;      // int32[max_frontier] its degree
    RgBuf first_key;    // int32[N] per batch, first-seen node order only (see SampleScratch)
    int last_sample_group = 0;     // batches of the last completed sampling call: their `visited` bitmaps are the batches'
    int64_t last_sample_nodes = 0; // input-node sets (rg_access_histogram_sampled), on graphs of this many nodes
    bool sampler_dirty = false;   // a sampling call was cut short by an error: the first-edge keys may hold stale entries
    // schedule scratch
    RgBuf sched_keys;   // uint64[npad]
    RgBuf sched_ids;    // int32[npad]
    // top-K scratch
    RgBuf topk_ctl;     // TopkCtl
    RgBuf topk_blk;     // int32[2 * nblocks]
    RgBuf topk_caps;    // rg_cache_hit_curve: int64[num_capacities] capacities, then uint32[num_capacities] flags
    // prefetch scratch
    RgBuf pf_list;      // int32[2 * n]: (slot, remote row) pairs still to pull
    RgBuf pf_ctl;       // uint32[4]: [0] = number of pairs
    RgBuf claim_bits, claim_blk;     // rg_plan_sampled: the group's new-node bits and per-block pair counts
    RgBuf plan_cursor;               // rg_plan_prefetch: per-chunk per-batch counts (ordered plan) or scatter cursors
    // gather scratch
    // RG_GATHER_TICKETS entries each, so that several batches can be classified by one launch ahead of their copies
    RgBuf gather_src;   // [ticket][gather_cap] uint32: resolved location word per output row
    RgBuf miss_list;    // [ticket][2 * gather_cap] int32: (output row, remote row) pairs of the miss rows
    RgBuf gather_ctl;   // [ticket][16] uint32: [0] = number of misses
    int64_t gather_cap = 0;                                  // rows per ticket the buffers hold
    int64_t gather_rows[RG_GATHER_TICKETS] = {-1, -1, -1, -1, -1, -1, -1, -1};   // rows a ticket was prepared for (-1: none)
    hipEvent_t ev_classified = nullptr, ev_miss_done = nullptr;
    void* static_scratch = nullptr;   // device address of the library's file-scope gather scratch on ctx->device
    std::vector<hipStream_t> streams;   // streams made by rg_stream_create and not yet destroyed (rg_destroy takes the rest)

    // profiling
    bool profiling = false;
    uint32_t prof_mask = 0xFFFFFFFFu;  // bit k: launches of kernel id k are bracketed while profiling is on
    std::vector<RgProfSpan> spans;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> free_events;
    double prof_ms[RG_K_COUNT_] = {0};
    int64_t prof_launches[RG_K_COUNT_] = {0};
};

rg_status rg_set_error(rg_ctx* ctx, rg_status code, const char* fmt, ...);
rg_status rg_ensure(rg_ctx* ctx, RgBuf& buf, size_t bytes, bool zero_new = false);
// RG_OK if kernels on the ctx's device may dereference p (device, managed or pinned/registered host memory).
rg_status rg_check_device_readable(rg_ctx* ctx, const void* p, const char* what);
// Makes every gather ticket hold at least `rows` rows (a reallocation invalidates prepared tickets).
rg_status rg_gather_reserve(rg_ctx* ctx, int64_t rows);
// Sizes the sampler scratch for `group` batches side by side on a graph of num_nodes nodes with cumulative
// frontiers of up to max_frontier nodes (what rg_sample_blocks_group would otherwise grow on demand).
rg_status rg_sampler_reserve(rg_ctx* ctx, int64_t num_nodes, int64_t max_frontier, int group, int64_t max_edges = 0,
                             bool first_seen = false);
// Resolves the device address of the file-scope gather scratch for ctx->device (the device must be current).
rg_status rg_gather_static_init(rg_ctx* ctx);
// Profiling brackets (no-ops unless profiling is enabled).
int rg_prof_begin(rg_ctx* ctx, int kernel, hipStream_t s);
void rg_prof_end(rg_ctx* ctx, int token, hipStream_t s);

#define RG_HIP(ctx, expr)                                                                     \
    do {                                                                                      \
        hipError_t rg_e_ = (expr);                                                            \
        if (rg_e_ != hipSuccess)                                                              \
            return rg_set_error((ctx), RG_ERR_HIP, "%s failed: %s (%s:%d)", #expr,            \
                                hipGetErrorString(rg_e_), __FILE__, __LINE__);                \
    } while (0)

#define RG_LAUNCH_CHECK(ctx, name)                                                            \
    do {                                                                                      \
        hipError_t rg_e_ = hipGetLastError();                                                 \
        if (rg_e_ != hipSuccess)                                                              \
            return rg_set_error((ctx), RG_ERR_HIP, "launch of %s failed: %s", name,           \
                                hipGetErrorString(rg_e_));                                    \
    } while (0)

#define RG_REQUIRE(ctx, cond, ...)                                                            \
    do {                                                                                      \
        if (!(cond)) return rg_set_error((ctx), RG_ERR_INVALID_ARG, __VA_ARGS__);             \
    } while (0)

static inline int64_t rg_div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t rg_min64(int64_t a, int64_t b) { return a < b ? a : b; }
static inline int64_t rg_max64(int64_t a, int64_t b) { return a > b ? a : b; }

// ---------------------------------------------------------------- device helpers
#define RG_WAVE 64

// Philox4x32-10 block function (Salmon et al., SC'11, Section 3.3).
__device__ __forceinline__ void rg_philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ int rg_lane() { return threadIdx.x & (RG_WAVE - 1); }

// Inclusive prefix sum across the 64 lanes of a wavefront.
__device__ __forceinline__ int rg_wave_incl_scan(int x) {
    const int lane = rg_lane();
#pragma unroll
    for (int off = 1; off < RG_WAVE; off <<= 1) {
        const int y = __shfl_up(x, off, RG_WAVE);
        if (lane >= off) x += y;
    }
    return x;
}

__device__ __forceinline__ int rg_wave_sum(int x) {
#pragma unroll
    for (int off = RG_WAVE / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, RG_WAVE);
    return x;
}

// Exclusive prefix sum over a workgroup of NW wavefronts; returns the exclusive prefix of x and
// stores the workgroup total in *total.  smem must hold NW + 1 ints.  Contains barriers: every
// thread of the workgroup must call it.
template <int NW>
__device__ __forceinline__ int rg_block_excl_scan(int x, int* smem, int* total) {
    const int lane = rg_lane();
    const int wave = threadIdx.x >> 6;
    const int incl = rg_wave_incl_scan(x);
    __syncthreads();                      // protect smem from a previous use
    if (lane == RG_WAVE - 1) smem[wave] = incl;
    __syncthreads();
    int wave_base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int s = smem[w];
        if (w < wave) wave_base += s;
        tot += s;
    }
    *total = tot;
    return wave_base + incl - x;
}
