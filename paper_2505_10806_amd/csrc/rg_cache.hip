// Access-frequency histogram (Section IV, offline stage), TopHot selection (Alg. 1 line 3), the hit curve
// against cache size (Section V), and VectorPull (Alg. 1 line 4) in its two forms: one bulk pull, or pulls by
// first use ahead of the gathers (the prefetcher of Section III: with a per-batch claim pass or from a
// per-epoch plan).
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

// Epoch-level histogram over many sampled batches.  Every tier after the seeds is ascending by id, so a
// workgroup that owns the id range [v0, v0 + kHistRange) finds its entries of each (batch, tier) run by
// binary search, accumulates them in an LDS-private copy of its counters with LDS atomics, and adds the
// range to `counts` once with plain coalesced read-modify-writes: no global atomics, every id read once.
constexpr int kHistRange = 8192;       // counters per workgroup (32 KB of LDS)
constexpr int kHistRangeFirst = 4096;  // when the first batch of every id is tracked as well (16 KB + 16 KB)
constexpr int kHistRunTile = 1024;     // runs whose bounds are resolved per pass

__device__ __forceinline__ int rg_lower_bound(const int32_t* __restrict__ a, int n, int key) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// FIRST: also record, per id, the smallest batch index whose list contains it (first_batch[v] = min(old, b)).
template <int RANGE, bool FIRST>
__global__ void __launch_bounds__(1024) k_histogram_runs(const int32_t* __restrict__ nodes, int64_t batch_stride,
                                                         const int32_t* __restrict__ tier_off, int num_batches, int num_hops,
                                                         uint32_t* __restrict__ counts, uint32_t* __restrict__ first_batch,
                                                         int64_t num_nodes) {
    __shared__ uint32_t priv[RANGE];
    __shared__ uint32_t firstb[FIRST ? RANGE : 1];
    __shared__ int seg_lo[kHistRunTile];
    __shared__ int seg_hi[kHistRunTile];
    const int64_t v0 = (int64_t)blockIdx.x * RANGE;
    const int64_t v1 = v0 + RANGE < num_nodes ? v0 + RANGE : num_nodes;
    for (int j = threadIdx.x; j < RANGE; j += blockDim.x) {
        priv[j] = 0u;
        if (FIRST) firstb[j] = 0xFFFFFFFFu;
    }
    const int num_runs = num_batches * num_hops;
    const int wave = threadIdx.x >> 6, lane = rg_lane(), nwaves = blockDim.x >> 6;
    for (int tile = 0; tile < num_runs; tile += kHistRunTile) {
        __syncthreads();                                  // priv zeroed / previous tile's segments consumed
        const int r = tile + threadIdx.x;
        if (threadIdx.x < kHistRunTile && r < num_runs) {
            const int b = r / num_hops, t = r % num_hops + 1;          // tier t of batch b
            const int32_t* to = tier_off + (int64_t)b * (num_hops + 2);
            const int begin = to[t], len = to[t + 1] - to[t];
            const int32_t* run = nodes + (int64_t)b * batch_stride + begin;
            seg_lo[threadIdx.x] = begin + rg_lower_bound(run, len, (int)v0);
            seg_hi[threadIdx.x] = begin + rg_lower_bound(run, len, (int)v1);
        }
        __syncthreads();
        const int in_tile = num_runs - tile < kHistRunTile ? num_runs - tile : kHistRunTile;
        for (int q = wave; q < in_tile; q += nwaves) {                  // one wavefront per run segment
            const int b = (tile + q) / num_hops;
            const int32_t* base = nodes + (int64_t)b * batch_stride;
            const int hi = seg_hi[q];
            for (int e = seg_lo[q] + lane; e < hi; e += RG_WAVE) {
                const uint32_t off = (uint32_t)(base[e] - (int)v0);
                if (off < (uint32_t)RANGE) {                            // always true for ascending tiers
                    atomicAdd(&priv[off], 1u);
                    if (FIRST) atomicMin(&firstb[off], (uint32_t)b);
                }
            }
        }
    }
    __syncthreads();
    for (int64_t j = threadIdx.x; v0 + j < v1; j += blockDim.x) {
        const uint32_t c = priv[j];
        if (c) {
            counts[v0 + j] += c;
            if (FIRST) { const uint32_t f = firstb[j], g = first_batch[v0 + j]; if (f < g) first_batch[v0 + j] = f; }
        }
    }
}

// Seeds are in caller order (not sorted): one global atomic each.
__global__ void __launch_bounds__(256) k_histogram_seeds(const int32_t* __restrict__ nodes, int64_t batch_stride,
                                                         const int32_t* __restrict__ tier_off, int num_hops,
                                                         uint32_t* __restrict__ counts, uint32_t* __restrict__ first_batch) {
    const int b = blockIdx.y;
    const int n_seeds = tier_off[(int64_t)b * (num_hops + 2) + 1];
    const int32_t* base = nodes + (int64_t)b * batch_stride;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_seeds; i += gridDim.x * blockDim.x) {
        atomicAdd(&counts[base[i]], 1u);
        if (first_batch) atomicMin(&first_batch[base[i]], (uint32_t)b);
    }
}

// ---------------------------------------------------------------------------- threshold select
// Finds the count threshold T of the K_eff-th best candidate.  Access counts are bounded by the number of batches of
// the period (a few hundred), so one streaming pass with a histogram of the counts clamped to kLowBins - 1 resolves T
// whenever T < kLowBins - 1.  Only when the K_eff-th best candidate sits in the clamped last bin do the four byte passes
// of a most-significant-byte-first radix select run; otherwise their kernels return at once.
constexpr int kLowBins = 2048;
constexpr int kBallotBins = 4;       // counts 1..kBallotBins are tallied with wave ballots instead of LDS atomics

struct TopkCtl {
    uint32_t prefix;     // the threshold T (radix passes: its resolved high bytes)
    uint32_t need;       // how many of the candidates tied with T are to be taken
    uint32_t k_eff;
    uint32_t resolved;   // 1: T and need are final, the radix passes are skipped
    uint32_t hist[4][256];
    uint32_t low[kLowBins];          // candidates per clamped count
    unsigned long long ovf_sum;      // sum of the counts of the candidates in the last (clamped) bin
};

__device__ __forceinline__ bool rg_is_candidate(uint32_t home_word, uint32_t count) {
    return (home_word >> RG_TAG_SHIFT) == RG_TAG_REMOTE && count >= 1u;
}

// force_radix = the address of a flag that, when set, sends this selection through the radix passes.
__global__ void __launch_bounds__(256) k_topk_init(TopkCtl* __restrict__ ctl, const uint32_t* __restrict__ skip_flag) {
    if (skip_flag) {                 // a later selection of the hit curve: keep the low histogram, redo only the radix state
        for (int i = threadIdx.x; i < 4 * 256; i += 256) (&ctl->hist[0][0])[i] = 0u;
        if (threadIdx.x == 0) { ctl->prefix = 0u; ctl->need = 0u; ctl->k_eff = 0u; ctl->resolved = *skip_flag; }
        return;
    }
    uint32_t* w = (uint32_t*)ctl;
    for (int i = threadIdx.x; i < (int)(sizeof(TopkCtl) / 4); i += 256) w[i] = 0u;
}

// low[min(count, kLowBins - 1)] += 1 for every candidate; ovf_sum += count for those in the last bin.
__global__ void __launch_bounds__(256) k_topk_hist_low(const uint32_t* __restrict__ counts, const int32_t* __restrict__ home, int64_t n,
                                                       TopkCtl* __restrict__ ctl) {
    __shared__ uint32_t h[kLowBins];
    __shared__ unsigned long long ovf_s;
    for (int i = threadIdx.x; i < kLowBins; i += 256) h[i] = 0u;
    if (threadIdx.x == 0) ovf_s = 0ull;
    __syncthreads();
    unsigned long long ovf = 0ull;
    const int lane = rg_lane();
    for (int64_t v0 = (int64_t)blockIdx.x * 256; v0 < n; v0 += (int64_t)gridDim.x * 256) {     // uniform per workgroup
        const int64_t v = v0 + threadIdx.x;
        uint32_t bin = 0u;                                   // bin 0: not a candidate
        if (v < n) {
            const uint32_t c = counts[v];
            if (rg_is_candidate((uint32_t)home[v], c)) {
                bin = c < (uint32_t)(kLowBins - 1) ? c : (uint32_t)(kLowBins - 1);
                if (c >= (uint32_t)(kLowBins - 1)) ovf += c;
            }
        }
        // most candidates of a long-tailed distribution have a count of 1..4: one LDS atomic per wavefront for each
#pragma unroll
        for (uint32_t q = 1; q <= (uint32_t)kBallotBins; ++q) {
            const unsigned long long m = __ballot(bin == q);
            if (lane == 0 && m) atomicAdd(&h[q], (uint32_t)__popcll(m));
        }
        if (bin > (uint32_t)kBallotBins) atomicAdd(&h[bin], 1u);
    }
    if (ovf) atomicAdd(&ovf_s, ovf);
    __syncthreads();
    for (int i = threadIdx.x; i < kLowBins; i += 256) {
        const uint32_t mine = h[i];
        if (mine) atomicAdd(&ctl->low[i], mine);
    }
    if (threadIdx.x == 0 && ovf_s) atomicAdd(&ctl->ovf_sum, ovf_s);
}

// One workgroup: K_eff = min(capacity, #candidates); T = the bin holding the K_eff-th best candidate.
__global__ void __launch_bounds__(256) k_topk_pick_low(TopkCtl* __restrict__ ctl, int64_t capacity, int64_t* __restrict__ num_cached) {
    __shared__ int smem[256 / RG_WAVE + 1];
    constexpr int PER = kLowBins / 256;                      // thread t owns bins kLowBins-1-PER*t downwards
    uint32_t h[PER];
    int mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        h[j] = ctl->low[kLowBins - 1 - (PER * (int)threadIdx.x + j)];
        mine += (int)h[j];
    }
    int total;
    int above = rg_block_excl_scan<256 / RG_WAVE>(mine, smem, &total);     // candidates in strictly larger bins
    const uint64_t k = (uint64_t)capacity < (uint64_t)total ? (uint64_t)capacity : (uint64_t)total;
    if (threadIdx.x == 0) {
        ctl->k_eff = (uint32_t)k;
        if (num_cached) *num_cached = (int64_t)k;
        if (k == 0) { ctl->prefix = 0xFFFFFFFFu; ctl->need = 0u; ctl->resolved = 1u; }   // a threshold no count reaches
    }
    if (k == 0) return;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int bin = kLowBins - 1 - (PER * (int)threadIdx.x + j);
        if ((uint64_t)above < k && k <= (uint64_t)above + h[j]) {         // exactly one bin satisfies this
            if (bin < kLowBins - 1) { ctl->prefix = (uint32_t)bin; ctl->need = (uint32_t)(k - above); ctl->resolved = 1u; }
            else ctl->resolved = 0u;                                       // inside the clamped bin: radix passes decide
        }
        above += (int)h[j];
    }
}

// Histogram of byte `pass` (0 = most significant) of the counts of candidates that match the prefix.
__global__ void __launch_bounds__(256) k_topk_hist(const uint32_t* __restrict__ counts, const int32_t* __restrict__ home, int64_t n,
                                                   int pass, TopkCtl* __restrict__ ctl) {
    __shared__ uint32_t h[256];
    if (ctl->resolved) return;                               // uniform
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
__global__ void __launch_bounds__(256) k_topk_pick(TopkCtl* __restrict__ ctl, int pass, int64_t capacity) {
    __shared__ uint32_t h[256];
    __shared__ uint32_t above[256];      // candidates in strictly larger byte values
    __shared__ uint32_t need_s;
    if (ctl->resolved) return;           // uniform
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

constexpr int kCapChunk = 64;
struct CapChunk { int64_t v[kCapChunk]; };

__global__ void k_store_caps(int64_t* __restrict__ dst, const CapChunk chunk, int count) {
    if ((int)threadIdx.x < count) dst[threadIdx.x] = chunk.v[threadIdx.x];
}

// One workgroup, after k_topk_hist_low: requests served by a cache of each capacity, read off the histogram.
// hits[j] = sum of the counts above the threshold of capacity j + (ties taken) x threshold.  A capacity whose
// threshold lies inside the clamped last bin is left to the radix passes: radix_flag[j] = 0 ("not resolved").
__global__ void __launch_bounds__(256) k_hit_curve_low(const TopkCtl* __restrict__ ctl, const int64_t* __restrict__ capacities,
                                                       int num_capacities, unsigned long long* __restrict__ hits,
                                                       unsigned long long* __restrict__ total_out, uint32_t* __restrict__ resolved_flag) {
    __shared__ uint32_t cnt_above[kLowBins];                 // candidates with a larger clamped count
    __shared__ unsigned long long sum_above[kLowBins];       // and the sum of their counts
    __shared__ unsigned long long grand_s;
    if (threadIdx.x == 0) {
        uint32_t cnt = 0u;
        unsigned long long sum = 0ull;
        for (int b = kLowBins - 1; b >= 1; --b) {
            cnt_above[b] = cnt;
            sum_above[b] = sum;
            const uint32_t hb = ctl->low[b];
            cnt += hb;
            sum += b == kLowBins - 1 ? ctl->ovf_sum : (unsigned long long)hb * (unsigned long long)b;
        }
        cnt_above[0] = cnt;                                  // = number of candidates (bin 0 holds none)
        sum_above[0] = sum;
        grand_s = sum;
        if (total_out) *total_out = sum;
    }
    __syncthreads();
    const uint32_t n_cand = cnt_above[0];
    for (int j = threadIdx.x; j < num_capacities; j += 256) {
        const uint64_t cap = (uint64_t)capacities[j];
        const uint32_t k = cap < (uint64_t)n_cand ? (uint32_t)cap : n_cand;
        if (k == 0u) { hits[j] = 0ull; resolved_flag[j] = 1u; continue; }
        if (k == n_cand) { hits[j] = grand_s; resolved_flag[j] = 1u; continue; }
        // the threshold bin T holds the k-th best candidate: cnt_above[T] < k <= cnt_above[T - 1].  cnt_above falls as
        // the bin index rises and cnt_above[kLowBins - 1] = 0 < k, so T is the smallest bin with cnt_above[T] < k.
        int lo = 1, hi = kLowBins - 1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (cnt_above[mid] < k) hi = mid; else lo = mid + 1;
        }
        if (lo == kLowBins - 1) { hits[j] = 0ull; resolved_flag[j] = 0u; continue; }
        hits[j] = sum_above[lo] + (unsigned long long)(k - cnt_above[lo]) * (unsigned long long)lo;
        resolved_flag[j] = 1u;
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

// Radix path of the hit curve: hits += sum of the counts above the threshold plus (ties taken) x threshold.
// `resolved` = 1 when the histogram pass already produced this capacity's value.
__global__ void __launch_bounds__(256) k_hit_sum(const uint32_t* __restrict__ counts, const int32_t* __restrict__ home, int64_t n,
                                                 const TopkCtl* __restrict__ ctl, const uint32_t* __restrict__ resolved,
                                                 unsigned long long* __restrict__ hits) {
    if (*resolved) return;                                   // uniform
    const uint32_t T = ctl->prefix;
    unsigned long long above = 0ull;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t c = counts[v];
        if (rg_is_candidate((uint32_t)home[v], c) && c > T) above += c;
    }
#pragma unroll
    for (int off = RG_WAVE / 2; off > 0; off >>= 1) above += __shfl_xor(above, off, RG_WAVE);
    __shared__ unsigned long long pa[4];
    if (rg_lane() == 0) pa[threadIdx.x >> 6] = above;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long a = pa[0] + pa[1] + pa[2] + pa[3];
        if (blockIdx.x == 0) a += (unsigned long long)ctl->need * (unsigned long long)T;   // need == 0 when nothing is selected
        if (a) atomicAdd(hits, a);
    }
}

// ---------------------------------------------------------------------------- VectorPull
// cache_rows[slot] = remote_store[row(home[cache_ids[slot]])] for slot < *num_cached.
template <int VEC>
__global__ void __launch_bounds__(256) k_cache_fill(const int32_t* __restrict__ cache_ids, const int32_t* __restrict__ home,
                                                    const int64_t* __restrict__ num_cached, const float* __restrict__ remote_store,
                                                    int64_t remote_stride, float* __restrict__ cache_rows, int64_t cache_stride,
                                                    int cpr, int log2L, int tail) {
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
            const bool head_only = tail < VEC && c == cpr - 1;      // only the row's own floats of its last chunk are stored
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u]) {
                    if (head_only) rg_store_head(&dst[u][c], val[u], tail);
                    else dst[u][c] = val[u];
                }
        }
    }
}

// filled[w] = all-ones for slots below *num_cached (value = 1) or all-zero (value = 0).
__global__ void __launch_bounds__(256) k_set_filled(uint32_t* __restrict__ filled, int64_t words, const int64_t* __restrict__ num_cached,
                                                    int value) {
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= words) return;
    uint32_t bits = 0u;
    if (value) {
        const int64_t k = *num_cached;
        const int64_t lo = w * 32;
        if (k >= lo + 32) bits = 0xFFFFFFFFu;
        else if (k > lo) bits = (1u << (uint32_t)(k - lo)) - 1u;
    }
    filled[w] = bits;
}

__global__ void k_prefetch_reset(uint32_t* __restrict__ pctl) {
    if (threadIdx.x == 0) pctl[0] = 0u;
}

// For every listed node whose location word names a cache slot that is not yet resident: claim the slot
// (atomic test-and-set of its bit) and append (slot, remote row) to the pull list.
__global__ void __launch_bounds__(256) k_prefetch_select(const int32_t* __restrict__ nodes, int64_t n, const int32_t* __restrict__ n_dev,
                                                         const int32_t* __restrict__ loc, const int32_t* __restrict__ home,
                                                         uint32_t* __restrict__ filled, int32_t* __restrict__ list,
                                                         uint32_t* __restrict__ pctl, int mirror) {
    __shared__ int smem[256 / RG_WAVE + 1];
    __shared__ uint32_t base_s;
    int64_t n_act = n;
    if (n_dev) { const int64_t d = *n_dev; n_act = d < n ? d : n; }
    if ((int64_t)blockIdx.x * blockDim.x >= n_act) return;        // uniform per workgroup
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int take = 0;
    uint32_t slot = 0u, rrow = 0u;
    if (i < n_act) {
        const int32_t v = nodes[i];
        bool wanted;
        if (mirror) {       // every remote row a batch names will be cached, at the row it has in the remote store
            const uint32_t hw = (uint32_t)home[v];
            wanted = (hw >> RG_TAG_SHIFT) == RG_TAG_REMOTE;
            slot = rrow = hw & RG_ROW_MASK;
        } else {
            const uint32_t w = (uint32_t)loc[v];
            wanted = (w >> RG_TAG_SHIFT) == RG_TAG_CACHE;
            slot = w & RG_ROW_MASK;
        }
        if (wanted) {
            const uint32_t bit = 1u << (slot & 31u);
            if (!(filled[slot >> 5] & bit)) {
                const uint32_t old = atomicOr(&filled[slot >> 5], bit);
                if (!(old & bit)) { take = 1; rrow = (uint32_t)home[v] & RG_ROW_MASK; }
            }
        }
    }
    int total;
    const int excl = rg_block_excl_scan<256 / RG_WAVE>(take, smem, &total);
    if (total == 0) return;                                        // uniform
    if (threadIdx.x == 0) base_s = atomicAdd(&pctl[0], (uint32_t)total);
    __syncthreads();
    if (take) {
        const int64_t j = (int64_t)base_s + excl;
        list[2 * j] = (int32_t)slot;
        list[2 * j + 1] = (int32_t)rrow;
    }
}

// dst_rows[list[2j]] = src_rows[list[2j+1]] for every pair of the list (host link or HBM source alike); with `mark` the
// destination rows' resident bits are set by the same kernel.
// The pairs are list[0..pctl[0]) or, when seg_off is given, list[seg_off[0]..seg_off[1]).
template <int VEC, int U>
__global__ void __launch_bounds__(1024) k_prefetch_pull(const int32_t* __restrict__ list, const uint32_t* __restrict__ pctl,
                                                       const int32_t* __restrict__ seg_off,
                                                       const float* __restrict__ remote_store, int64_t remote_stride,
                                                       float* __restrict__ cache_rows, int64_t cache_stride, int64_t dst_rows,
                                                       int cpr, int log2L, int tail, uint32_t* __restrict__ mark) {
    typedef typename RgVec<VEC>::type V;
    int64_t n;
    if (seg_off) { list += 2 * (int64_t)seg_off[0]; n = seg_off[1] - seg_off[0]; } else { n = pctl[0]; }
    const int lane = rg_lane();
    const int L = 1 << log2L;
    const int R = RG_WAVE >> log2L;
    const int sub = lane >> log2L;
    const int c0 = lane & (L - 1);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t j0 = wave * (R * U); j0 < n; j0 += nwaves * (R * U)) {
        // Few wavefronts feed the link, so each must keep all U row loads in flight: the loads are unconditional
        // (a lane group without a row reads destination row 0, which is in HBM and costs no link traffic; the value
        // is discarded) and only the stores are predicated.
        const V* src[U];
        V* dst[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t j = j0 + u * R + sub;
            src[u] = (const V*)cache_rows;
            dst[u] = nullptr;
            if (j < n) {
                const int64_t slot = list[2 * j], rrow = list[2 * j + 1];
                if (slot >= 0 && slot < dst_rows) {      // a list built for another destination must not write outside this one
                    src[u] = (const V*)(remote_store + rrow * remote_stride);
                    dst[u] = (V*)(cache_rows + slot * cache_stride);
                    // the row's resident bit, by the first lane of its group (whoever reads the bits waits for this kernel)
                    if (mark && c0 == 0) atomicOr(&mark[slot >> 5], 1u << (slot & 31));
                }
            }
        }
        for (int c = c0; c < cpr; c += L) {
            V val[U];
#pragma unroll
            for (int u = 0; u < U; ++u) val[u] = src[u][c];
            const bool head_only = tail < VEC && c == cpr - 1;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u]) {
                    if (head_only) rg_store_head(&dst[u][c], val[u], tail);
                    else dst[u][c] = val[u];
                }
        }
    }
}

// ---------------------------------------------------------------------------- prefetch plan
// counters[b + 1] += 1 for every selected slot whose node is first used by batch b (b = num_batches: by none).
__global__ void __launch_bounds__(256) k_plan_count(const int32_t* __restrict__ cache_ids, const int64_t* __restrict__ num_cached,
                                                    const uint32_t* __restrict__ first_batch, int num_batches,
                                                    int32_t* __restrict__ counters) {
    const int64_t k = *num_cached;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < k; s += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t f = first_batch[cache_ids[s]];
        atomicAdd(&counters[(f < (uint32_t)num_batches ? (int)f : num_batches) + 1], 1);
    }
}

// One workgroup: offsets[0] = 0, offsets[b + 1] = inclusive prefix of the counters; cursor[b] = offsets[b].
__global__ void __launch_bounds__(1024) k_plan_scan(int32_t* __restrict__ offsets, int32_t* __restrict__ cursor, int n_seg) {
    __shared__ int smem[1024 / RG_WAVE + 1];
    __shared__ int carry_s;
    if (threadIdx.x == 0) { carry_s = 0; offsets[0] = 0; }
    __syncthreads();
    for (int base = 0; base < n_seg; base += 1024) {
        const int i = base + threadIdx.x;
        const int x = i < n_seg ? offsets[i + 1] : 0;
        int total;
        const int excl = rg_block_excl_scan<1024 / RG_WAVE>(x, smem, &total);
        const int carry = carry_s;
        if (i < n_seg) { offsets[i + 1] = carry + excl + x; cursor[i] = carry + excl; }
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
}

// list[cursor[b]++] = (slot, remote row).  The order inside a segment is unspecified; the rows pulled are not.
__global__ void __launch_bounds__(256) k_plan_scatter(const int32_t* __restrict__ cache_ids, const int64_t* __restrict__ num_cached,
                                                      const uint32_t* __restrict__ first_batch, const int32_t* __restrict__ home,
                                                      int num_batches, int32_t* __restrict__ cursor, int32_t* __restrict__ list) {
    const int64_t k = *num_cached;
    for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < k; s += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = cache_ids[s];
        const uint32_t f = first_batch[v];
        const int64_t j = atomicAdd(&cursor[f < (uint32_t)num_batches ? (int)f : num_batches], 1);
        list[2 * j] = (int32_t)s;
        list[2 * j + 1] = (int32_t)((uint32_t)home[v] & RG_ROW_MASK);
    }
}

// Ordered plan (num_batches + 1 <= 1024): a stable counting sort of the slots by first batch, so that every segment
// lists its slots in ascending order, i.e. ascending remote rows: the link serves ascending host addresses
// measurably faster than scattered ones (52 against 46 GB/s on 1 KiB rows).
constexpr int kPlanChunk = 2048;     // slots per workgroup

__device__ __forceinline__ int rg_plan_key(const uint32_t* __restrict__ first_batch, int32_t v, int num_batches) {
    const uint32_t f = first_batch[v];
    return f < (uint32_t)num_batches ? (int)f : num_batches;
}

// hist[key * nblocks + blk] = number of slots of chunk blk first used by batch `key`.
__global__ void __launch_bounds__(1024) k_plan_block_hist(const int32_t* __restrict__ cache_ids, const int64_t* __restrict__ num_cached,
                                                          const uint32_t* __restrict__ first_batch, int num_batches, int nblocks,
                                                          int32_t* __restrict__ hist) {
    __shared__ int h[1024];
    const int n_seg = num_batches + 1;
    if ((int)threadIdx.x < n_seg) h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t k = *num_cached;
    const int64_t s0 = (int64_t)blockIdx.x * kPlanChunk;
    for (int i = threadIdx.x; i < kPlanChunk; i += blockDim.x) {
        const int64_t s = s0 + i;
        if (s < k) atomicAdd(&h[rg_plan_key(first_batch, cache_ids[s], num_batches)], 1);
    }
    __syncthreads();
    if ((int)threadIdx.x < n_seg) hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

// One workgroup: in-place exclusive scan of hist (key-major), segment starts to offsets[0..n_seg], total to offsets[n_seg].
__global__ void __launch_bounds__(1024) k_plan_hist_scan(int32_t* __restrict__ hist, int64_t n, int nblocks, int n_seg,
                                                         int32_t* __restrict__ offsets) {
    __shared__ int smem[1024 / RG_WAVE + 1];
    __shared__ int carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int x = i < n ? hist[i] : 0;
        int total;
        const int excl = rg_block_excl_scan<1024 / RG_WAVE>(x, smem, &total);
        const int carry = carry_s;
        if (i < n) {
            hist[i] = carry + excl;
            if (i % nblocks == 0) offsets[i / nblocks] = carry + excl;
        }
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) offsets[n_seg] = carry_s;
}

// Thread `key` of a workgroup walks the chunk's keys in slot order and emits the chunk's slots of that key.
__global__ void __launch_bounds__(1024) k_plan_block_scatter(const int32_t* __restrict__ cache_ids, const int64_t* __restrict__ num_cached,
                                                             const uint32_t* __restrict__ first_batch, const int32_t* __restrict__ home,
                                                             int num_batches, int nblocks, const int32_t* __restrict__ hist,
                                                             int32_t* __restrict__ list) {
    __shared__ uint16_t keys[kPlanChunk];
    __shared__ int32_t rrow[kPlanChunk];
    const int64_t k = *num_cached;
    const int64_t s0 = (int64_t)blockIdx.x * kPlanChunk;
    const int cnt = (int)(k - s0 < kPlanChunk ? (k - s0 > 0 ? k - s0 : 0) : kPlanChunk);
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
        const int32_t v = cache_ids[s0 + i];
        keys[i] = (uint16_t)rg_plan_key(first_batch, v, num_batches);
        rrow[i] = (int32_t)((uint32_t)home[v] & RG_ROW_MASK);
    }
    __syncthreads();
    const int key = threadIdx.x;
    if (key > num_batches) return;
    int64_t pos = hist[(int64_t)key * nblocks + blockIdx.x];
    for (int i = 0; i < cnt; ++i)
        if (keys[i] == key) {
            list[2 * pos] = (int32_t)(s0 + i);
            list[2 * pos + 1] = rrow[i];
            ++pos;
        }
}

// ---------------------------------------------------------------------------- plan segments straight from the sampler's bitmaps
// After the last hop the `visited` bitmaps of a sampler group are its batches' input-node sets.  The remote rows the
// group is the first to name are the new bits of their union against `claimed` (all nodes any earlier group named)
// whose home is the remote store: two streaming passes over N/32 words and one home[] lookup per new node, instead of
// one lookup and one probe per input node of every batch.  The pairs come out ascending by node id, i.e. by remote row.
constexpr int kClaimWordsPerBlock = 1024;   // 256 threads x 4 words

__device__ __forceinline__ int rg_count_remote(uint32_t bits, int64_t word, const int32_t* __restrict__ home) {
    int c = 0;
    while (bits) {
        const int j = __ffs(bits) - 1;
        bits &= bits - 1u;
        c += ((uint32_t)home[(word << 5) + j] >> RG_TAG_SHIFT) == RG_TAG_REMOTE;
    }
    return c;
}

__global__ void __launch_bounds__(256) k_claim_count(const uint32_t* __restrict__ visited, int64_t words, int group,
                                                     uint32_t* __restrict__ claimed, uint32_t* __restrict__ newbits,
                                                     const int32_t* __restrict__ home, int32_t* __restrict__ blk_count) {
    const int64_t w0 = (int64_t)blockIdx.x * kClaimWordsPerBlock + threadIdx.x * 4;
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t w = w0 + q;
        if (w >= words) break;
        uint32_t u = 0u;
        for (int g = 0; g < group; ++g) u |= visited[g * words + w];
        const uint32_t old = claimed[w];
        const uint32_t nw = u & ~old;
        newbits[w] = nw;
        if (nw) {
            claimed[w] = old | nw;
            c += rg_count_remote(nw, w, home);
        }
    }
    c = rg_wave_sum(c);
    __shared__ int part[4];
    if (rg_lane() == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) blk_count[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// One workgroup: block counts -> exclusive offsets; the segment's end goes behind its start in the plan's offsets.
__global__ void __launch_bounds__(1024) k_claim_scan(int32_t* __restrict__ blk_count, int nblocks, int32_t* __restrict__ seg_off,
                                                     int64_t list_capacity) {
    __shared__ int smem[1024 / RG_WAVE + 1];
    __shared__ int carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < nblocks; base += 1024) {
        const int i = base + threadIdx.x;
        const int x = i < nblocks ? blk_count[i] : 0;
        int total;
        const int excl = rg_block_excl_scan<1024 / RG_WAVE>(x, smem, &total);
        const int carry = carry_s;
        if (i < nblocks) blk_count[i] = carry + excl;
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        // a list that cannot take the segment (it holds one pair per remote row, so this means a caller error) gets an
        // empty segment instead of an overrun
        const int64_t end = (int64_t)seg_off[0] + carry_s;
        seg_off[1] = end <= list_capacity ? (int32_t)end : seg_off[0];
    }
}

__global__ void __launch_bounds__(256) k_claim_emit(const uint32_t* __restrict__ newbits, int64_t words, const int32_t* __restrict__ home,
                                                    const int32_t* __restrict__ blk_off, const int32_t* __restrict__ seg_off,
                                                    int32_t* __restrict__ list) {
    __shared__ int smem[256 / RG_WAVE + 1];
    if (seg_off[1] == seg_off[0]) return;                             // nothing new (or refused): uniform
    const int64_t w0 = (int64_t)blockIdx.x * kClaimWordsPerBlock + threadIdx.x * 4;
    uint32_t bits[4];
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        bits[q] = w0 + q < words ? newbits[w0 + q] : 0u;
        if (bits[q]) c += rg_count_remote(bits[q], w0 + q, home);
    }
    int total;
    const int excl = rg_block_excl_scan<256 / RG_WAVE>(c, smem, &total);
    if (total == 0) return;                                           // uniform
    int64_t j = (int64_t)seg_off[0] + blk_off[blockIdx.x] + excl;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t b = bits[q];
        while (b) {
            const int bit = __ffs(b) - 1;
            b &= b - 1u;
            const uint32_t hw = (uint32_t)home[((w0 + q) << 5) + bit];
            if ((hw >> RG_TAG_SHIFT) == RG_TAG_REMOTE) {
                const int32_t row = (int32_t)(hw & RG_ROW_MASK);
                list[2 * j] = row;                                    // mirrored cache: the row's place is its remote-store row
                list[2 * j + 1] = row;
                ++j;
            }
        }
    }
}

__global__ void __launch_bounds__(256) k_zero_i32(int32_t* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Launches the list-driven row copy.  `blocks` and `threads` bound the wavefronts in flight.
rg_status launch_list_copy(rg_ctx* ctx, const int32_t* list, const uint32_t* pctl, const float* src, int64_t src_stride,
                           float* dst, int64_t dst_stride, int64_t dst_rows, int32_t dim, int64_t n_upper, int64_t blocks,
                           int threads, hipStream_t s, const int32_t* seg_off = nullptr, uint32_t* mark = nullptr) {
    const void* ptrs[2] = {src, dst};
    const int64_t strides[2] = {src_stride, dst_stride};
    const int vec = rg_pick_vec(dim, ptrs, 2, strides, 2);
    const RgRowShape shp = rg_row_shape(dim, vec);
    const int U = ctx->knobs.pull_rows == 8 ? 8 : 4;        // rows in flight per lane group
    const int rows_per_block = (threads / RG_WAVE) * (RG_WAVE >> shp.log2L) * U;
    const int grid = (int)rg_max64(1, rg_min64(rg_div_up(n_upper, rows_per_block), blocks));
    const int tok = rg_prof_begin(ctx, RG_K_CACHE_FILL, s);
#define RG_LAUNCH_PULL(V, UU)                                                                                          \
    k_prefetch_pull<V, UU><<<grid, threads, 0, s>>>(list, pctl, seg_off, src, src_stride, dst, dst_stride, dst_rows, shp.cpr, \
                                                    shp.log2L, shp.tail, mark)
    if (vec == 4) { if (U == 8) RG_LAUNCH_PULL(4, 8); else RG_LAUNCH_PULL(4, 4); }
    else if (vec == 2) RG_LAUNCH_PULL(2, 4);
    else RG_LAUNCH_PULL(1, 4);
#undef RG_LAUNCH_PULL
    rg_prof_end(ctx, tok, s);
    RG_LAUNCH_CHECK(ctx, "k_prefetch_pull");
    return RG_OK;
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

rg_status rg_access_histogram_epoch(rg_ctx* ctx, const int32_t* nodes, int64_t batch_stride, const int32_t* tier_off,
                                    int32_t num_batches, int32_t num_hops, int32_t max_seeds, uint32_t* counts,
                                    uint32_t* first_batch, int64_t num_nodes, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, num_batches >= 0 && num_batches <= 65535, "rg_access_histogram_epoch: num_batches = %d not in [0, 65535]", num_batches);
    RG_REQUIRE(ctx, num_hops >= 1 && num_hops <= RG_MAX_HOPS, "rg_access_histogram_epoch: num_hops = %d not in [1,%d]", num_hops, RG_MAX_HOPS);
    RG_REQUIRE(ctx, batch_stride >= 0 && max_seeds >= 0 && num_nodes >= 0, "rg_access_histogram_epoch: negative size");
    RG_REQUIRE(ctx, num_nodes <= (int64_t)RG_ROW_MASK + 1, "rg_access_histogram_epoch: num_nodes exceeds 2^30");
    if (num_batches == 0 || num_nodes == 0) return RG_OK;
    RG_REQUIRE(ctx, nodes && tier_off && counts, "rg_access_histogram_epoch: null pointer");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int tok = rg_prof_begin(ctx, RG_K_HISTOGRAM, s);
    if (max_seeds > 0) {
        dim3 grid((unsigned)rg_min64(rg_div_up(max_seeds, 256), 64), (unsigned)num_batches);
        k_histogram_seeds<<<grid, 256, 0, s>>>(nodes, batch_stride, tier_off, num_hops, counts, first_batch);
    }
    if (first_batch)
        k_histogram_runs<kHistRangeFirst, true><<<(int)rg_div_up(num_nodes, kHistRangeFirst), 1024, 0, s>>>(
            nodes, batch_stride, tier_off, num_batches, num_hops, counts, first_batch, num_nodes);
    else
        k_histogram_runs<kHistRange, false><<<(int)rg_div_up(num_nodes, kHistRange), 1024, 0, s>>>(
            nodes, batch_stride, tier_off, num_batches, num_hops, counts, nullptr, num_nodes);
    rg_prof_end(ctx, tok, s);
    RG_LAUNCH_CHECK(ctx, "k_histogram_runs");
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
    RG_REQUIRE(ctx, cache->row_stride >= dim && (!remote_store || remote_stride >= dim), "rg_build_cache: row stride smaller than dim");
    RG_REQUIRE(ctx, remote_store || cache->filled || cache->capacity_rows == 0 || num_nodes == 0,
               "rg_build_cache: select-only mode (remote_store == NULL) needs cache->filled");
    RG_REQUIRE(ctx, cache->num_cached, "rg_build_cache: num_cached is NULL");
    RG_REQUIRE(ctx, cache->mirror_rows >= 0 && cache->mirror_rows <= cache->capacity_rows,
               "rg_build_cache: mirror_rows = %lld exceeds capacity_rows = %lld", (long long)cache->mirror_rows, (long long)cache->capacity_rows);
    RG_REQUIRE(ctx, cache->mirror_rows == 0 || (!remote_store && cache->home),
               "rg_build_cache: a mirrored cache is filled by rg_prefetch_cache_rows (remote_store must be NULL) and needs cache->home");
    RG_REQUIRE(ctx, num_nodes == 0 || (counts && home && cache->loc), "rg_build_cache: null node array");
    const bool may_select = cache->capacity_rows > 0 && num_nodes > 0;
    RG_REQUIRE(ctx, !may_select || (cache->cache_ids && cache->cache_rows), "rg_build_cache: null cache buffer");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    if (may_select && remote_store) {
        const rg_status chk = rg_check_device_readable(ctx, remote_store, "rg_build_cache: remote_store");
        if (chk != RG_OK) return chk;
    }
    hipStream_t s = (hipStream_t)stream;

    const int64_t nblocks = rg_max64(1, rg_div_up(num_nodes, kNodesPerBlock));
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->topk_ctl, sizeof(TopkCtl))) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->topk_blk, (size_t)nblocks * 8)) != RG_OK) return st;
    TopkCtl* ctl = (TopkCtl*)ctx->topk_ctl.p;
    int32_t* blk_gt = (int32_t*)ctx->topk_blk.p;
    int32_t* blk_eq = blk_gt + nblocks;

    k_topk_init<<<1, 256, 0, s>>>(ctl, nullptr);
    RG_LAUNCH_CHECK(ctx, "k_topk_init");
    const int hist_grid = (int)rg_max64(1, rg_min64(rg_div_up(num_nodes, 256 * 8), (int64_t)ctx->num_cus * 8));
    k_topk_hist_low<<<hist_grid, 256, 0, s>>>(counts, home, num_nodes, ctl);
    RG_LAUNCH_CHECK(ctx, "k_topk_hist_low");
    k_topk_pick_low<<<1, 256, 0, s>>>(ctl, cache->capacity_rows, cache->num_cached);
    RG_LAUNCH_CHECK(ctx, "k_topk_pick_low");
    for (int pass = 0; pass < 4; ++pass) {                   // return at once unless the threshold is in the clamped bin
        k_topk_hist<<<hist_grid, 256, 0, s>>>(counts, home, num_nodes, pass, ctl);
        RG_LAUNCH_CHECK(ctx, "k_topk_hist");
        k_topk_pick<<<1, 256, 0, s>>>(ctl, pass, cache->capacity_rows);
        RG_LAUNCH_CHECK(ctx, "k_topk_pick");
    }
    k_topk_count<<<(int)nblocks, 256, 0, s>>>(counts, home, num_nodes, ctl, blk_gt, blk_eq);
    RG_LAUNCH_CHECK(ctx, "k_topk_count");
    k_topk_scan<<<1, 1024, 0, s>>>(blk_gt, blk_eq, nblocks);
    RG_LAUNCH_CHECK(ctx, "k_topk_scan");
    k_topk_emit<<<(int)nblocks, 256, 0, s>>>(counts, home, num_nodes, ctl, blk_gt, blk_eq, cache->cache_ids, cache->loc);
    RG_LAUNCH_CHECK(ctx, "k_topk_emit");

    const int64_t filled_words = rg_div_up(rg_min64(cache->capacity_rows, num_nodes), 32);
    if (may_select && remote_store) {
        const void* ptrs[2] = {remote_store, cache->cache_rows};
        const int64_t strides[2] = {remote_stride, cache->row_stride};
        const int vec = rg_pick_vec(dim, ptrs, 2, strides, 2);
        const RgRowShape shp = rg_row_shape(dim, vec);
        const int64_t rows_ub = rg_min64(cache->capacity_rows, num_nodes);
        const int rows_per_block = 4 * (RG_WAVE >> shp.log2L) * 4;
        const int grid = (int)rg_max64(1, rg_min64(rg_div_up(rows_ub, rows_per_block), (int64_t)ctx->num_cus * 16));
        const int tok = rg_prof_begin(ctx, RG_K_CACHE_FILL, s);
        if (vec == 4)
            k_cache_fill<4><<<grid, 256, 0, s>>>(cache->cache_ids, home, cache->num_cached, remote_store, remote_stride, cache->cache_rows, cache->row_stride, shp.cpr, shp.log2L, shp.tail);
        else if (vec == 2)
            k_cache_fill<2><<<grid, 256, 0, s>>>(cache->cache_ids, home, cache->num_cached, remote_store, remote_stride, cache->cache_rows, cache->row_stride, shp.cpr, shp.log2L, shp.tail);
        else
            k_cache_fill<1><<<grid, 256, 0, s>>>(cache->cache_ids, home, cache->num_cached, remote_store, remote_stride, cache->cache_rows, cache->row_stride, shp.cpr, shp.log2L, shp.tail);
        rg_prof_end(ctx, tok, s);
        RG_LAUNCH_CHECK(ctx, "k_cache_fill");
    }
    if (cache->filled && filled_words > 0 && cache->mirror_rows == 0) {
        k_set_filled<<<(int)rg_div_up(filled_words, 256), 256, 0, s>>>(cache->filled, filled_words, cache->num_cached, remote_store ? 1 : 0);
        RG_LAUNCH_CHECK(ctx, "k_set_filled");
    }
    return RG_OK;
}

rg_status rg_cache_hit_curve(rg_ctx* ctx, const uint32_t* counts, const int32_t* home, int64_t num_nodes,
                             const int64_t* capacities, int32_t num_capacities, uint64_t* hits, uint64_t* remote_total,
                             void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, num_nodes >= 0 && num_nodes <= (int64_t)RG_ROW_MASK + 1, "rg_cache_hit_curve: num_nodes out of range");
    RG_REQUIRE(ctx, num_capacities >= 0 && num_capacities <= 4096, "rg_cache_hit_curve: num_capacities not in [0, 4096]");
    RG_REQUIRE(ctx, num_capacities == 0 || (capacities && hits), "rg_cache_hit_curve: null capacities / hits");
    RG_REQUIRE(ctx, num_nodes == 0 || (counts && home), "rg_cache_hit_curve: null node array");
    for (int j = 0; j < num_capacities; ++j)
        RG_REQUIRE(ctx, capacities[j] >= 0 && capacities[j] <= (int64_t)RG_ROW_MASK + 1, "rg_cache_hit_curve: capacities[%d] out of range", j);
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->topk_ctl, sizeof(TopkCtl))) != RG_OK) return st;
    TopkCtl* ctl = (TopkCtl*)ctx->topk_ctl.p;
    // device copy of the capacities and one "resolved" flag per capacity
    const size_t caps_bytes = (size_t)rg_max64(num_capacities, 1) * 8;
    if ((st = rg_ensure(ctx, ctx->topk_caps, caps_bytes + (size_t)rg_max64(num_capacities, 1) * 4)) != RG_OK) return st;
    int64_t* caps_dev = (int64_t*)ctx->topk_caps.p;
    uint32_t* resolved = (uint32_t*)((char*)ctx->topk_caps.p + caps_bytes);
    for (int j0 = 0; j0 < num_capacities; j0 += kCapChunk) {             // by value: the host array is not read after the call
        CapChunk chunk;
        const int cnt = num_capacities - j0 < kCapChunk ? num_capacities - j0 : kCapChunk;
        for (int j = 0; j < kCapChunk; ++j) chunk.v[j] = j < cnt ? capacities[j0 + j] : 0;
        k_store_caps<<<1, kCapChunk, 0, s>>>(caps_dev + j0, chunk, cnt);
        RG_LAUNCH_CHECK(ctx, "k_store_caps");
    }
    const int grid = (int)rg_max64(1, rg_min64(rg_div_up(num_nodes, 256 * 8), (int64_t)ctx->num_cus * 8));
    // one pass over the nodes gives the histogram of the counts; every capacity is read off it
    k_topk_init<<<1, 256, 0, s>>>(ctl, nullptr);
    RG_LAUNCH_CHECK(ctx, "k_topk_init");
    k_topk_hist_low<<<grid, 256, 0, s>>>(counts, home, num_nodes, ctl);
    RG_LAUNCH_CHECK(ctx, "k_topk_hist_low");
    k_hit_curve_low<<<1, 256, 0, s>>>(ctl, caps_dev, num_capacities, (unsigned long long*)hits, (unsigned long long*)remote_total, resolved);
    RG_LAUNCH_CHECK(ctx, "k_hit_curve_low");
    // capacities whose threshold lies among counts >= kLowBins - 1 (never the case when the counts are bounded by a few
    // hundred batches) go through the radix select one by one; for all others these kernels return at once
    for (int j = 0; j < num_capacities; ++j) {
        k_topk_init<<<1, 256, 0, s>>>(ctl, resolved + j);
        RG_LAUNCH_CHECK(ctx, "k_topk_init");
        for (int pass = 0; pass < 4; ++pass) {
            k_topk_hist<<<grid, 256, 0, s>>>(counts, home, num_nodes, pass, ctl);
            RG_LAUNCH_CHECK(ctx, "k_topk_hist");
            k_topk_pick<<<1, 256, 0, s>>>(ctl, pass, capacities[j]);
            RG_LAUNCH_CHECK(ctx, "k_topk_pick");
        }
        k_hit_sum<<<grid, 256, 0, s>>>(counts, home, num_nodes, ctl, resolved + j, (unsigned long long*)hits + j);
        RG_LAUNCH_CHECK(ctx, "k_hit_sum");
    }
    return RG_OK;
}

rg_status rg_prefetch_cache_rows(rg_ctx* ctx, const int32_t* input_nodes, int64_t n, const int32_t* n_dev,
                                 const rg_cache* cache, const int32_t* home, const float* remote_store,
                                 int64_t remote_stride, int32_t dim, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, n >= 0 && n <= (1ll << 31) - 1, "rg_prefetch_cache_rows: n = %lld out of range", (long long)n);
    if (n == 0) return RG_OK;
    RG_REQUIRE(ctx, cache && cache->filled && cache->cache_rows && (cache->loc || cache->mirror_rows > 0),
               "rg_prefetch_cache_rows: cache needs filled, cache_rows and (unless mirrored) loc");
    RG_REQUIRE(ctx, cache->mirror_rows >= 0 && cache->mirror_rows <= cache->capacity_rows,
               "rg_prefetch_cache_rows: mirror_rows = %lld exceeds capacity_rows = %lld", (long long)cache->mirror_rows, (long long)cache->capacity_rows);
    RG_REQUIRE(ctx, input_nodes && home && remote_store, "rg_prefetch_cache_rows: null pointer");
    RG_REQUIRE(ctx, dim >= 1 && cache->row_stride >= dim && remote_stride >= dim, "rg_prefetch_cache_rows: bad dim / stride");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    { const rg_status chk = rg_check_device_readable(ctx, remote_store, "rg_prefetch_cache_rows: remote_store"); if (chk != RG_OK) return chk; }
    hipStream_t s = (hipStream_t)stream;
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->pf_ctl, 64)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->pf_list, (size_t)n * 8)) != RG_OK) return st;
    uint32_t* pctl = (uint32_t*)ctx->pf_ctl.p;
    int32_t* list = (int32_t*)ctx->pf_list.p;
    k_prefetch_reset<<<1, 64, 0, s>>>(pctl);
    RG_LAUNCH_CHECK(ctx, "k_prefetch_reset");
    const bool mirror = cache->mirror_rows > 0;
    k_prefetch_select<<<(int)rg_div_up(n, 256), 256, 0, s>>>(input_nodes, n, n_dev, cache->loc, home, cache->filled, list, pctl, mirror ? 1 : 0);
    RG_LAUNCH_CHECK(ctx, "k_prefetch_select");
    return launch_list_copy(ctx, list, pctl, remote_store, remote_stride, cache->cache_rows, cache->row_stride,
                            mirror ? cache->mirror_rows : cache->capacity_rows, dim, n, ctx->knobs.pull_blocks, ctx->knobs.pull_threads, s);
}

rg_status rg_plan_prefetch(rg_ctx* ctx, const rg_cache* cache, const int32_t* home, const uint32_t* first_batch,
                           int64_t num_nodes, const rg_prefetch_plan* plan, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, cache && cache->num_cached && plan && plan->offsets, "rg_plan_prefetch: null cache / plan");
    RG_REQUIRE(ctx, cache->mirror_rows == 0, "rg_plan_prefetch: a mirrored cache is filled by rg_prefetch_cache_rows");
    RG_REQUIRE(ctx, plan->num_batches >= 0 && plan->num_batches <= 65535, "rg_plan_prefetch: num_batches not in [0, 65535]");
    RG_REQUIRE(ctx, num_nodes >= 0 && cache->capacity_rows >= 0, "rg_plan_prefetch: negative size");
    const int64_t rows_ub = rg_min64(cache->capacity_rows, num_nodes);
    RG_REQUIRE(ctx, rows_ub == 0 || (cache->cache_ids && home && first_batch && plan->list), "rg_plan_prefetch: null array");
    RG_REQUIRE(ctx, plan->list_capacity >= rows_ub, "rg_plan_prefetch: plan list holds %lld pairs, %lld required",
               (long long)plan->list_capacity, (long long)rows_ub);
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int n_seg = plan->num_batches + 1;
    rg_status st;
    if (n_seg <= 1024) {
        // ordered plan: stable counting sort by first batch
        const int nblocks = (int)rg_max64(1, rg_div_up(rows_ub, kPlanChunk));
        const int64_t n_hist = (int64_t)n_seg * nblocks;
        if ((st = rg_ensure(ctx, ctx->plan_cursor, (size_t)n_hist * 4)) != RG_OK) return st;
        int32_t* hist = (int32_t*)ctx->plan_cursor.p;
        if (rows_ub == 0) {
            k_zero_i32<<<(n_seg + 1 + 255) / 256, 256, 0, s>>>(plan->offsets, n_seg + 1);
            RG_LAUNCH_CHECK(ctx, "k_zero_i32");
            return RG_OK;
        }
        k_plan_block_hist<<<nblocks, 1024, 0, s>>>(cache->cache_ids, cache->num_cached, first_batch, plan->num_batches, nblocks, hist);
        RG_LAUNCH_CHECK(ctx, "k_plan_block_hist");
        k_plan_hist_scan<<<1, 1024, 0, s>>>(hist, n_hist, nblocks, n_seg, plan->offsets);
        RG_LAUNCH_CHECK(ctx, "k_plan_hist_scan");
        k_plan_block_scatter<<<nblocks, 1024, 0, s>>>(cache->cache_ids, cache->num_cached, first_batch, home, plan->num_batches,
                                                      nblocks, hist, plan->list);
        RG_LAUNCH_CHECK(ctx, "k_plan_block_scatter");
        return RG_OK;
    }
    // more than 1023 batches: unordered scatter with atomics (segments hold the right slots in arbitrary order)
    if ((st = rg_ensure(ctx, ctx->plan_cursor, (size_t)n_seg * 4)) != RG_OK) return st;
    int32_t* cursor = (int32_t*)ctx->plan_cursor.p;
    k_zero_i32<<<(n_seg + 1 + 255) / 256, 256, 0, s>>>(plan->offsets, n_seg + 1);
    RG_LAUNCH_CHECK(ctx, "k_zero_i32");
    const int grid = (int)rg_max64(1, rg_min64(rg_div_up(rows_ub, 256), (int64_t)ctx->num_cus * 8));
    if (rows_ub > 0) {
        k_plan_count<<<grid, 256, 0, s>>>(cache->cache_ids, cache->num_cached, first_batch, plan->num_batches, plan->offsets);
        RG_LAUNCH_CHECK(ctx, "k_plan_count");
    }
    k_plan_scan<<<1, 1024, 0, s>>>(plan->offsets, cursor, n_seg);
    RG_LAUNCH_CHECK(ctx, "k_plan_scan");
    if (rows_ub > 0) {
        k_plan_scatter<<<grid, 256, 0, s>>>(cache->cache_ids, cache->num_cached, first_batch, home, plan->num_batches, cursor, plan->list);
        RG_LAUNCH_CHECK(ctx, "k_plan_scatter");
    }
    return RG_OK;
}

rg_status rg_prefetch_planned(rg_ctx* ctx, const rg_prefetch_plan* plan, int32_t batch, const rg_cache* cache,
                              const float* remote_store, int64_t remote_stride, int32_t dim, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, plan && plan->offsets && plan->list, "rg_prefetch_planned: incomplete plan");
    RG_REQUIRE(ctx, batch >= 0 && batch <= plan->num_batches, "rg_prefetch_planned: batch = %d not in [0, %d]", batch, plan->num_batches);
    RG_REQUIRE(ctx, cache && cache->cache_rows && cache->filled && remote_store, "rg_prefetch_planned: null cache rows / filled / store");
    RG_REQUIRE(ctx, cache->mirror_rows >= 0 && cache->mirror_rows <= cache->capacity_rows, "rg_prefetch_planned: mirror_rows out of range");
    RG_REQUIRE(ctx, dim >= 1 && cache->row_stride >= dim && remote_stride >= dim, "rg_prefetch_planned: bad dim / stride");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    { const rg_status chk = rg_check_device_readable(ctx, remote_store, "rg_prefetch_planned: remote_store"); if (chk != RG_OK) return chk; }
    hipStream_t s = (hipStream_t)stream;
    const int64_t dst_rows = cache->mirror_rows > 0 ? cache->mirror_rows : cache->capacity_rows;
    rg_status st = launch_list_copy(ctx, plan->list, nullptr, remote_store, remote_stride, cache->cache_rows, cache->row_stride,
                                    dst_rows, dim, rg_max64(plan->list_capacity, 1), ctx->knobs.pull_blocks,
                                    ctx->knobs.pull_threads, s, plan->offsets + batch, cache->filled);   // marks the slots resident too
    return st;
}

rg_status rg_plan_sampled(rg_ctx* ctx, int32_t group, const rg_cache* cache, uint32_t* claimed, const rg_prefetch_plan* plan,
                          int32_t segment, int64_t num_nodes, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, group >= 1 && group <= RG_MAX_GROUP, "rg_plan_sampled: group = %d not in [1,%d]", group, RG_MAX_GROUP);
    RG_REQUIRE(ctx, cache && cache->mirror_rows > 0 && cache->home, "rg_plan_sampled: needs a mirrored cache with its home words");
    RG_REQUIRE(ctx, claimed && plan && plan->list && plan->offsets, "rg_plan_sampled: null claimed bitmap / plan");
    RG_REQUIRE(ctx, segment >= 0 && segment < plan->num_batches, "rg_plan_sampled: segment = %d not in [0, %d)", segment, plan->num_batches);
    RG_REQUIRE(ctx, plan->list_capacity >= cache->mirror_rows, "rg_plan_sampled: plan list holds %lld pairs, %lld required",
               (long long)plan->list_capacity, (long long)cache->mirror_rows);
    if (ctx->last_sample_group != group || ctx->last_sample_nodes != num_nodes)
        return rg_set_error(ctx, RG_ERR_STATE, "rg_plan_sampled: the last sampling call of this context covered %d batches on %lld "
                            "nodes, not %d on %lld", ctx->last_sample_group, (long long)ctx->last_sample_nodes, group, (long long)num_nodes);
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const int64_t words = rg_div_up(num_nodes, 32);
    const int nblocks = (int)rg_max64(1, rg_div_up(words, kClaimWordsPerBlock));
    rg_status st;
    if ((st = rg_ensure(ctx, ctx->claim_bits, (size_t)rg_max64(words, 1) * 4)) != RG_OK) return st;
    if ((st = rg_ensure(ctx, ctx->claim_blk, (size_t)nblocks * 4)) != RG_OK) return st;
    uint32_t* newbits = (uint32_t*)ctx->claim_bits.p;
    int32_t* blk = (int32_t*)ctx->claim_blk.p;
    k_claim_count<<<nblocks, 256, 0, s>>>((const uint32_t*)ctx->visited.p, words, group, claimed, newbits, cache->home, blk);
    RG_LAUNCH_CHECK(ctx, "k_claim_count");
    k_claim_scan<<<1, 1024, 0, s>>>(blk, nblocks, plan->offsets + segment, plan->list_capacity);
    RG_LAUNCH_CHECK(ctx, "k_claim_scan");
    k_claim_emit<<<nblocks, 256, 0, s>>>(newbits, words, cache->home, blk, plan->offsets + segment, plan->list);
    RG_LAUNCH_CHECK(ctx, "k_claim_emit");
    return RG_OK;
}

}  // extern "C"
