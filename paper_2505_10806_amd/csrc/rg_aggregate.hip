// Consumer of the gathered features: mean aggregation over a sampled block (Eq. 1 with AGG = mean, the
// GraphSAGE aggregator of Section II-A).  Bandwidth-bound: every sampled edge reads one feature row.
#include "rg_rowcopy.h"

namespace {

// agg[i] = (1/m_i) * sum over the block's edges e of row i, in edge order, of feat[nbr_local[e]].
// A wavefront is split into groups of L lanes per destination row; each lane owns chunk c0 (+ L, + 2L, ...) of the
// row and accumulates it in registers, E edges at a time so that E independent row loads are in flight.
template <int VEC, int E>
__global__ void __launch_bounds__(256) k_mean_aggregate(const int32_t* __restrict__ indptr, const int32_t* __restrict__ nbr_local,
                                                        int64_t n_dst, const int32_t* __restrict__ n_dst_dev,
                                                        const float* __restrict__ feat, int64_t feat_stride,
                                                        float* __restrict__ agg, int64_t agg_stride, int cpr, int log2L, int tail) {
    typedef typename RgVec<VEC>::type V;
    int64_t n_act = n_dst;
    if (n_dst_dev) { const int64_t d = *n_dst_dev; n_act = d < n_dst ? d : n_dst; }
    const int lane = rg_lane();
    const int L = 1 << log2L;
    const int R = RG_WAVE >> log2L;
    const int sub = lane >> log2L;
    const int c0 = lane & (L - 1);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t row0 = wave * R; row0 < n_act; row0 += nwaves * R) {
        const int64_t i = row0 + sub;
        if (i >= n_act) continue;
        const int e0 = indptr[i], e1 = indptr[i + 1];
        const float m = (float)(e1 - e0);
        V* dst = (V*)(agg + i * agg_stride);
        for (int c = c0; c < cpr; c += L) {
            V acc;
#pragma unroll
            for (int q = 0; q < VEC; ++q) ((float*)&acc)[q] = 0.0f;
            for (int e = e0; e < e1; e += E) {
                V val[E];
#pragma unroll
                for (int u = 0; u < E; ++u)
                    if (e + u < e1) val[u] = ((const V*)(feat + (int64_t)nbr_local[e + u] * feat_stride))[c];
#pragma unroll
                for (int u = 0; u < E; ++u)
                    if (e + u < e1) {
#pragma unroll
                        for (int q = 0; q < VEC; ++q) ((float*)&acc)[q] += ((const float*)&val[u])[q];
                    }
            }
            if (e1 > e0) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) ((float*)&acc)[q] = ((float*)&acc)[q] / m;
            }
            // a 16-byte chunk may reach into the sources' row padding: only the row's own floats are stored
            if (tail < VEC && c == cpr - 1) rg_store_head(&dst[c], acc, tail);
            else __builtin_nontemporal_store(acc, &dst[c]);
        }
    }
}

}  // namespace

extern "C" {

rg_status rg_mean_aggregate(rg_ctx* ctx, const int32_t* indptr, const int32_t* nbr_local, int64_t n_dst,
                            const int32_t* n_dst_dev, const float* feat, int64_t feat_stride, int32_t dim,
                            float* agg, int64_t agg_stride, void* stream) {
    if (!ctx) return RG_ERR_INVALID_ARG;
    RG_REQUIRE(ctx, n_dst >= 0 && n_dst <= (1ll << 31) - 1, "rg_mean_aggregate: n_dst = %lld out of range", (long long)n_dst);
    RG_REQUIRE(ctx, dim >= 1 && feat_stride >= dim && agg_stride >= dim, "rg_mean_aggregate: bad dim / stride");
    if (n_dst == 0) return RG_OK;
    RG_REQUIRE(ctx, indptr && nbr_local && feat && agg, "rg_mean_aggregate: null pointer");
    RG_HIP(ctx, hipSetDevice(ctx->device));
    hipStream_t s = (hipStream_t)stream;
    const void* ptrs[2] = {feat, agg};
    const int64_t strides[2] = {feat_stride, agg_stride};
    const int vec = rg_pick_vec(dim, ptrs, 2, strides, 2);
    const RgRowShape shp = rg_row_shape(dim, vec);
    const int rows_per_block = 4 * (RG_WAVE >> shp.log2L);
    const int grid = (int)rg_max64(1, rg_min64(rg_div_up(n_dst, rows_per_block), (int64_t)ctx->num_cus * 64));
    const int tok = rg_prof_begin(ctx, RG_K_AGGREGATE, s);
    if (vec == 4)
        k_mean_aggregate<4, 4><<<grid, 256, 0, s>>>(indptr, nbr_local, n_dst, n_dst_dev, feat, feat_stride, agg, agg_stride, shp.cpr, shp.log2L, shp.tail);
    else if (vec == 2)
        k_mean_aggregate<2, 4><<<grid, 256, 0, s>>>(indptr, nbr_local, n_dst, n_dst_dev, feat, feat_stride, agg, agg_stride, shp.cpr, shp.log2L, shp.tail);
    else
        k_mean_aggregate<1, 4><<<grid, 256, 0, s>>>(indptr, nbr_local, n_dst, n_dst_dev, feat, feat_stride, agg, agg_stride, shp.cpr, shp.log2L, shp.tail);
    rg_prof_end(ctx, tok, s);
    RG_LAUNCH_CHECK(ctx, "k_mean_aggregate");
    return RG_OK;
}

}  // extern "C"
