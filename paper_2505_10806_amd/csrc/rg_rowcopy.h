// Row-copy building blocks shared by the cache pulls, the gather and the mean aggregation.
//
// A feature row is moved as `cpr` chunks of VEC floats (VEC = 4 -> 16-byte accesses).  In the link kernels
// and the aggregation a wavefront is split into groups of L = 2^log2L lanes, one group per row, so 64/L rows
// move per wave step and short rows (256 B, 400 B, 512 B) still fill most lanes; U row groups are unrolled
// so every lane has U independent loads in flight before the first store.  (The HBM gather kernel splits
// the work by chunks instead of rows.)
#pragma once

#include "rg_internal.h"

template <int VEC> struct RgVec;
template <> struct RgVec<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct RgVec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct RgVec<1> { typedef float type; };

// Stores the first `count` floats of a chunk (a row's last chunk when dim is not a multiple of the chunk width).
template <typename V>
__device__ __forceinline__ void rg_store_head(V* dst, const V& val, int count) {
    float* d = (float*)dst;
    const float* v = (const float*)&val;
    for (int q = 0; q < count; ++q) d[q] = v[q];
}

struct RgRowShape {
    int cpr;      // chunks per row = ceil(dim / VEC)
    int log2L;    // lanes per row group = 1 << log2L (<= 64)
    int tail;     // floats of the row's last chunk that belong to the row (1..VEC); only those are stored
};

static inline int rg_pick_vec(int32_t dim, const void* const* ptrs, int nptrs, const int64_t* strides, int nstrides) {
    int vec = 4;
    for (int i = 0; i < nptrs; ++i) {
        const uintptr_t a = (uintptr_t)ptrs[i];
        if (!a) continue;
        while (vec > 1 && (a % (vec * 4)) != 0) vec >>= 1;
    }
    for (int i = 0; i < nstrides; ++i)
        while (vec > 1 && (strides[i] % vec) != 0) vec >>= 1;
    // A 16-byte chunk may read the padding behind a source row (stride >= round_up(dim, 4) is implied by
    // stride % 4 == 0 and stride >= dim); stores are trimmed to dim.  Narrower chunks tile dim exactly.
    if (vec == 2 && (dim % 2) != 0) vec = 1;
    return vec;
}

static inline RgRowShape rg_row_shape(int32_t dim, int vec) {
    RgRowShape s;
    s.cpr = (dim + vec - 1) / vec;
    int l = 0;
    while ((1 << l) < s.cpr && l < 6) ++l;
    s.log2L = l;
    s.tail = dim - (s.cpr - 1) * vec;
    return s;
}

// Kernels that read rows over the host link (cache pulls, miss rows) wait on the link, not on the GPU.  A compute unit
// that hosts their wavefronts is all but lost to the HBM kernels running beside them: loads that stay outstanding for
// microseconds fill the unit's vector-memory queues, so a gather workgroup placed there crawls.  What matters is
// therefore the number of compute units the link kernels touch, not their number of wavefronts: few, large workgroups.
// Measured on the stress workload (pull grid -> link rate, HBM gather beside it as a fraction of peak, whole epoch):
//   48 x 256 threads   53.0 GB/s   0.616   1354 batches/s
//   16 x 1024          55.8 GB/s   0.656   1407 batches/s      (default)
//    8 x 1024          47.3 GB/s   0.677   1292 batches/s      (too few loads in flight for the link)
//    8 x 1024, 8 rows in flight per lane group   51.1 GB/s   0.675   1338 batches/s
// against 56.9 GB/s for the pull kernel alone, 57.3 GB/s for a plain runtime copy from pinned memory and 0.69 for
// the gather alone.  Miss rows go through one more dependent lookup per step than the pulls and need more wavefronts
// to fill the link (swept on the 602-dim workload: 48 workgroups of 256 threads 46 GB/s, 192 -> 51, 384 -> 53).
// The grids are RgKnobs::pull_blocks x pull_threads and RgKnobs::miss_blocks x miss_threads.
