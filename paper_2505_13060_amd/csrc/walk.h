// Chunk walkers: which elements of a unit a given thread of a workgroup touches for a
// given chunk.  Written once, as host+device templates over a context object, so that the
// device kernels and a host-side replay (used by the CPU tests to prove that every element
// is visited exactly once and that no access leaves the unit) run the very same index code.
//
// A context provides
//   template <int U> void full(int64_t eu, int le, int64_t stride)
//       U whole 8-element vectors whose first elements are x[eu + le + k*stride], k < U; eu and
//       stride are the same for every thread of the workgroup, le is the thread's own offset;
//       each vector is 16-byte aligned in memory
//   void partial(int64_t e, int jlo, int jhi)
//       elements x[e + j], jlo <= j < jhi, to be fetched one by one
// Element indices are relative to the unit's first element.
#pragma once

#include "internal.h"

namespace ampsens {

#if defined(__HIP_DEVICE_COMPILE__)
#define AMPSENS_HD __host__ __device__ __forceinline__
#else
#define AMPSENS_HD __host__ __device__ inline
#endif

constexpr int kUnroll = 4;           // independent 128-bit loads per stream in flight per lane

// True when every vector of dense chunk `chunk_local` is whole and aligned.
AMPSENS_HD bool dense_chunk_interior(int64_t n, uint32_t head, bool scalar, uint32_t chunk_local) {
    const int64_t v0 = (int64_t)chunk_local * kChunkVecs;
    return !scalar && (v0 * kVec >= (int64_t)head) && ((v0 + kChunkVecs) * kVec - head <= n);
}

template <class Ctx>
AMPSENS_HD void walk_dense_chunk(int64_t n, uint32_t head, bool scalar, uint32_t chunk_local,
                                 int tid, Ctx& ctx) {
    const int64_t nvec = (n + head + (kVec - 1)) / kVec;
    const int64_t v0 = (int64_t)chunk_local * kChunkVecs;
    int64_t v1 = v0 + kChunkVecs;
    if (dense_chunk_interior(n, head, scalar, chunk_local)) {
        const int64_t eu = v0 * kVec - head;
#pragma unroll
        for (int k = 0; k < kChunkVecs / kWG; k += kUnroll)
            ctx.template full<kUnroll>(eu + (int64_t)k * kWG * kVec, tid * kVec, (int64_t)kWG * kVec);
        return;
    }
    if (v1 > nvec) v1 = nvec;
    for (int64_t v = v0 + tid; v < v1; v += kWG) {
        const int64_t e = v * kVec - head;
        const int jlo = e < 0 ? (int)(-e) : 0;
        const int64_t rem = n - e;
        const int jhi = rem < kVec ? (int)rem : kVec;
        if (!scalar && jlo == 0 && jhi == kVec) ctx.template full<1>(e, 0, 0);
        else ctx.partial(e, jlo, jhi);
    }
}

AMPSENS_HD int32_t causal_row_len(int32_t i, int32_t rows, int32_t cols) {
    int64_t len = (int64_t)i + 1 + ((int64_t)cols - rows);
    if (len < 0) len = 0;
    if (len > cols) len = cols;
    return (int32_t)len;
}

template <class Ctx>
AMPSENS_HD void walk_causal_chunk(int32_t rows, int32_t cols, bool scalar, uint32_t chunks_per_mat,
                                  uint32_t chunk_local, int tid, Ctx& ctx) {
    const uint32_t mat = chunk_local / chunks_per_mat;
    const int32_t band0 = (int32_t)(chunk_local % chunks_per_mat) * kBandsPerChunk;
    const int64_t mat_base = (int64_t)mat * rows * cols;
    const int32_t nbands = (rows + kBandRows - 1) / kBandRows;
    for (int b = 0; b < kBandsPerChunk; ++b) {
        const int32_t band = band0 + b;
        if (band >= nbands) break;
        const int32_t i0 = band * kBandRows;
        const int32_t ilast = (i0 + kBandRows - 1 < rows) ? i0 + kBandRows - 1 : rows - 1;
        const int32_t lmax = causal_row_len(ilast, rows, cols);
        const int32_t items = ((lmax + kVec - 1) / kVec) * kBandRows;
        for (int32_t k = tid; k < items; k += kWG) {
            const int32_t i = i0 + (k & (kBandRows - 1));
            const int32_t e0 = (k / kBandRows) * kVec;
            if (i >= rows) continue;
            const int32_t li = causal_row_len(i, rows, cols);
            if (e0 >= li) continue;
            const int jhi = (li - e0 < kVec) ? (li - e0) : kVec;
            const int64_t e = mat_base + (int64_t)i * cols + e0;
            if (!scalar && jhi == kVec) ctx.template full<1>(e, 0, 0);
            else ctx.partial(e, 0, jhi);
        }
    }
}

template <class Unit, class Ctx>
AMPSENS_HD void walk_chunk(const Unit& u, uint32_t chunk_local, int tid, Ctx& ctx) {
    const bool scalar = (u.flags & kUnitScalar) != 0;
    if (u.flags & kUnitCausal)
        walk_causal_chunk(u.rows, u.cols, scalar, u.chunks_per_mat, chunk_local, tid, ctx);
    else
        walk_dense_chunk(u.n, u.head, scalar, chunk_local, tid, ctx);
}

// Largest u with chunk_begin[u] <= c (chunk_begin has n_units + 1 entries, the last being the
// total; units without chunks are skipped because a later unit shares their begin).
AMPSENS_HD uint32_t find_unit(const uint32_t* chunk_begin, uint32_t n_units, uint32_t c) {
    uint32_t lo = 0, hi = n_units;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (chunk_begin[mid] <= c) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace ampsens
