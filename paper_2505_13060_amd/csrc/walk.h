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
//   template <int U> void full_masked(int64_t e, int stride, int count, int tail)
//       `count` (0..U) whole, 16-byte aligned vectors starting at x[e + k*stride], k < count, of
//       which the last one contributes only its first `tail` (1..8) elements: the rest of that
//       vector lies inside the unit's memory but does not belong to the operand and must not
//       influence the result; e differs from lane to lane
//   void partial(int64_t e, int jlo, int jhi)
//       elements x[e + j], jlo <= j < jhi, to be fetched one by one
//   void begin_dense(int64_t e0, int le)
//       a dense chunk starts: the vectors this thread is about to be given (by full and partial,
//       one after the other) start at elements e0 + le, e0 + le + kWG*kVec, e0 + le + 2*kWG*kVec, ...
//       A context that needs the row of every vector follows them with a RowCursor.
//   static constexpr bool kRollDense
//       true: the walk over a whole dense chunk stays a loop instead of being unrolled
//   void set_row(int64_t row)
//       causal chunks: the vectors that follow, until the next call, lie in row `row` of the unit
//       (matrix index * rows + row index)
// Element indices are relative to the unit's first element.
#pragma once

#include "internal.h"

namespace ampsens {

#if defined(__HIP_DEVICE_COMPILE__)
#define AMPSENS_HD __host__ __device__ __forceinline__
#else
#define AMPSENS_HD __host__ __device__ inline
#endif

// Row of a lane's vector when only the wave's first lane is tracked (cursor `cur` of that lane):
// the 64 lanes cover 512 contiguous elements.  Rows of at least 512 elements: the step meets row
// cur.row and, from the lane on that passes the row's end, the next row.  Shorter rows whose length
// is a power of two (sub_shift = log2(row_len / 8)): the step covers whole rows.
AMPSENS_HD int wave_sub_shift(int32_t row_len) {
    if (row_len >= 64 * kVec) return -1;
    int s = 0;
    while ((kVec << (s + 1)) <= row_len) ++s;
    return s;
}
constexpr int kUnroll = 4;           // independent 128-bit loads per stream in flight per lane

// Row of every vector of a thread's strided walk over a [rows, row_len] array, without a
// division per vector: one division where the walk starts, then additions.  row_len == 0 means
// the array is one row.  Vectors must not straddle rows (row_len a multiple of kVec, walk
// starting on a vector boundary of the array).
struct RowCursor {
    int32_t row, col, drow, dcol, len;
    // The walk starts at element e0 + le (e0 common to the workgroup, 0 <= le < 2^16) and moves
    // `stride` (< 2^30) elements per step.
    AMPSENS_HD void begin(int64_t e0, int le, int32_t stride, int32_t row_len) {
        len = row_len;
        if (row_len <= 0) { row = col = drow = dcol = 0; return; }
        const int64_t r0 = e0 / row_len;
        const uint32_t off = (uint32_t)(e0 - r0 * row_len) + (uint32_t)le;   // < 2^30 + 2^16
        const uint32_t q = off / (uint32_t)row_len;
        row = (int32_t)r0 + (int32_t)q;
        col = (int32_t)(off - q * (uint32_t)row_len);
        drow = stride / row_len;
        dcol = stride % row_len;
    }
    AMPSENS_HD void advance() {
        col += dcol;
        row += drow;
        if (col >= len && len > 0) { col -= len; ++row; }
    }
};

// True when every vector of dense chunk `chunk_local` is whole and aligned.
AMPSENS_HD bool dense_chunk_interior(int64_t n, uint32_t head, bool scalar, uint32_t chunk_local) {
    const int64_t v0 = (int64_t)chunk_local * kChunkVecs;
    return !scalar && (v0 * kVec >= (int64_t)head) && ((v0 + kChunkVecs) * kVec - head <= n);
}

AMPSENS_HD int32_t wave_lane_row(const RowCursor& cur, int32_t last_row, int sub_shift, int lane) {
    if (sub_shift >= 0) return cur.row + (lane >> sub_shift);
    if (lane * kVec < cur.len - cur.col) return cur.row;
    return cur.row < last_row ? cur.row + 1 : last_row;
}

template <class Ctx>
AMPSENS_HD void walk_dense_chunk(int64_t n, uint32_t head, bool scalar, uint32_t chunk_local,
                                 int tid, Ctx& ctx) {
    const int64_t nvec = (n + head + (kVec - 1)) / kVec;
    const int64_t v0 = (int64_t)chunk_local * kChunkVecs;
    int64_t v1 = v0 + kChunkVecs;
    ctx.begin_dense(v0 * kVec - head, tid * kVec);
    if (dense_chunk_interior(n, head, scalar, chunk_local)) {
        const int64_t eu = v0 * kVec - head;
        if constexpr (Ctx::kRollDense) {               // the context's code per group is large: keep one copy
#pragma unroll 1
            for (int k = 0; k < kChunkVecs / kWG; k += kUnroll)
                ctx.template full<kUnroll>(eu + (int64_t)k * kWG * kVec, tid * kVec, (int64_t)kWG * kVec);
        } else {
#pragma unroll
            for (int k = 0; k < kChunkVecs / kWG; k += kUnroll)
                ctx.template full<kUnroll>(eu + (int64_t)k * kWG * kVec, tid * kVec, (int64_t)kWG * kVec);
        }
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

// Causal chunks.  A band is 8 consecutive rows of one matrix.  Band j of a lower-triangular
// matrix holds about (j + 1) vectors per row, so bands are paired, j with nbands - 1 - j, into
// slots of equal work; a chunk is kBandsPerChunk consecutive slots (one per wave on the aligned
// path).  Slot s < nbands / 2 has two bands, the middle band of an odd count stands alone.
AMPSENS_HD int32_t causal_bands(int32_t rows) { return (rows + kBandRows - 1) / kBandRows; }

// The bands of slot `slot`: returns how many (0, 1 or 2) and writes them to band[].
AMPSENS_HD int causal_slot_bands(int32_t nbands, int32_t slot, int32_t band[2]) {
    const int32_t mirror = nbands - 1 - slot;
    if (slot > mirror) return 0;
    band[0] = slot;
    if (slot == mirror) return 1;
    band[1] = mirror;
    return 2;
}

// Generic causal walk (any alignment): all threads stride over the vectors of each band.
template <class Ctx>
AMPSENS_HD void walk_causal_chunk(int32_t rows, int32_t cols, bool scalar, uint32_t chunks_per_mat,
                                  uint32_t chunk_local, int tid, Ctx& ctx) {
    const uint32_t mat = chunk_local / chunks_per_mat;
    const int32_t slot0 = (int32_t)(chunk_local % chunks_per_mat) * kBandsPerChunk;
    const int64_t mat_base = (int64_t)mat * rows * cols;
    const int32_t nbands = causal_bands(rows);
    for (int s = 0; s < kBandsPerChunk; ++s) {
        int32_t bands[2];
        const int nb = causal_slot_bands(nbands, slot0 + s, bands);
        for (int b = 0; b < nb; ++b) {
            const int32_t i0 = bands[b] * kBandRows;
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
                ctx.set_row((int64_t)mat * rows + i);
                if (!scalar && jhi == kVec) ctx.template full<1>(e, 0, 0);
                else ctx.partial(e, 0, jhi);
            }
        }
    }
}

// Causal chunk whose rows start on 16-byte boundaries (aligned base, cols a multiple of 8):
// wave w of the workgroup owns slot w of the chunk, i.e. one band from the top of the triangle
// and its mirror from the bottom; its 64 lanes cover 8 rows x 8 vectors (128 contiguous bytes
// of each row) per step and run along the rows; the vector that holds a row's end is loaded
// whole and masked.
template <class Ctx>
AMPSENS_HD void walk_causal_chunk_aligned(int32_t rows, int32_t cols, uint32_t chunks_per_mat,
                                          uint32_t chunk_local, int tid, Ctx& ctx) {
    static_assert(kBandsPerChunk == kWaves, "one wave per slot");
    static_assert(kBandRows * (64 / kBandRows) == 64 && ((64 / kBandRows) & (64 / kBandRows - 1)) == 0, "lanes = rows x vectors");
    const uint32_t mat = chunk_local / chunks_per_mat;
    const int32_t slot = (int32_t)(chunk_local % chunks_per_mat) * kBandsPerChunk + (tid >> 6);
    const int32_t nbands = causal_bands(rows);
    int32_t bands[2];
    const int nb = causal_slot_bands(nbands, slot, bands);
    const int lane = tid & 63;
    constexpr int kStep = 64 / kBandRows;                       // vectors of a row per wave step
    for (int b = 0; b < nb; ++b) {
        const int32_t i0 = bands[b] * kBandRows;
        const int32_t i = i0 + (lane / kStep);                  // 8 adjacent lanes own 128 contiguous bytes of a row
        const int32_t ilast = (i0 + kBandRows - 1 < rows) ? i0 + kBandRows - 1 : rows - 1;
        const int32_t nv_band = (causal_row_len(ilast, rows, cols) + kVec - 1) / kVec;   // same for the wave
        const int32_t li = i < rows ? causal_row_len(i, rows, cols) : 0;
        const int32_t nv_row = (li + kVec - 1) / kVec;
        const int tail = li - (nv_row - 1) * kVec;              // 1..8 when the row has elements
        const int64_t e_row = ((int64_t)mat * rows + (i < rows ? i : 0)) * cols;
        ctx.set_row((int64_t)mat * rows + (i < rows ? i : 0));
        for (int32_t v0 = 0; v0 < nv_band; v0 += kStep * kUnroll) {
            const int32_t v = v0 + (lane & (kStep - 1));
            int count = nv_row > v ? (nv_row - v + kStep - 1) / kStep : 0;
            if (count > kUnroll) count = kUnroll;
            const bool ends = count > 0 && v + (count - 1) * kStep == nv_row - 1;
            ctx.template full_masked<kUnroll>(e_row + (int64_t)v * kVec, kStep * kVec, count,
                                              ends ? tail : kVec);
        }
    }
}

template <class Unit, class Ctx>
AMPSENS_HD void walk_chunk(const Unit& u, uint32_t chunk_local, int tid, Ctx& ctx) {
    const bool scalar = (u.flags & kUnitScalar) != 0;
    if ((u.flags & kUnitCausal) && !scalar)
        walk_causal_chunk_aligned(u.rows, u.cols, u.chunks_per_mat, chunk_local, tid, ctx);
    else if (u.flags & kUnitCausal)
        walk_causal_chunk(u.rows, u.cols, scalar, u.chunks_per_mat, chunk_local, tid, ctx);
    else
        walk_dense_chunk(u.n, u.head, scalar, chunk_local, tid, ctx);
}

// Schedule position of chunk `local` of a unit with `chunks` chunks, both counted after the
// chunks the unit leaves to the weight kernel (see UnitSchedule).
AMPSENS_HD uint32_t schedule_position(const UnitSchedule& sch, uint32_t local, uint32_t chunks) {
    const uint32_t b = local / sch.block;
    const uint32_t left = chunks - b * sch.block;
    const uint32_t w = left < sch.block ? left : sch.block;
    return sch.begin + b * sch.block * sch.interleave + sch.member * w + local % sch.block;
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
