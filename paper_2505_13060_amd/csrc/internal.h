// Internal declarations shared by the C-ABI layer and the HIP kernels of libampsens.
// Not installed; the public interface is include/ampsens.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ampsens {

// ---- work decomposition ------------------------------------------------------------------
// Every operand block of one calibration sample is a "unit".  A unit is cut into chunks by a
// rule that depends only on the unit (never on the grid), and chunk c of a launch writes its
// partial sums into slot c, so results are independent of how many workgroups run.
//
// Dense unit: its elements are viewed as 8-element vectors on the 16-byte grid of the x
// pointer (the first and last vector may be partial); a chunk is kChunkVecs vectors.
// Causal unit [batch, rows, cols]: a band is 8 consecutive rows of one batch entry; band j is
// paired with band nbands-1-j into a slot, so that every slot of a triangle carries the same
// work; a chunk is kBandsPerChunk slots.
constexpr int kWG = 256;             // threads per workgroup (4 wave64)
constexpr int kVec = 8;              // bf16 elements per 128-bit load
constexpr int kChunkVecs = 4096;     // dense: vectors per chunk (128 KiB of x + xdot)
constexpr int kBandRows = 8;
constexpr int kBandsPerChunk = 4;
constexpr int kMaxFormats = 2;
constexpr int kWaves = kWG / 64;     // every wave writes its own partial, so no barrier is needed

enum : uint32_t {
    kUnitCausal = 1u,                // causal layout
    kUnitScalar = 2u,                // x and xdot are not mutually 16-byte aligned (or causal rows
                                     // are not): every vector takes the guarded 2-byte path
    kUnitKeepX = 4u,                 // x is read again soon (a weight shared by the samples): load it
                                     // with ordinary caching; everything else streams non-temporally
    kUnitRowScale = 8u,              // one scale per row: scale / inv point at [rows][n_fmts] tables whose
                                     // first row is the unit's first row; dense units keep the row
                                     // length in `cols` and their number of rows in `rows`, causal
                                     // units use their own rows and cols
    kUnitFused = 16u,                // with kUnitRowScale: the pass itself computes the row scales (each row
                                     // is read once, kept in registers, reduced, scaled) and writes them to
                                     // the tables; `head` holds the FusedGeom of the unit
};

// Single-read pass over an operand with one scale per row.  A workgroup handles a tile of rows at
// a time: `lanes` (a power of two, 4..256) threads per row, 256 / lanes rows per tile, each thread
// owning up to kFusedNv 8-element vectors of its row (more only for rows beyond 256 * kFusedNv
// vectors).  A thread stages its vectors of x in LDS while the row's absmax is found, then streams the
// row's gradient against them: HBM delivers every byte once.  Dense units: every tile has the lanes
// the row length asks for.  Causal units: row i owns i + 1 + (cols - rows) entries, so the lanes
// follow the row: the rows of a matrix fall into classes (lanes = 4, 8, ..., 256) by length, tiles are
// consecutive rows of one class, and a tile's work is about the same whatever its class.  A chunk is
// `tiles` consecutive tiles of a unit (dense) or of a matrix (causal).
#ifndef AMPSENS_FUSED_GROUP
#define AMPSENS_FUSED_GROUP 4
#endif
constexpr int kFusedRegNv = 4;                     // rows that leave a thread at most this many vectors stay in registers
constexpr int kFusedNv = kFusedRegNv;              // vectors of a row per thread the geometry aims at
constexpr int kFusedGroup = AMPSENS_FUSED_GROUP;   // LDS path: vectors per thread handled (and in flight) together
constexpr int kFusedMaxNv = 12;                    // LDS: 256 threads x 16 bytes x nv <= 48 KiB per workgroup
constexpr int64_t kFusedMaxRowLen = (int64_t)kWG * kFusedMaxNv * kVec;     // 24576 elements
constexpr int64_t kFusedChunkVecs = 8192;          // vectors per chunk the geometry aims at
static_assert(kFusedNv % kFusedGroup == 0 && kFusedMaxNv % kFusedGroup == 0, "whole groups");

// lanes (as log2) for a row of row_vecs vectors
inline __host__ __device__ int fused_lanes_log2(int64_t row_vecs) {
    int lg = 2;
    while (lg < 8 && ((int64_t)kFusedNv << lg) < row_vecs) ++lg;
    return lg;
}
// causal [rows, cols] matrix: rows whose valid length is at most `cap` elements
inline __host__ __device__ int64_t fused_causal_rows_upto(int64_t rows, int64_t cols, int64_t cap) {
    // row i owns clamp(i + 1 + cols - rows, 0, cols) entries
    if (cap >= cols) return rows;
    int64_t n = cap - (cols - rows);             // i + 1 + off <= cap  <=>  i < cap - off
    return n < 0 ? 0 : (n > rows ? rows : n);
}
// Tile q of a causal matrix: its lanes, first row and number of rows.  Returns false past the last tile.
struct FusedCausalTile { int lanes_log2; int64_t row0; int32_t n_rows; };
inline __host__ __device__ bool fused_causal_tile(int64_t rows, int64_t cols, int64_t q, FusedCausalTile* out) {
    int64_t a = 0;
    for (int lg = 2; lg <= 8; ++lg) {
        const int64_t b = lg == 8 ? rows : fused_causal_rows_upto(rows, cols, (int64_t)kVec * ((int64_t)kFusedNv << lg));
        const int64_t rt = kWG >> lg;
        const int64_t cnt = (b - a + rt - 1) / rt;
        if (q < cnt) {
            out->lanes_log2 = lg;
            out->row0 = a + q * rt;
            out->n_rows = (int32_t)(b - out->row0 < rt ? b - out->row0 : rt);
            return true;
        }
        q -= cnt;
        a = b;
    }
    return false;
}
inline __host__ __device__ int64_t fused_causal_tiles(int64_t rows, int64_t cols) {
    int64_t a = 0, total = 0;
    for (int lg = 2; lg <= 8; ++lg) {
        const int64_t b = lg == 8 ? rows : fused_causal_rows_upto(rows, cols, (int64_t)kVec * ((int64_t)kFusedNv << lg));
        const int64_t rt = kWG >> lg;
        total += (b - a + rt - 1) / rt;
        a = b;
    }
    return total;
}

struct FusedGeom {
    int lanes_log2, nv, tiles;                     // dense: lanes and vectors per thread; tiles per chunk
    bool wide;                                     // short dense rows of 2^lanes_log2 vectors: a tile is kFusedRegNv * 256
                                                   // consecutive vectors, one lane per vector (see wide_tile)
    __host__ __device__ uint32_t pack() const {
        return (uint32_t)lanes_log2 | ((uint32_t)tiles << 4) | ((uint32_t)nv << 12) | (wide ? 0x80000000u : 0u);
    }
    static __host__ __device__ FusedGeom unpack(uint32_t h) {
        FusedGeom g;
        g.lanes_log2 = (int)(h & 0xFu);
        g.tiles = (int)((h >> 4) & 0xFFu);
        g.nv = (int)((h >> 12) & 0xFFFFu);
        g.wide = (h & 0x80000000u) != 0;
        return g;
    }
    __host__ __device__ int rows_per_tile() const { return (wide ? kFusedRegNv * kWG : kWG) >> lanes_log2; }
};
// Geometry for rows of row_len elements (a multiple of 8): about kFusedNv vectors per thread, about
// 4096 vectors per chunk.  nv is rounded up to whole groups (what lies past a row's end is masked).
inline FusedGeom fused_geometry(int64_t row_len, bool causal) {
    const int64_t row_vecs = row_len / kVec;
    FusedGeom g;
    g.wide = false;
    // (rows of 32 vectors were measured too: 5.07 TB/s this way, 5.38 with eight threads per row)
    if (!causal && row_vecs >= 4 && row_vecs <= 16 && (row_vecs & (row_vecs - 1)) == 0) {
        g.wide = true;
        g.lanes_log2 = 2;
        while (((int64_t)1 << g.lanes_log2) < row_vecs) ++g.lanes_log2;
        g.nv = kFusedRegNv;
        g.tiles = (int)(kFusedChunkVecs / (kFusedRegNv * kWG));
        return g;
    }
    g.lanes_log2 = fused_lanes_log2(row_vecs);
    auto nv_of = [&](int lg) {
        const int64_t lanes = (int64_t)1 << lg;
        int64_t nv = (row_vecs + lanes - 1) / lanes;
        nv = (nv + kFusedGroup - 1) / kFusedGroup * kFusedGroup;
        return nv < kFusedGroup ? (int64_t)kFusedGroup : nv;
    };
    if (!causal && nv_of(g.lanes_log2) > kFusedRegNv) {
        // dense rows too long for the register path: the lanes that waste the fewest vector slots (a
        // thread's vectors come in whole groups), among those that leave at most kFusedMaxNv vectors per
        // thread; ties go to more lanes (less LDS per workgroup)
        int best = -1;
        int64_t best_slots = 0;
        for (int lg = 2; lg <= 8; ++lg) {
            const int64_t nv = nv_of(lg);
            if (nv > kFusedMaxNv) continue;
            const int64_t slots = nv << lg;
            if (best < 0 || slots <= best_slots) { best = lg; best_slots = slots; }
        }
        if (best >= 0) g.lanes_log2 = best;
    }
    g.nv = (int)nv_of(g.lanes_log2);
    // vectors per tile: dense rows_per_tile whole rows; causal about three quarters of 256 x kFusedNv
    const int64_t per = causal ? (int64_t)kWG * kFusedNv * 3 / 4 : (int64_t)g.rows_per_tile() * row_vecs;
    int64_t t = per > 0 ? (kFusedChunkVecs + per / 2) / per : 1;
    g.tiles = (int)(t < 1 ? 1 : (t > 64 ? 64 : t));
    return g;
}
inline uint64_t fused_chunks_dense(int64_t rows, const FusedGeom& g) {
    const uint64_t per = (uint64_t)g.rows_per_tile() * (uint64_t)g.tiles;
    return rows > 0 ? ((uint64_t)rows + per - 1) / per : 0;
}
inline uint32_t fused_chunks_per_mat(int64_t rows, int64_t cols, const FusedGeom& g) {
    const uint64_t tiles = (uint64_t)fused_causal_tiles(rows, cols);
    return (uint32_t)((tiles + g.tiles - 1) / g.tiles);
}
// LDS bytes a workgroup needs for a unit: its threads' vectors of x
inline size_t fused_lds_bytes(int nv) { return (size_t)kWG * 16 * (size_t)nv; }

struct alignas(16) WorkUnit {        // 64 bytes
    const uint16_t* x;               // first element of the block
    const uint16_t* dx;              // gradient block (sens) / unused (absmax)
    const float* scale;              // device [n_fmts] (sens) / unused
    const float* inv;                // device [n_fmts] (sens) / unused
    int64_t n;                       // dense: elements; causal: batch (number of matrices)
    int32_t rows, cols;              // causal
    uint32_t flags;
    uint32_t head;                   // dense: elements between the 16-byte grid and x (0..7)
    uint32_t out;                    // sens: float offset of this unit's (E, A) pair for format 0
                                     // absmax: tensor index
    uint32_t chunks_per_mat;         // causal: chunks per [rows, cols] matrix
};
static_assert(sizeof(WorkUnit) == 64, "WorkUnit layout");

// Device-side companions of the table, written by the prepare kernel of each call:
// the unit with its scales resolved to values, and for every chunk its unit and its index
// inside that unit, so that the streaming kernels need no search.
struct alignas(16) ResolvedUnit {    // 64 bytes
    const uint16_t* x;
    const uint16_t* dx;
    int64_t n;
    int32_t rows, cols;
    uint32_t flags;
    uint32_t head;
    uint32_t out;
    uint32_t chunks_per_mat;
    union {
        struct {                     // one scale per tensor: the values
            float inv[kMaxFormats];
            float scale[kMaxFormats];
        };
        struct {                     // kUnitRowScale: [rows][n_fmts] tables, first row = the unit's first
            const float* row_inv;
            const float* row_scale;
        };
    };
};
static_assert(sizeof(ResolvedUnit) == 64, "ResolvedUnit layout");

// Entry p of the map is the chunk processed at schedule position p.  The schedule is a
// permutation chosen on the host (see UnitSchedule); `slot` is the chunk's canonical number
// (chunk_begin[unit] + local): partial results are stored by slot, so the schedule never changes a
// result.
struct ChunkRef {
    uint32_t unit;
    uint32_t local;                  // chunk index inside the unit
    uint32_t slot;
    uint32_t reserved;
};

// Where the chunks of a unit sit in the schedule.  Units that read the same x with different
// gradients (a weight and the R per-sample weight gradients) form a group of `interleave`
// members with equal chunk counts; their chunks are laid out block by block (8 chunks), member
// after member inside a block of `block` chunks:
//     position = begin + (local / block) * block * interleave + member * w + local % block,
//     w = min(block, chunks - block * (local / block)),
// so that the `interleave` readers of one x chunk run at the same time and, the grid being a
// multiple of 8, on the same XCD: x is fetched from HBM once and found in that XCD's L2 by the
// others.  A unit on its own has interleave 1, member 0: position = begin + local.
struct UnitSchedule {
    uint32_t begin;
    uint16_t interleave;
    uint16_t member;
    uint32_t block;                  // chunks of one member that sit next to each other
    uint32_t skip;                   // leading chunks of the unit that the weight kernel handles:
                                     // they get no position; `local` above counts from the first
                                     // chunk after them
};

// A weight shared by the samples of an op, for the weight kernel: `members` units (first_unit,
// first_unit + unit_stride, ...) read the same x with their own gradients; the kernel takes the
// first `chunks` (whole, aligned) chunks of each, kWBatch members at a time, reading and
// quantising x once per batch.  Work item i of a call belongs to the group with the largest
// item_begin <= i; inside the group items run chunk by chunk, batch after batch.
constexpr int kWBatch = 8;
struct alignas(16) WGroup {          // 32 bytes
    uint32_t first_unit, unit_stride, members, chunks;
    uint32_t item_begin, reserved[3];
};
static_assert(sizeof(WGroup) == 32, "WGroup layout");

// Number of chunks of a unit (host side; the kernels use the same constants).
inline uint64_t unit_chunks_dense(int64_t n, uint32_t head) {
    if (n <= 0) return 0;
    uint64_t vecs = ((uint64_t)n + head + kVec - 1) / kVec;
    return (vecs + kChunkVecs - 1) / kChunkVecs;
}
inline uint32_t causal_chunks_per_mat(int64_t rows) {
    uint64_t bands = ((uint64_t)rows + kBandRows - 1) / kBandRows;
    uint64_t slots = (bands + 1) / 2;                  // bands are paired top with bottom
    return (uint32_t)((slots + kBandsPerChunk - 1) / kBandsPerChunk);
}

// ---- launchers (kernels.hip) ---------------------------------------------------------------
// All enqueue on `stream` and return the launch error, never synchronise.
// Persistent-grid size for the streaming kernels on the current device (resident workgroups).
// cls: the class of units the variant is for: 0 = one scale per tensor; 1 = row scales, rows of at
// least 512 elements or aligned causal rows; 2 = row scales, any other shape; 3 = row scales, rows
// of a power-of-two length below 512; 4, 5, 6 = row scales computed by the pass itself (single read),
// by the vectors of a row a thread holds: up to 4 (kept in registers), 8, 12 (parked in LDS; the launch
// of each class asks for the LDS its units need and no more, which decides how many workgroups a
// compute unit holds).
constexpr int kSensClasses = 7;
constexpr int kFirstFusedClass = 4;
inline int fused_class_of(int nv) { return kFirstFusedClass + (nv > kFusedRegNv ? 1 : 0) + (nv > 8 ? 1 : 0); }
inline size_t sens_class_lds_bytes(int cls) {
    return cls > kFirstFusedClass ? fused_lds_bytes(4 * (cls - kFirstFusedClass + 1)) : 0;   // class 4 keeps its rows in registers
}
int sens_resident_blocks(int n_fmts, int fmt0, int fmt1, int cls, int cus);
int absmax_resident_blocks(int cus);
int absmax_rows_resident_blocks(int cus);

// Host memory -> device memory through kernel arguments, one launch per piece; d_dst is 16-byte
// aligned and has room for `bytes` rounded up to 16.  The source is read before the call returns.
struct TablePiece { uint4 w[240]; };                   // 3840 bytes: fits the kernel-argument segment
hipError_t launch_table_write(const void* host_src, size_t bytes, void* d_dst, hipStream_t stream);
// The same table in fewer launches when its records repeat with fixed steps (the units of the R
// samples of one operand: pointers, output slots and schedule members advance by the same amount
// from sample to sample).  A run record stands for `count` units a fixed stride apart: the k-th is,
// 64-bit word by word of its WorkUnit and its UnitSchedule, first + k * step in wrapping arithmetic;
// a literal record is one unit as it stands.  Records travel as kernel arguments like the raw pieces
// and are expanded on the device to exactly the bytes launch_table_write would have written; the
// chunk_begin array (4 bytes per unit, a running sum that ragged samples make irregular) and the
// weight groups travel raw.
struct TableRun {                    // 176 bytes
    uint32_t first_unit, count;      // units first_unit + k * stride, k < count
    uint32_t stride, reserved;       // (the two operands of an op alternate in the table: stride 2)
    uint64_t unit[8], unit_step[8];  // WorkUnit
    uint64_t sched[2], sched_step[2];   // UnitSchedule
};
struct TableLiteral {                // 88 bytes
    uint32_t unit_index, reserved;
    uint64_t unit[8];
    uint64_t sched[2];
};
static_assert(sizeof(TableRun) == 176 && sizeof(TableLiteral) == 88, "record layout");
constexpr int kRunsPerPiece = (int)(sizeof(TablePiece) / sizeof(TableRun));            // 21
constexpr int kLiteralsPerPiece = (int)(sizeof(TablePiece) / sizeof(TableLiteral));    // 43
// Expands `n` run records (n literal records) taken from host memory into the unit table at d_table
// (units at offset 0, schedule at off_schedule), one launch per piece, one workgroup per record.
hipError_t launch_table_runs(const TableRun* host_runs, size_t n, void* d_table, size_t off_schedule,
                             hipStream_t stream);
hipError_t launch_table_literals(const TableLiteral* host_literals, size_t n, void* d_table, size_t off_schedule,
                                 hipStream_t stream);
// Once per set-up: unit records for the streaming kernels (scales not yet filled in) and the chunk map.
// Table, prepare and (resolve_fmts > 0) resolve of a small call in one launch of one workgroup: the
// table must fit one piece and the call have at most kSmallSetupChunks chunks.
constexpr uint32_t kSmallSetupChunks = 8192;
hipError_t launch_small_setup(const void* host_src, size_t bytes, void* d_dst, size_t off_cb, size_t off_schedule,
                              uint32_t n_units, uint32_t n_chunks, ResolvedUnit* d_runits, ChunkRef* d_map,
                              int resolve_fmts, hipStream_t stream);
hipError_t launch_prepare(const WorkUnit* d_units, const uint32_t* d_chunk_begin,
                          const UnitSchedule* d_schedule, uint32_t n_units, uint32_t n_chunks,
                          ResolvedUnit* d_runits, ChunkRef* d_map, hipStream_t stream);
// Every run: units with one scale per tensor get the values their scale pointers hold now; units
// with kUnitRowScale keep their table pointers.
hipError_t launch_resolve(const WorkUnit* d_units, uint32_t n_units, int n_fmts, ResolvedUnit* d_runits,
                          hipStream_t stream);
hipError_t launch_absmax(const ResolvedUnit* d_runits, const ChunkRef* d_map, uint32_t n_chunks,
                         uint32_t* d_partial_max, int grid, hipStream_t stream);
hipError_t launch_absmax_finalize(const uint32_t* d_chunk_begin, const uint32_t* d_partial_max,
                                  int n_tensors, int n_fmts, int fmt0, int fmt1, float* d_amax,
                                  float* d_scale, float* d_inv, uint32_t* d_flags,
                                  hipStream_t stream);
hipError_t launch_fake_quant(const uint16_t* d_x, int64_t n, float scale, float inv, int fmt,
                             uint8_t* d_codes, float* d_dequant, int grid, hipStream_t stream);
// fmt0 / fmt1 may carry the scale-rule flag: it selects the scaled-conversion variants (classes 0 and
// 4 to 6) and is the rule by which classes 4 to 6 derive their row scales.
hipError_t launch_sens(const ResolvedUnit* d_runits, const ChunkRef* d_map, uint32_t n_chunks,
                       int n_fmts, int fmt0, int fmt1, int cls, float* d_partials, int grid,
                       hipStream_t stream);
int sens_w_resident_blocks(int n_fmts, int fmt0, int fmt1, int rows, int cus);
hipError_t launch_sens_w(const WGroup* d_groups, uint32_t n_groups, uint32_t n_items,
                         const ResolvedUnit* d_runits, const uint32_t* d_chunk_begin, int n_fmts, int fmt0,
                         int fmt1, int rows, float* d_partials, int grid, hipStream_t stream);

// Per-row absmax (one scale per row).  One table entry per tensor; a work item is a run of
// rows_per_item consecutive rows of one tensor and belongs to one wave.
struct alignas(16) RowTensor {       // 48 bytes
    const uint16_t* x;
    int64_t n_rows;                  // all samples
    int32_t row_len;                 // elements between row starts
    int32_t causal_rows;             // 0: every row owns row_len entries; else rows per matrix, row i of a
                                     // matrix owns its first i + 1 + (row_len - causal_rows) entries
    uint32_t out_row;                // first row of this tensor in the output arrays
    uint32_t item_begin;             // first work item of this tensor
    uint32_t rows_per_item;
    uint32_t aligned;                // rows start on 16-byte boundaries and row_len % 8 == 0
    uint32_t items_per_mat;          // causal: a work item is a band of 8 rows from the top of a matrix and
                                     // its mirror from the bottom (equal work per item); 0 otherwise
    uint32_t reserved;
};
static_assert(sizeof(RowTensor) == 48, "RowTensor layout");
// Lanes of a wave that share one row in the per-row absmax: a power of two, at most 64, chosen so
// that a lane has about four vectors of its row to fetch; causal rows (whose valid length varies
// from one vector to the whole row) take 8 lanes, i.e. 8 neighbouring rows per wave step.
inline __host__ __device__ int absmax_row_lanes(int32_t row_len, bool causal) {
    const int nv = row_len / kVec;
    int L = 64;
    while (L > 1 && (L >> 1) * 4 >= nv) L >>= 1;
    if (causal && L > 8) L = 8;
    return L;
}
hipError_t launch_absmax_rows(const RowTensor* d_tensors, uint32_t n_tensors, uint32_t n_items,
                              int n_fmts, int fmt0, int fmt1, float* d_amax, float* d_scale,
                              float* d_inv, uint32_t* d_flags, int grid, hipStream_t stream);
hipError_t launch_sens_finalize(const ResolvedUnit* d_runits, const uint32_t* d_chunk_begin,
                                uint32_t n_units, int n_fmts, const float* d_partials,
                                float* d_out, hipStream_t stream);

}  // namespace ampsens
