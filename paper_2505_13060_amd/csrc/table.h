// Host side of a call: argument validation and the work table (units, chunk counts, schedule,
// weight groups) that the kernels of libampsens walk.  Header-only so that the C-ABI layer and the
// host-only test hooks (tests/host_hooks.cpp: replay of the kernels' index code, schedule checks)
// compile the very same code; nothing here touches the GPU.
#pragma once

#include "../../include/ampsens.h"
#include "internal.h"
#include "walk.h"

#include <algorithm>
#include <cstring>
#include <unordered_map>
#include <vector>

namespace ampsens {
namespace host {

constexpr int64_t kMaxDim = (int64_t)1 << 30;          // causal rows / cols
constexpr int64_t kMaxElems = (int64_t)1 << 46;        // per unit
constexpr uint64_t kMaxChunks = 0x7FFFFFFFull;

inline bool fmt_ok(int f) { return f == AMP_FP8_E4M3 || f == AMP_FP8_E5M2; }

// scale_flags: AMP_SCALE_POW2 may be or-ed into the formats (the absmax calls).
inline amp_status_t check_fmts(const amp_fp8_format_t* fmts, int n_fmts, bool scale_flags = false) {
    if (n_fmts < 1 || n_fmts > AMP_MAX_FORMATS) return AMP_ERR_BAD_FORMAT;
    if (!fmts) return AMP_ERR_INVALID_ARG;
    for (int f = 0; f < n_fmts; ++f)
        if (!fmt_ok(scale_flags ? ((int)fmts[f] & ~AMP_SCALE_POW2) : (int)fmts[f])) return AMP_ERR_BAD_FORMAT;
    return AMP_OK;
}

inline bool aligned2(const void* p) { return ((uintptr_t)p & 1u) == 0; }

inline amp_status_t check_layout(const amp_layout_t& L) {
    if (L.causal != 0 && L.causal != 1) return AMP_ERR_INVALID_ARG;
    if (L.causal) {
        if (L.batch < 0 || L.rows < 0 || L.cols < 0) return AMP_ERR_INVALID_ARG;
        if (L.rows > kMaxDim || L.cols > kMaxDim) return AMP_ERR_TOO_LARGE;
        if (L.rows && L.cols && L.batch > kMaxElems / L.rows / L.cols) return AMP_ERR_TOO_LARGE;
    } else {
        if (L.n_elems < 0) return AMP_ERR_INVALID_ARG;
        if (L.n_elems > kMaxElems) return AMP_ERR_TOO_LARGE;
    }
    return AMP_OK;
}

// Entries of one [rows, cols] matrix that belong to the operand: row i owns its first
// i + 1 + (cols - rows) columns, clipped to [0, cols] (the diagonal ends at the last column).
inline uint64_t causal_valid(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    const uint64_t r = (uint64_t)rows, c = (uint64_t)cols;
    if (cols >= rows) return r * (c - r + 1) + r * (r - 1) / 2;      // lengths c-r+1 .. c
    return c * (c + 1) / 2;                                          // the last c rows: lengths 1 .. c
}

inline int64_t layout_span(const amp_layout_t& L) {
    return L.causal ? L.batch * L.rows * L.cols : L.n_elems;
}

// The table that travels to the device: units, then chunk_begin[n_units + 1].
struct WorkTable {
    std::vector<WorkUnit> units;
    std::vector<uint32_t> chunk_begin;
    std::vector<uint32_t> group;                  // units with the same non-zero id share their x
    std::vector<uint64_t> unit_pairs;             // elements of each unit that belong to its operand
    uint64_t n_chunks = 0;
    uint64_t n_pairs = 0;                         // elements that belong to the operands
    bool any_rows = false;                        // some unit has one scale per row

    // x / dx may be null only for blocks without elements.
    amp_status_t add(const uint16_t* x, const uint16_t* dx, const amp_layout_t& L, int64_t batch_mul,
                     const float* scale, const float* inv, uint32_t out, uint32_t extra_flags = 0,
                     uint32_t group_id = 0, int64_t row_len = 0, bool fused = false) {
        // row_len != 0: scale / inv are [rows][n_fmts] tables starting at this unit's first row;
        // a dense unit is [n / row_len, row_len], a causal unit uses its own rows (row_len = cols).
        WorkUnit u;
        std::memset(&u, 0, sizeof(u));
        u.x = x; u.dx = dx; u.scale = scale; u.inv = inv; u.out = out;
        u.flags = extra_flags;
        if (row_len != 0) {
            u.flags |= kUnitRowScale;
            any_rows = true;
        }
        // fused: the pass computes the row scales itself (scale / inv are then outputs); only for rows
        // made of whole, aligned vectors
        if (fused) {
            const int64_t len = L.causal ? L.cols : row_len;
            const bool nice = ((uintptr_t)x % 16 == 0) && ((uintptr_t)dx % 16 == 0) && len % kVec == 0;
            if (row_len == 0 || !nice || len > kFusedMaxRowLen) return AMP_ERR_INVALID_ARG;
            u.flags |= kUnitFused;
        }
        uint64_t chunks;
        if (L.causal) {
            const int64_t batch = L.batch * batch_mul;
            u.flags |= kUnitCausal;
            u.n = batch;
            u.rows = (int32_t)L.rows;
            u.cols = (int32_t)L.cols;
            const bool nice = ((uintptr_t)x % 16 == 0) && (dx == nullptr || (uintptr_t)dx % 16 == 0) &&
                              (L.cols % kVec == 0);
            if (!nice) u.flags |= kUnitScalar;
            u.chunks_per_mat = (L.rows > 0 && L.cols > 0) ? causal_chunks_per_mat(L.rows) : 0;
            if (fused) {
                const FusedGeom g = fused_geometry(L.cols, true);
                u.head = g.pack();
                u.chunks_per_mat = (L.rows > 0 && L.cols > 0) ? fused_chunks_per_mat(L.rows, L.cols, g) : 0;
            }
            chunks = (uint64_t)batch * u.chunks_per_mat;
            if (chunks == 0) u.chunks_per_mat = 1;         // never divide by zero on the device
            const uint64_t valid = causal_valid(L.rows, L.cols);
            n_pairs += valid * (uint64_t)batch;
            unit_pairs.push_back(valid * (uint64_t)batch);
        } else {
            const int64_t n = L.n_elems * batch_mul;
            u.n = n;
            const uint32_t hx = (uint32_t)(((uintptr_t)x % 16) / 2);
            const bool mutual = dx == nullptr || ((uintptr_t)x % 16) == ((uintptr_t)dx % 16);
            if (mutual) u.head = hx; else { u.flags |= kUnitScalar; u.head = 0; }
            if (row_len != 0) {
                if (row_len < 0 || row_len > kMaxDim || n % row_len != 0) return AMP_ERR_INVALID_ARG;
                if (n / row_len > 0x7FFFFFFFll) return AMP_ERR_TOO_LARGE;
                u.cols = (int32_t)row_len;
                u.rows = (int32_t)(n / row_len);
                // rows must be made of whole vectors for the vector path
                if (row_len % kVec != 0 || u.head != 0) { u.flags |= kUnitScalar; u.head = 0; }
            }
            u.chunks_per_mat = 1;
            chunks = unit_chunks_dense(n, u.head);
            if (fused) {
                const FusedGeom g = fused_geometry(row_len, false);
                u.head = g.pack();
                chunks = fused_chunks_dense(u.rows, g);
            }
            n_pairs += (uint64_t)n;
            unit_pairs.push_back((uint64_t)n);
        }
        chunk_begin.push_back((uint32_t)n_chunks);
        group.push_back(group_id);
        n_chunks += chunks;
        if (n_chunks > kMaxChunks) return AMP_ERR_TOO_LARGE;
        units.push_back(u);
        return AMP_OK;
    }

    // units | chunk_begin[n + 1] (+ pad to 8 bytes) | schedule[n] (+ pad to 16) | weight groups
    size_t schedule_offset() const {
        return round8(units.size() * sizeof(WorkUnit) + (units.size() + 1) * sizeof(uint32_t));
    }
    size_t groups_offset() const {
        return (schedule_offset() + units.size() * sizeof(UnitSchedule) + 15) / 16 * 16;
    }
    size_t max_groups() const {
        std::vector<uint32_t> ids;
        for (uint32_t g : group) if (g != 0) ids.push_back(g);
        std::sort(ids.begin(), ids.end());
        return (size_t)(std::unique(ids.begin(), ids.end()) - ids.begin());
    }
    size_t table_bytes() const { return (groups_offset() + max_groups() * sizeof(WGroup) + 15) / 16 * 16; }
    static size_t round8(size_t v) { return (v + 7) / 8 * 8; }

    uint64_t chunks_of(size_t u) const {
        return (u + 1 < units.size() ? chunk_begin[u + 1] : n_chunks) - chunk_begin[u];
    }

    // Which streaming kernel takes a unit: 0 = one scale per tensor; 1 = one scale per row with
    // rows long enough that a wave's 512 contiguous elements meet at most two of them, or an
    // aligned causal unit; 3 = short rows of a power-of-two length (a wave step covers whole rows);
    // 2 = any other unit with row scales (other short rows, rows not made of whole vectors);
    // 4, 5, 6 = the single-read pass, by the LDS a workgroup needs for the unit's rows.
    static int unit_class(const WorkUnit& u) {
        if (!(u.flags & kUnitRowScale)) return 0;
        if (u.flags & kUnitFused) return fused_class_of(FusedGeom::unpack(u.head).nv);
        if (u.flags & kUnitScalar) return 2;
        if (u.flags & kUnitCausal) return 1;
        if (u.cols >= kVec * 64) return 1;
        return (u.cols & (u.cols - 1)) == 0 ? 3 : 2;        // a power of two (>= 8): whole rows per wave step
    }

    // How a call is split between the kernels.
    struct Plan {
        std::vector<UnitSchedule> schedule;       // positions of the chunks the streaming kernels take
        std::vector<WGroup> wgroups;              // work of the weight kernel: groups with one scale per
                                                  // tensor first, then those with row scales; item_begin
                                                  // counts from the first item of the group's launch
        uint64_t class_pos[kSensClasses + 1] = {};   // streaming kernel of class c: positions [class_pos[c], class_pos[c+1])
        uint64_t class_pairs[kSensClasses] = {};
        uint64_t n_positions = 0;
        size_t w_groups[2] = {0, 0};              // weight kernel launch v: groups, items, pairs, bytes
        uint64_t w_items[2] = {0, 0};
        uint64_t w_pairs[2] = {0, 0};             // element pairs the launch covers
        uint64_t w_bytes[2] = {0, 0};             // bytes it is defined to read: x once per batch, xdot per member
    };

    // Units stay in call order inside their class, except that the members of a group (same group
    // id, equal chunk counts, at most 65535 of them) are interleaved block by block.  With use_w, a
    // group whose members are whole-vector aligned and evenly spaced in the unit list hands its
    // whole chunks to the weight kernel; the ragged last chunk stays with the streaming kernel.
    Plan plan(uint32_t block, bool use_w) const {
        Plan P;
        P.schedule.resize(units.size());
        std::unordered_map<uint32_t, std::vector<size_t>> by_group;
        for (size_t u = 0; u < units.size(); ++u)
            if (group[u] != 0) by_group[group[u]].push_back(u);
        std::vector<char> done(units.size(), 0);
        for (int cls = 0; cls < kSensClasses; ++cls) {
            P.class_pos[cls] = P.n_positions;
            for (size_t u = 0; u < units.size(); ++u) {
                if (done[u] || unit_class(units[u]) != cls) continue;
                std::vector<size_t> members(1, u);
                if (group[u] != 0)
                    for (size_t v : by_group[group[u]])
                        if (v > u && !done[v] && chunks_of(v) == chunks_of(u) && members.size() < 65535 &&
                            unit_class(units[v]) == cls)
                            members.push_back(v);
                uint32_t skip = 0;
                if (use_w && members.size() >= 2) {
                    bool ok = true;
                    const size_t stride = members[1] - members[0];
                    for (size_t m = 0; m < members.size() && ok; ++m) {
                        const WorkUnit& w = units[members[m]];
                        ok = w.flags == units[u].flags && (w.flags & (kUnitCausal | kUnitScalar)) == 0 &&
                             w.head == 0 && w.x == units[u].x && w.n == units[u].n &&
                             w.scale == units[u].scale && w.inv == units[u].inv && w.cols == units[u].cols &&
                             members[m] == u + m * stride;
                    }
                    const uint64_t whole = (uint64_t)units[u].n / ((uint64_t)kChunkVecs * kVec);
                    if (ok && whole > 0) {
                        const int v = cls == 0 ? 0 : 1;
                        skip = (uint32_t)whole;
                        WGroup G;
                        std::memset(&G, 0, sizeof(G));
                        G.first_unit = (uint32_t)u;
                        G.unit_stride = (uint32_t)stride;
                        G.members = (uint32_t)members.size();
                        G.chunks = skip;
                        G.item_begin = (uint32_t)P.w_items[v];
                        P.wgroups.push_back(G);
                        P.w_groups[v] += 1;
                        P.w_items[v] += whole * ((members.size() + kWBatch - 1) / kWBatch);
                        P.w_pairs[v] += whole * (uint64_t)kChunkVecs * kVec * members.size();
                        P.w_bytes[v] += whole * (uint64_t)kChunkVecs * kVec * 2 *
                                        (members.size() + (members.size() + kWBatch - 1) / kWBatch);
                    }
                }
                for (size_t m = 0; m < members.size(); ++m) {
                    P.schedule[members[m]] = UnitSchedule{(uint32_t)P.n_positions, (uint16_t)members.size(),
                                                          (uint16_t)m, block, skip};
                    done[members[m]] = 1;
                    P.class_pairs[cls] += unit_pairs[members[m]] - (uint64_t)skip * kChunkVecs * kVec;
                }
                P.n_positions += (chunks_of(u) - skip) * members.size();
            }
        }
        P.class_pos[kSensClasses] = P.n_positions;
        return P;
    }

    // The table as it sits at the head of the workspace (table_bytes() bytes at `blob`).
    void fill_blob(const Plan& plan, uint8_t* blob) const {
        std::memset(blob, 0, table_bytes());
        if (!units.empty()) std::memcpy(blob, units.data(), units.size() * sizeof(WorkUnit));
        uint8_t* cb = blob + units.size() * sizeof(WorkUnit);
        if (!chunk_begin.empty()) std::memcpy(cb, chunk_begin.data(), chunk_begin.size() * 4);
        const uint32_t total = (uint32_t)n_chunks;
        std::memcpy(cb + chunk_begin.size() * 4, &total, 4);
        if (!plan.schedule.empty())
            std::memcpy(blob + schedule_offset(), plan.schedule.data(), plan.schedule.size() * sizeof(UnitSchedule));
        if (!plan.wgroups.empty())
            std::memcpy(blob + groups_offset(), plan.wgroups.data(), plan.wgroups.size() * sizeof(WGroup));
    }
};

// ---- the table as runs (internal.h: TableRun, TableLiteral) ------------------------------------------
// Cuts the units of a filled blob (units | chunk_begin | schedule) into runs of units, a fixed stride
// apart, whose 64-bit words (WorkUnit and UnitSchedule) advance by fixed steps; what is left of runs
// shorter than kMinRun becomes literals.
struct TableRecords {
    std::vector<TableRun> runs;
    std::vector<TableLiteral> literals;
    // launches the records need, with what travels raw (chunk_begin, weight groups)
    size_t launches(size_t raw_bytes) const {
        return (runs.size() + kRunsPerPiece - 1) / kRunsPerPiece +
               (literals.size() + kLiteralsPerPiece - 1) / kLiteralsPerPiece +
               (raw_bytes + sizeof(TablePiece) - 1) / sizeof(TablePiece);
    }
};
constexpr size_t kMinRun = 3;
constexpr size_t kMaxRunStride = 2;         // the two operands of an op alternate in the table

inline TableRecords table_records(const uint8_t* blob, size_t n_units, size_t off_schedule) {
    TableRecords T;
    auto unit_word = [&](size_t u, int w) { uint64_t v; std::memcpy(&v, blob + u * 64 + (size_t)w * 8, 8); return v; };
    auto sched_word = [&](size_t u, int w) { uint64_t v; std::memcpy(&v, blob + off_schedule + u * 16 + (size_t)w * 8, 8); return v; };
    // units a, a + s and b, b + s differ by the same steps
    auto same_step = [&](size_t a, size_t b, size_t s) {
        for (int w = 0; w < 8; ++w)
            if (unit_word(b + s, w) - unit_word(b, w) != unit_word(a + s, w) - unit_word(a, w)) return false;
        for (int w = 0; w < 2; ++w)
            if (sched_word(b + s, w) - sched_word(b, w) != sched_word(a + s, w) - sched_word(a, w)) return false;
        return true;
    };
    std::vector<char> done(n_units, 0);
    for (size_t u = 0; u < n_units; ++u) {
        if (done[u]) continue;
        size_t best_len = 1, best_stride = 1;
        for (size_t s = 1; s <= kMaxRunStride; ++s) {           // the longest run of units not yet covered
            size_t len = 1;
            while (u + len * s < n_units && !done[u + len * s] &&
                   (len == 1 || same_step(u, u + (len - 1) * s, s)))
                ++len;
            if (len > best_len) { best_len = len; best_stride = s; }
        }
        if (best_len >= kMinRun) {
            const size_t s = best_stride;
            TableRun R;
            std::memset(&R, 0, sizeof(R));
            R.first_unit = (uint32_t)u;
            R.count = (uint32_t)best_len;
            R.stride = (uint32_t)s;
            for (int w = 0; w < 8; ++w) { R.unit[w] = unit_word(u, w); R.unit_step[w] = unit_word(u + s, w) - unit_word(u, w); }
            for (int w = 0; w < 2; ++w) { R.sched[w] = sched_word(u, w); R.sched_step[w] = sched_word(u + s, w) - sched_word(u, w); }
            T.runs.push_back(R);
            for (size_t k = 0; k < best_len; ++k) done[u + k * s] = 1;
        } else {
            TableLiteral L;
            std::memset(&L, 0, sizeof(L));
            L.unit_index = (uint32_t)u;
            for (int w = 0; w < 8; ++w) L.unit[w] = unit_word(u, w);
            for (int w = 0; w < 2; ++w) L.sched[w] = sched_word(u, w);
            T.literals.push_back(L);
            done[u] = 1;
        }
    }
    return T;
}

// What the device makes of the records, on the host: the bytes of the units and of the schedule;
// everything else in `blob` is left as it is.
inline void table_expand(const TableRecords& T, uint8_t* blob, size_t off_schedule) {
    auto put = [&](size_t u, const uint64_t* unit, const uint64_t* sched) {
        std::memcpy(blob + u * 64, unit, 64);
        std::memcpy(blob + off_schedule + u * 16, sched, 16);
    };
    for (const TableRun& R : T.runs)
        for (uint32_t k = 0; k < R.count; ++k) {
            uint64_t unit[8], sched[2];
            for (int w = 0; w < 8; ++w) unit[w] = R.unit[w] + (uint64_t)k * R.unit_step[w];
            for (int w = 0; w < 2; ++w) sched[w] = R.sched[w] + (uint64_t)k * R.sched_step[w];
            put((size_t)R.first_unit + (size_t)k * R.stride, unit, sched);
        }
    for (const TableLiteral& L : T.literals) put(L.unit_index, L.unit, L.sched);
}

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace layout shared by the absmax and the sensitivity calls:
//   [ WorkUnit x n_units | chunk_begin | schedule | weight groups ]   written from the host's table
//   [ ResolvedUnit x n_units ] [ ChunkRef x n_chunks ]       written by the prepare kernel
//   [ per-wave partials ]                                    written by the streaming kernel
struct WsLayout {
    size_t runits, map, partials, total;
};

inline WsLayout ws_layout(const WorkTable& t, size_t partial_bytes_per_chunk) {
    WsLayout L;
    L.runits = round_up(t.table_bytes(), 256);
    L.map = L.runits + round_up(t.units.size() * sizeof(ResolvedUnit), 256);
    L.partials = L.map + round_up((size_t)t.n_chunks * sizeof(ChunkRef), 256);
    L.total = L.partials + round_up((size_t)t.n_chunks * partial_bytes_per_chunk, 256);
    return L;
}

constexpr uint32_t kDefaultScheduleBlock = 8;

inline WsLayout sens_layout(const WorkTable& t, int n_fmts) {
    return ws_layout(t, (size_t)kWaves * (n_fmts + 1) * sizeof(float));
}

// out_base (in / out): samples of the ops already in the table; this call's sums start there in d_out.
inline amp_status_t build_linear(const amp_linear_desc_t* ops, int n_ops, int n_fmts, WorkTable* t,
                          uint64_t* out_base = nullptr) {
    if (n_ops < 0 || (n_ops > 0 && !ops)) return AMP_ERR_INVALID_ARG;
    if (n_fmts < 1 || n_fmts > AMP_MAX_FORMATS) return AMP_ERR_BAD_FORMAT;
    uint64_t base = out_base ? *out_base : 0;
    for (int k = 0; k < n_ops; ++k) {
        const amp_linear_desc_t& op = ops[k];
        if (op.R < 0 || op.C < 0 || op.K < 0 || op.tokens < 0) return AMP_ERR_INVALID_ARG;
        // a weight is shared by the samples and small next to its R gradients: its row scales come from
        // amp_absmax_scale_rows, only the activations' can be computed by the pass itself
        const int32_t how = op.scale_rows & 0xFF;
        const int64_t blk = AMP_ROWS_BLOCK_OF(op.scale_rows);  // 0, or the length of a scale block inside a row
        if (how & ~(AMP_ROWS_OPERAND0 | AMP_ROWS_OPERAND1 | AMP_ROWS_COMPUTE0)) return AMP_ERR_INVALID_ARG;
        const bool x_fused = (how & AMP_ROWS_COMPUTE0) != 0;
        const bool x_rows = (how & AMP_ROWS_OPERAND0) != 0 || x_fused;
        const bool w_rows = (how & AMP_ROWS_OPERAND1) != 0;
        if (blk != 0 && (!(x_rows || w_rows) || op.C % blk != 0)) return AMP_ERR_INVALID_ARG;
        const int64_t scale_len = blk ? blk : op.C;          // elements that share a scale
        const int64_t per_row = blk ? op.C / blk : 1;
        if ((x_rows || w_rows) && op.C > kMaxDim) return AMP_ERR_TOO_LARGE;
        if (op.C > kMaxElems || op.K > kMaxElems || (op.C && op.K > kMaxElems / op.C)) return AMP_ERR_TOO_LARGE;
        if (!aligned2(op.x) || !aligned2(op.dx) || !aligned2(op.w) || !aligned2(op.dw)) return AMP_ERR_INVALID_ARG;
        const int64_t wn = op.K * op.C;
        int64_t prev = 0;
        for (int r = 0; r < op.R; ++r) {
            int64_t r0, r1;
            if (op.sample_row_offsets) {
                r0 = op.sample_row_offsets[r];
                r1 = op.sample_row_offsets[r + 1];
                if ((r == 0 && r0 != 0) || r0 != prev || r1 < r0) return AMP_ERR_INVALID_ARG;
                prev = r1;
            } else {
                r0 = (int64_t)r * op.tokens;
                r1 = r0 + op.tokens;
            }
            if (op.C && r1 > kMaxElems / op.C) return AMP_ERR_TOO_LARGE;
            const int64_t xn = (r1 - r0) * op.C;
            if (xn > 0 && (!op.x || !op.dx || !op.x_scale || !op.x_inv)) return AMP_ERR_INVALID_ARG;
            if (wn > 0 && (!op.w || !op.dw || !op.w_scale || !op.w_inv)) return AMP_ERR_INVALID_ARG;
            const uint64_t o = (base + r) * (uint64_t)n_fmts * 4;
            if (o + 4 * n_fmts > 0xFFFFFFFFull) return AMP_ERR_TOO_LARGE;
            amp_layout_t Lx = {xn, 0, 0, 0, 0, 0};
            amp_layout_t Lw = {wn, 0, 0, 0, 0, 0};
            const int64_t xs = x_rows ? r0 * per_row * n_fmts : 0;   // the sample's first token in the table
            amp_status_t st = t->add(xn ? op.x + r0 * op.C : op.x, xn ? op.dx + r0 * op.C : op.dx, Lx, 1,
                                     op.x_scale ? op.x_scale + xs : op.x_scale, op.x_inv ? op.x_inv + xs : op.x_inv,
                                     (uint32_t)o, 0u, 0u, x_rows && xn > 0 ? scale_len : 0, x_fused && xn > 0);
            if (st != AMP_OK) return st;
            st = t->add(op.w, wn ? op.dw + (int64_t)r * wn : op.dw, Lw, 1, op.w_scale, op.w_inv, (uint32_t)o + 2,
                        op.R > 1 ? kUnitKeepX : 0u, op.R > 1 ? (uint32_t)k + 1u : 0u, w_rows && wn > 0 ? scale_len : 0);
            if (st != AMP_OK) return st;
        }
        base += (uint64_t)op.R;
    }
    if (out_base) *out_base = base;
    return AMP_OK;
}

// Rows of one sample's block for per-row scales: a causal block has batch * rows rows of cols
// entries; a dense block is [n_elems / cols, cols] and must say its row length in cols.
inline amp_status_t row_geometry(const amp_layout_t& L, int64_t* row_len, int64_t* rows) {
    if (L.causal) {
        *row_len = L.cols;
        *rows = L.batch * L.rows;
        return AMP_OK;
    }
    if (L.n_elems == 0) { *row_len = 0; *rows = 0; return AMP_OK; }
    if (L.cols <= 0 || L.cols > kMaxDim || L.n_elems % L.cols != 0) return AMP_ERR_INVALID_ARG;
    *row_len = L.cols;
    *rows = L.n_elems / L.cols;
    return AMP_OK;
}

inline amp_status_t build_bgemm(const amp_bgemm_desc_t* ops, int n_ops, int n_fmts, WorkTable* t,
                         uint64_t* out_base = nullptr) {
    if (n_ops < 0 || (n_ops > 0 && !ops)) return AMP_ERR_INVALID_ARG;
    if (n_fmts < 1 || n_fmts > AMP_MAX_FORMATS) return AMP_ERR_BAD_FORMAT;
    uint64_t base = out_base ? *out_base : 0;
    for (int k = 0; k < n_ops; ++k) {
        const amp_bgemm_desc_t& op = ops[k];
        if (op.R < 0) return AMP_ERR_INVALID_ARG;
        amp_status_t st = check_layout(op.layout0);
        if (st != AMP_OK) return st;
        st = check_layout(op.layout1);
        if (st != AMP_OK) return st;
        if (!aligned2(op.x0) || !aligned2(op.dx0) || !aligned2(op.x1) || !aligned2(op.dx1)) return AMP_ERR_INVALID_ARG;
        const int64_t n0 = layout_span(op.layout0), n1 = layout_span(op.layout1);
        if (op.R > 0 && n0 > 0 && (!op.x0 || !op.dx0 || !op.scale0 || !op.inv0)) return AMP_ERR_INVALID_ARG;
        if (op.R > 0 && n1 > 0 && (!op.x1 || !op.dx1 || !op.scale1 || !op.inv1)) return AMP_ERR_INVALID_ARG;
        if (op.R > 0 && (n0 > kMaxElems / op.R || n1 > kMaxElems / op.R)) return AMP_ERR_TOO_LARGE;
        const int32_t how = op.scale_rows & 0xFF;
        const int64_t blk = AMP_ROWS_BLOCK_OF(op.scale_rows);
        if (how & ~(AMP_ROWS_OPERAND0 | AMP_ROWS_OPERAND1 | AMP_ROWS_COMPUTE0 | AMP_ROWS_COMPUTE1))
            return AMP_ERR_INVALID_ARG;
        if (blk != 0 && how == 0) return AMP_ERR_INVALID_ARG;
        const bool fused0 = (how & AMP_ROWS_COMPUTE0) != 0, fused1 = (how & AMP_ROWS_COMPUTE1) != 0;
        int64_t len0 = 0, len1 = 0, rows0 = 0, rows1 = 0;    // row length and rows per sample, 0 = one scale
        // a block of a dense row is a shorter row of the same buffer
        auto geometry = [&](const amp_layout_t& L, int64_t* len, int64_t* rows) -> amp_status_t {
            amp_status_t g = row_geometry(L, len, rows);
            if (g != AMP_OK || blk == 0 || (L.n_elems == 0 && !L.causal)) return g;
            if (L.causal || *len % blk != 0) return AMP_ERR_INVALID_ARG;
            *rows *= *len / blk;
            *len = blk;
            return AMP_OK;
        };
        if ((how & AMP_ROWS_OPERAND0) || fused0) {
            st = geometry(op.layout0, &len0, &rows0);
            if (st != AMP_OK) return st;
        }
        if ((how & AMP_ROWS_OPERAND1) || fused1) {
            st = geometry(op.layout1, &len1, &rows1);
            if (st != AMP_OK) return st;
        }
        for (int r = 0; r < op.R; ++r) {
            const uint64_t o = (base + r) * (uint64_t)n_fmts * 4;
            if (o + 4 * n_fmts > 0xFFFFFFFFull) return AMP_ERR_TOO_LARGE;
            const int64_t s0 = r * rows0 * n_fmts, s1 = r * rows1 * n_fmts;
            st = t->add(n0 ? op.x0 + r * n0 : op.x0, n0 ? op.dx0 + r * n0 : op.dx0, op.layout0, 1,
                        op.scale0 ? op.scale0 + s0 : op.scale0, op.inv0 ? op.inv0 + s0 : op.inv0, (uint32_t)o, 0u, 0u,
                        n0 > 0 ? len0 : 0, fused0 && n0 > 0);
            if (st != AMP_OK) return st;
            st = t->add(n1 ? op.x1 + r * n1 : op.x1, n1 ? op.dx1 + r * n1 : op.dx1, op.layout1, 1,
                        op.scale1 ? op.scale1 + s1 : op.scale1, op.inv1 ? op.inv1 + s1 : op.inv1, (uint32_t)o + 2, 0u,
                        0u, n1 > 0 ? len1 : 0, fused1 && n1 > 0);
            if (st != AMP_OK) return st;
        }
        base += (uint64_t)op.R;
    }
    if (out_base) *out_base = base;
    return AMP_OK;
}

inline amp_status_t build_absmax(const amp_tensor_t* tensors, int n_tensors, WorkTable* t) {
    if (n_tensors < 0 || (n_tensors > 0 && !tensors)) return AMP_ERR_INVALID_ARG;
    for (int k = 0; k < n_tensors; ++k) {
        const amp_tensor_t& T = tensors[k];
        amp_status_t st = check_layout(T.layout);
        if (st != AMP_OK) return st;
        if (T.n_samples < 0 || !aligned2(T.data)) return AMP_ERR_INVALID_ARG;
        const int64_t span = layout_span(T.layout);
        if (span > 0 && T.n_samples > kMaxElems / span) return AMP_ERR_TOO_LARGE;
        if (span * T.n_samples > 0 && !T.data) return AMP_ERR_INVALID_ARG;
        st = t->add(T.data, nullptr, T.layout, T.n_samples, nullptr, nullptr, (uint32_t)k);
        if (st != AMP_OK) return st;
    }
    return AMP_OK;
}

inline WsLayout absmax_layout(const WorkTable& t) { return ws_layout(t, (size_t)kWaves * sizeof(uint32_t)); }

struct RowPlan {
    std::vector<RowTensor> tensors;
    uint64_t n_items = 0, n_rows = 0;
};

inline amp_status_t build_absmax_rows(const amp_tensor_t* tensors, int n_tensors, RowPlan* P) {
    if (n_tensors < 0 || (n_tensors > 0 && !tensors)) return AMP_ERR_INVALID_ARG;
    for (int k = 0; k < n_tensors; ++k) {
        const amp_tensor_t& T = tensors[k];
        amp_status_t st = check_layout(T.layout);
        if (st != AMP_OK) return st;
        if (T.n_samples < 0 || !aligned2(T.data)) return AMP_ERR_INVALID_ARG;
        int64_t row_len = 0, rows = 0;
        st = row_geometry(T.layout, &row_len, &rows);
        if (st != AMP_OK) return st;
        if (rows > 0 && T.n_samples > kMaxElems / rows) return AMP_ERR_TOO_LARGE;
        const int64_t n_rows = row_len > 0 ? rows * T.n_samples : 0;
        if (n_rows > 0 && !T.data) return AMP_ERR_INVALID_ARG;
        RowTensor R;
        std::memset(&R, 0, sizeof(R));
        R.x = T.data;
        R.n_rows = n_rows;
        R.row_len = (int32_t)row_len;
        R.causal_rows = T.layout.causal ? (int32_t)T.layout.rows : 0;
        R.aligned = ((uintptr_t)T.data % 16 == 0 && row_len % kVec == 0) ? 1u : 0u;
        // about 16384 elements per work item: a whole number of the row groups a wave handles at once
        int64_t per = 1;
        if (row_len > 0) {
            const int64_t group = R.aligned ? 64 / absmax_row_lanes((int32_t)row_len, T.layout.causal != 0) : 1;
            per = 16384 / row_len > 0 ? 16384 / row_len : 1;
            per = (per + group - 1) / group * group;
        }
        R.rows_per_item = (uint32_t)per;
        if (P->n_rows + (uint64_t)n_rows > 0xFFFFFFFFull) return AMP_ERR_TOO_LARGE;
        R.out_row = (uint32_t)P->n_rows;
        R.item_begin = (uint32_t)P->n_items;
        P->n_rows += (uint64_t)n_rows;
        if (T.layout.causal && n_rows > 0) {
            const uint64_t bands = ((uint64_t)T.layout.rows + kBandRows - 1) / kBandRows;
            R.items_per_mat = (uint32_t)((bands + 1) / 2);
            P->n_items += (uint64_t)(n_rows / T.layout.rows) * R.items_per_mat;
        } else {
            P->n_items += ((uint64_t)n_rows + per - 1) / per;
        }
        if (P->n_items > kMaxChunks) return AMP_ERR_TOO_LARGE;
        P->tensors.push_back(R);
    }
    return AMP_OK;
}

}  // namespace host
}  // namespace ampsens
