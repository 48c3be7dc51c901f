// TEST INFRASTRUCTURE, host only.  Replays on the CPU, thread by thread, the element walk the
// library's kernels perform (csrc/walk.h is a host+device template, csrc/table.h builds the same
// work table the C-ABI layer builds) and checks schedules.  Built into a shared library of its own
// by tests/conftest.py; the product library exports none of this.
#include "../include/ampsens.h"
#include "../paper_2505_13060_amd/csrc/internal.h"
#include "../paper_2505_13060_amd/csrc/table.h"
#include "../paper_2505_13060_amd/csrc/walk.h"

#include <vector>

using namespace ampsens;
using namespace ampsens::host;

namespace {

// A context for walk_chunk that records which elements a thread touches.  counts has `span`
// entries (the unit's memory span in elements); bad counts accesses outside [0, span), "full"
// vectors that are not 16-byte aligned, and vectors whose tracked row is wrong.
struct ReplayCtx {
    static constexpr bool kRollDense = false;
    int32_t* counts;
    int64_t span;
    uintptr_t addr;          // byte address the unit would have
    int64_t bad;
    // row tracking as a context with one scale per row would do it; row_len 0 = no check
    int32_t row_len = 0;
    bool cursor_mode = false, have_row = false;
    bool wave_mode = false;                         // track the wave's first lane only (see wave_lane_row)
    int32_t last_row = 0;
    int lane = 0;
    RowCursor cur;
    int64_t row = 0;
    void begin_dense(int64_t e0, int le) {
        if (row_len > 0 && cursor_mode) cur.begin(e0, wave_mode ? le - lane * kVec : le, kWG * kVec, row_len);
    }
    void set_row(int64_t r) { row = r; have_row = true; }
    // a vector that starts at element s is about to be consumed
    void vector_row(int64_t s) {
        if (row_len <= 0) return;
        if (cursor_mode && wave_mode) {
            if (wave_lane_row(cur, last_row, wave_sub_shift(row_len), lane) != s / row_len ||
                s % row_len + kVec > row_len)
                ++bad;
            cur.advance();
        } else if (cursor_mode) {
            if (cur.row != s / row_len || cur.col != s % row_len || cur.col + kVec > row_len) ++bad;
            cur.advance();
        } else if (!have_row || s / row_len != row || s % row_len + kVec > row_len) {
            ++bad;
        }
    }
    void touch(int64_t e) { if (e < 0 || e >= span) ++bad; else ++counts[e]; }
    template <int U> void full(int64_t eu, int le, int64_t stride) {
        for (int k = 0; k < U; ++k) {
            const int64_t s = eu + le + k * stride;
            if ((addr + 2 * (uintptr_t)s) % 16) ++bad;
            vector_row(s);
            for (int j = 0; j < kVec; ++j) touch(s + j);
        }
    }
    template <int U> void full_masked(int64_t e, int stride, int count, int tail) {
        if (count < 0 || count > U || (count > 0 && (tail < 1 || tail > kVec))) ++bad;
        for (int k = 0; k < count; ++k) {
            const int64_t s = e + (int64_t)k * stride;
            if ((addr + 2 * (uintptr_t)s) % 16) ++bad;
            if (s < 0 || s + kVec > span) ++bad;              // the whole vector is fetched
            vector_row(s);
            const int valid = (k == count - 1) ? tail : kVec;
            for (int j = 0; j < valid; ++j) touch(s + j);
        }
    }
    void partial(int64_t e, int jlo, int jhi) {
        // element-wise contexts divide per element; a cursor context is never given a partial
        // vector of a unit whose rows are whole vectors, except in causal chunks (explicit row)
        if (row_len > 0 && cursor_mode) ++bad;
        if (row_len > 0 && !cursor_mode && have_row)
            for (int j = jlo; j < jhi; ++j) if ((e + j) / row_len != row) ++bad;
        for (int j = jlo; j < jhi; ++j) touch(e + j);
    }
};

}  // namespace

extern "C" {

// Checks that the schedule of a linear call is a permutation of its chunks; returns the number of
// positions that are out of range, hit twice or never hit, and reports the number of chunks and how
// many units are interleaved with others.  block 0 = the default; use_w as the set-up flag.
int64_t hooks_check_linear_schedule(const amp_linear_desc_t* ops, int n_ops, int n_fmts, int block, int use_w,
                                    uint64_t* n_chunks_out, uint64_t* interleaved_units) {
    WorkTable t;
    if (build_linear(ops, n_ops, n_fmts, &t) != AMP_OK) return -1;
    const WorkTable::Plan plan = t.plan(block > 0 ? (uint32_t)block : kDefaultScheduleBlock, use_w != 0);
    const std::vector<UnitSchedule>& sch = plan.schedule;
    std::vector<uint8_t> hit(plan.n_positions, 0);
    int64_t bad = 0;
    uint64_t inter = 0;
    for (size_t u = 0; u < t.units.size(); ++u) {
        const uint32_t chunks = (uint32_t)t.chunks_of(u) - sch[u].skip;
        if (sch[u].interleave > 1) ++inter;
        for (uint32_t l = 0; l < chunks; ++l) {
            const uint32_t pos = schedule_position(sch[u], l, chunks);
            if (pos >= plan.n_positions || hit[pos]) ++bad; else hit[pos] = 1;
        }
    }
    for (uint8_t h : hit) if (!h) ++bad;
    // the weight kernel's items: every (member, whole chunk) of a group exactly once, in bounds
    std::vector<uint32_t> covered(t.units.size(), 0);
    uint64_t items = 0;
    size_t gi = 0;
    for (const WGroup& G : plan.wgroups) {
        if (gi++ == plan.w_groups[0]) {                        // the second launch counts from 0 again
            if (items != plan.w_items[0]) ++bad;
            items = 0;
        }
        if (G.item_begin != items) ++bad;
        items += (uint64_t)G.chunks * ((G.members + kWBatch - 1) / kWBatch);
        for (uint32_t m = 0; m < G.members; ++m) {
            const size_t u = G.first_unit + (size_t)m * G.unit_stride;
            if (u >= t.units.size()) { ++bad; continue; }
            covered[u] += G.chunks;
            if ((uint64_t)G.chunks * kChunkVecs * kVec > (uint64_t)t.units[u].n) ++bad;
        }
    }
    if (items != plan.w_items[plan.w_groups[1] > 0 ? 1 : 0]) ++bad;
    for (size_t u = 0; u < t.units.size(); ++u)
        if (covered[u] != sch[u].skip) ++bad;
    // the table that travels to the device has room for what the plan holds
    if (plan.wgroups.size() > t.max_groups()) ++bad;
    std::vector<uint8_t> blob(t.table_bytes());
    t.fill_blob(plan, blob.data());
    if (n_chunks_out) *n_chunks_out = t.n_chunks;
    if (interleaved_units) *interleaved_units = inter;
    return bad;
}

// The table of a linear call as run and literal records: expands them on the host and compares with
// the table itself; returns the number of differing bytes (or -1), and reports the record counts and
// the launches the raw table would take.
int64_t hooks_table_records(const amp_linear_desc_t* ops, int n_ops, int n_fmts, uint64_t* n_runs,
                            uint64_t* n_literals, uint64_t* raw_pieces, uint64_t* n_units) {
    WorkTable t;
    if (build_linear(ops, n_ops, n_fmts, &t) != AMP_OK) return -1;
    const WorkTable::Plan plan = t.plan(kDefaultScheduleBlock, true);
    std::vector<uint8_t> blob(t.table_bytes());
    t.fill_blob(plan, blob.data());
    const size_t n = t.units.size(), off_cb = n * sizeof(WorkUnit), off_sched = t.schedule_offset();
    const TableRecords rec = table_records(blob.data(), n, off_sched);
    std::vector<uint8_t> check(blob);
    std::memset(check.data(), 0xEE, off_cb);                                          // the units
    std::memset(check.data() + off_sched, 0xEE, n * sizeof(UnitSchedule));
    table_expand(rec, check.data(), off_sched);
    int64_t bad = 0;
    for (size_t i = 0; i < blob.size(); ++i) bad += blob[i] != check[i];
    uint64_t covered = rec.literals.size();
    for (const TableRun& R : rec.runs) covered += R.count;
    if (covered != n) ++bad;
    *n_runs = rec.runs.size();
    *n_literals = rec.literals.size();
    *raw_pieces = (blob.size() + sizeof(TablePiece) - 1) / sizeof(TablePiece);
    *n_units = n;
    return bad;
}

// row_len != 0 also replays the row tracking of a unit with one scale per row and counts every
// vector whose tracked row differs from (element index / row_len), or that straddles two rows.
int64_t hooks_replay_unit_rows(uint64_t x_addr, uint64_t dx_addr, const amp_layout_t* layout,
                               int64_t batch_mul, int64_t row_len, int32_t* counts, int64_t span,
                               uint64_t* n_chunks_out) {
    WorkTable t;
    if (t.add((const uint16_t*)(uintptr_t)x_addr, (const uint16_t*)(uintptr_t)dx_addr, *layout, batch_mul,
              nullptr, nullptr, 0, 0u, 0u, row_len) != AMP_OK)
        return -1;
    std::vector<uint32_t> cb = t.chunk_begin;
    cb.push_back((uint32_t)t.n_chunks);
    const WorkUnit& u = t.units[0];
    for (uint32_t c = 0; c < t.n_chunks; ++c) {
        if (find_unit(cb.data(), 1, c) != 0) return -2;
    }
    int64_t bad = 0;
    for (uint32_t c = 0; c < t.n_chunks; ++c) {
        for (int tid = 0; tid < kWG; ++tid) {
            ReplayCtx ctx{counts, span, (uintptr_t)x_addr, 0};
            if (u.flags & kUnitRowScale) {
                ctx.row_len = u.cols;
                ctx.cursor_mode = !(u.flags & kUnitCausal) && !(u.flags & kUnitScalar);
                if (!(u.flags & kUnitCausal) && (u.flags & kUnitScalar)) ctx.row_len = 0;   // divides per element
                ctx.wave_mode = ctx.cursor_mode && WorkTable::unit_class(u) != 2;
                ctx.last_row = u.rows - 1;
                ctx.lane = tid & 63;
            }
            walk_chunk(u, c, tid, ctx);
            bad += ctx.bad;
        }
    }
    if (n_chunks_out) *n_chunks_out = t.n_chunks;
    return bad;
}

int64_t hooks_replay_unit(uint64_t x_addr, uint64_t dx_addr, const amp_layout_t* layout, int64_t batch_mul,
                          int32_t* counts, int64_t span, uint64_t* n_chunks_out) {
    WorkTable t;
    if (t.add((const uint16_t*)(uintptr_t)x_addr, (const uint16_t*)(uintptr_t)dx_addr, *layout, batch_mul,
              nullptr, nullptr, 0) != AMP_OK)
        return -1;
    std::vector<uint32_t> cb = t.chunk_begin;
    cb.push_back((uint32_t)t.n_chunks);
    ReplayCtx ctx{counts, span, (uintptr_t)x_addr, 0};
    for (uint32_t c = 0; c < t.n_chunks; ++c) {
        if (find_unit(cb.data(), 1, c) != 0) ++ctx.bad;
        for (int tid = 0; tid < kWG; ++tid) walk_chunk(t.units[0], c, tid, ctx);
    }
    if (n_chunks_out) *n_chunks_out = t.n_chunks;
    return ctx.bad;
}

}  // extern "C"
