// C-ABI layer of libampsens: argument validation, work-table construction on the host, and
// the launches.  See include/ampsens.h for the contract of every entry point.
//
// Every device call has two halves.  Set-up (host work proportional to the number of ops): validate,
// build the work table, send it to the head of the workspace as kernel arguments, and launch the
// prepare kernel, which derives the chunk map from it; what a run needs on the host afterwards is
// a few dozen numbers, kept in the caller's amp_plan_t.  Run: kernel launches only.  The one-shot
// entry points are set-up followed by run on the same stream.
#include "../../include/ampsens.h"
#include "internal.h"
#include "table.h"
#include "walk.h"

#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

using namespace ampsens;
using namespace ampsens::host;

namespace {

thread_local int g_last_device_error = 0;

amp_status_t device_error(hipError_t e) {
    g_last_device_error = (int)e;
    return AMP_ERR_DEVICE;
}

#define AMP_HIP(call)                                          \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return device_error(e_);         \
    } while (0)

int device_index() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    return dev;
}

int device_cus() {
    static std::mutex mu;
    static int cached[64];
    const int dev = device_index();
    if (dev < 0) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

// Persistent grid: as many workgroups as the kernel keeps resident on the device, never more
// than there are chunks, never more than the plan's limit (0 = none).
int persistent_grid(uint64_t n_chunks, int resident, int limit) {
    uint64_t cap = resident > 0 ? (uint64_t)resident : 1;
    if (limit > 0 && (uint64_t)limit < cap) cap = (uint64_t)limit;
    return (int)(n_chunks < cap ? n_chunks : cap);
}

int sens_resident(int n_fmts, int f0, int f1, int cls) {
    static std::mutex mu;
    static int cached[64][2][2][2][kSensClasses];
    const int dev = device_index();
    if (dev < 0) return sens_resident_blocks(n_fmts, f0, f1, cls, device_cus());
    std::lock_guard<std::mutex> lock(mu);
    int& slot = cached[dev][n_fmts - 1][f0][f1][cls];
    if (slot == 0) slot = sens_resident_blocks(n_fmts, f0, f1, cls, device_cus());
    return slot;
}

int sens_w_resident(int n_fmts, int f0, int f1, int rows) {
    static std::mutex mu;
    static int cached[64][2][2][2][2];
    const int dev = device_index();
    if (dev < 0) return sens_w_resident_blocks(n_fmts, f0, f1, rows, device_cus());
    std::lock_guard<std::mutex> lock(mu);
    int& slot = cached[dev][n_fmts - 1][f0][f1][rows];
    if (slot == 0) slot = sens_w_resident_blocks(n_fmts, f0, f1, rows, device_cus());
    return slot;
}

int absmax_resident(bool rows) {
    static std::mutex mu;
    static int cached[64][2];
    const int dev = device_index();
    if (dev < 0) return rows ? absmax_rows_resident_blocks(device_cus()) : absmax_resident_blocks(device_cus());
    std::lock_guard<std::mutex> lock(mu);
    int& slot = cached[dev][rows ? 1 : 0];
    if (slot == 0) slot = rows ? absmax_rows_resident_blocks(device_cus()) : absmax_resident_blocks(device_cus());
    return slot;
}

// ---- what a run needs to know, kept in the caller's amp_plan_t ----------------------------------
enum : uint32_t { kPlanMagic = 0x414D5031u, kPlanEmpty = 0, kPlanAbsmax = 1, kPlanAbsmaxRows = 2, kPlanSens = 3 };

struct PlanData {
    uint32_t magic, kind;
    uint8_t* ws;                                   // the workspace the set-up wrote
    int32_t n_fmts, fmt0, fmt1, grid_limit;
    uint32_t n_units, n_chunks;
    uint32_t resolved;                             // the set-up launch resolved the scales: the run that follows at once skips that
    uint32_t reserved;
    uint64_t off_cb, off_groups, off_runits, off_map, off_partials;    // the unit table sits at offset 0
    // sensitivity pass
    float* d_out;
    uint32_t w_groups[2], w_items[2];
    uint64_t w_pairs[2], w_bytes[2];
    uint64_t class_pos[kSensClasses + 1], class_pairs[kSensClasses];
    // absmax, per tensor and per row
    float *d_amax, *d_scale, *d_inv;
    uint32_t* d_flags;
    int32_t n_tensors;
    uint32_t n_items;
};
static_assert(sizeof(PlanData) <= sizeof(amp_plan_t), "amp_plan_t must hold the plan");

PlanData* plan_of(amp_plan_t* p) { return reinterpret_cast<PlanData*>(p); }

void plan_clear(PlanData* P, uint32_t kind) {
    std::memset(P, 0, sizeof(PlanData));
    P->magic = kPlanMagic;
    P->kind = kind;
}

// ---- optional timing of the sensitivity kernels -------------------------------------------------
struct Profile {
    std::mutex mu;
    std::vector<hipEvent_t> start, stop;
    std::vector<uint64_t> pairs, bytes;
    std::vector<int> kinds;
    int used = 0;
};
Profile g_profile;

// ---- set-up and run of the sensitivity pass ------------------------------------------------------

bool small_table(const WorkTable& t) {
    return t.table_bytes() <= sizeof(TablePiece) && t.n_chunks <= kSmallSetupChunks;
}

// A table of several pieces: units and schedule as runs with fixed steps and literal units, the rest
// raw, when that takes fewer launches (and reproduces the table byte for byte, which is checked here
// on the host); else piece by piece.
hipError_t send_table(const WorkTable& t, const std::vector<uint8_t>& blob, void* workspace, hipStream_t stream) {
    const size_t n = t.units.size(), off_cb = n * sizeof(WorkUnit), off_sched = t.schedule_offset();
    const size_t off_groups = t.groups_offset(), tail = blob.size() - off_groups;
    const size_t cb_bytes = (off_sched - off_cb + 15) / 16 * 16;            // chunk_begin[n + 1] and its padding
    const TableRecords rec = table_records(blob.data(), n, off_sched);
    const size_t raw = (blob.size() + sizeof(TablePiece) - 1) / sizeof(TablePiece);
    const size_t pieces = sizeof(TablePiece);
    if (rec.launches(0) + (cb_bytes + pieces - 1) / pieces + (tail + pieces - 1) / pieces < raw) {
        std::vector<uint8_t> check(blob);
        std::memset(check.data(), 0xEE, off_cb);
        std::memset(check.data() + off_sched, 0xEE, n * sizeof(UnitSchedule));
        table_expand(rec, check.data(), off_sched);
        if (std::memcmp(check.data(), blob.data(), blob.size()) == 0) {
            hipError_t e = launch_table_runs(rec.runs.data(), rec.runs.size(), workspace, off_sched, stream);
            if (e != hipSuccess) return e;
            e = launch_table_literals(rec.literals.data(), rec.literals.size(), workspace, off_sched, stream);
            if (e != hipSuccess) return e;
            // chunk_begin in whole 16-byte words: the word that also holds the first schedule entry's
            // bytes carries the same bytes the records have written (unit tables are multiples of 64)
            e = launch_table_write(blob.data() + off_cb, cb_bytes, (uint8_t*)workspace + off_cb, stream);
            if (e != hipSuccess) return e;
            return tail ? launch_table_write(blob.data() + off_groups, tail, (uint8_t*)workspace + off_groups, stream)
                        : hipSuccess;
        }
    }
    return launch_table_write(blob.data(), blob.size(), workspace, stream);
}

// run_at_once: the caller runs the plan right after, on the same stream, and never again: a small
// call then resolves its scales in the set-up launch.
amp_status_t sens_setup(const WorkTable& t, const amp_fp8_format_t* fmts, int n_fmts, float* d_out,
                        void* workspace, size_t workspace_bytes, uint32_t flags, hipStream_t stream,
                        PlanData* P, bool run_at_once = false) {
    plan_clear(P, kPlanEmpty);
    if (flags & ~(AMP_PLAN_STREAM_WEIGHTS | 0xFF00u)) return AMP_ERR_INVALID_ARG;
    if (t.units.empty()) return AMP_OK;
    if (!d_out || (uintptr_t)d_out % 4) return AMP_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 256) return AMP_ERR_INVALID_ARG;
    const WsLayout L = sens_layout(t, n_fmts);
    if (workspace_bytes < L.total) return AMP_ERR_WORKSPACE_TOO_SMALL;
    const uint32_t block = (flags >> 8) & 0xFFu;
    const WorkTable::Plan plan = t.plan(block ? block : kDefaultScheduleBlock, !(flags & AMP_PLAN_STREAM_WEIGHTS));
    std::vector<uint8_t> blob(t.table_bytes());
    t.fill_blob(plan, blob.data());
    const bool small = small_table(t);
    if (!small) AMP_HIP(send_table(t, blob, workspace, stream));
    uint8_t* ws = (uint8_t*)workspace;
    P->kind = kPlanSens;
    P->ws = ws;
    P->n_fmts = n_fmts;
    P->fmt0 = (int)fmts[0];
    P->fmt1 = (int)fmts[n_fmts - 1];
    P->n_units = (uint32_t)t.units.size();
    P->n_chunks = (uint32_t)t.n_chunks;
    P->off_cb = t.units.size() * sizeof(WorkUnit);
    P->off_groups = t.groups_offset();
    P->off_runits = L.runits;
    P->off_map = L.map;
    P->off_partials = L.partials;
    P->d_out = d_out;
    for (int v = 0; v < 2; ++v) {
        P->w_groups[v] = (uint32_t)plan.w_groups[v];
        P->w_items[v] = (uint32_t)plan.w_items[v];
        P->w_pairs[v] = plan.w_pairs[v];
        P->w_bytes[v] = plan.w_bytes[v];
    }
    for (int c = 0; c <= kSensClasses; ++c) P->class_pos[c] = plan.class_pos[c];
    for (int c = 0; c < kSensClasses; ++c) P->class_pairs[c] = plan.class_pairs[c];
    if (small) {
        AMP_HIP(launch_small_setup(blob.data(), blob.size(), ws, P->off_cb, t.schedule_offset(), P->n_units,
                                   P->n_chunks, (ResolvedUnit*)(ws + L.runits), (ChunkRef*)(ws + L.map),
                                   run_at_once ? n_fmts : 0, stream));
        P->resolved = run_at_once ? 1u : 0u;
        return AMP_OK;
    }
    AMP_HIP(launch_prepare((const WorkUnit*)ws, (const uint32_t*)(ws + P->off_cb),
                           (const UnitSchedule*)(ws + t.schedule_offset()), P->n_units, P->n_chunks,
                           (ResolvedUnit*)(ws + L.runits), (ChunkRef*)(ws + L.map), stream));
    return AMP_OK;
}

amp_status_t sens_run(const PlanData& P, hipStream_t stream) {
    uint8_t* ws = P.ws;
    const WorkUnit* d_units = (const WorkUnit*)ws;
    const uint32_t* d_cb = (const uint32_t*)(ws + P.off_cb);
    ResolvedUnit* d_runits = (ResolvedUnit*)(ws + P.off_runits);
    const ChunkRef* d_map = (const ChunkRef*)(ws + P.off_map);
    float* d_partials = (float*)(ws + P.off_partials);
    const WGroup* d_groups = (const WGroup*)(ws + P.off_groups);
    const int nf = P.n_fmts, f0 = P.fmt0 & 0xFF, f1 = P.fmt1 & 0xFF;     // fmt0 / fmt1 may carry the scale rule
    if (!P.resolved) AMP_HIP(launch_resolve(d_units, P.n_units, nf, d_runits, stream));
    // one pair of events around a fused kernel while the profile has room
    auto timed = [&](int kind, uint64_t pairs, uint64_t bytes, auto&& launch) -> hipError_t {
        int slot = -1;
        {
            std::lock_guard<std::mutex> lock(g_profile.mu);
            if (g_profile.used < (int)g_profile.start.size()) {
                slot = g_profile.used++;
                g_profile.pairs[slot] = pairs;
                g_profile.kinds[slot] = kind;
                g_profile.bytes[slot] = bytes;
            }
        }
        hipError_t e = slot >= 0 ? hipEventRecord(g_profile.start[slot], stream) : hipSuccess;
        if (e != hipSuccess) return e;
        e = launch();
        if (e != hipSuccess) return e;
        return slot >= 0 ? hipEventRecord(g_profile.stop[slot], stream) : hipSuccess;
    };
    // weight kernel: groups with one scale per tensor, then groups with one per output channel
    uint32_t g0 = 0;
    for (int v = 0; v < 2; ++v) {
        if (P.w_items[v] > 0) {
            const int grid = persistent_grid(P.w_items[v], sens_w_resident(nf, f0, f1, v), P.grid_limit);
            AMP_HIP(timed(AMP_KERNEL_WEIGHTS + v, P.w_pairs[v], P.w_bytes[v], [&]() {
                return launch_sens_w(d_groups + g0, P.w_groups[v], P.w_items[v], d_runits, d_cb, nf, f0, f1, v,
                                     d_partials, grid, stream);
            }));
        }
        g0 += P.w_groups[v];
    }
    // streaming kernels, one launch per class of units
    for (int cls = 0; cls < kSensClasses; ++cls) {
        const uint64_t n_pos = P.class_pos[cls + 1] - P.class_pos[cls];
        if (n_pos == 0) continue;
        const int grid = persistent_grid(n_pos, sens_resident(nf, f0, f1, cls), P.grid_limit);
        AMP_HIP(timed(AMP_KERNEL_STREAM + cls, P.class_pairs[cls], P.class_pairs[cls] * 4, [&]() {
            return launch_sens(d_runits, d_map + P.class_pos[cls], (uint32_t)n_pos, nf, P.fmt0, P.fmt1, cls,
                               d_partials, grid, stream);
        }));
    }
    AMP_HIP(launch_sens_finalize(d_runits, d_cb, P.n_units, nf, d_partials, P.d_out, stream));
    return AMP_OK;
}

// ---- set-up and run of the per-tensor absmax ------------------------------------------------------

amp_status_t absmax_setup(const WorkTable& t, int n_tensors, const amp_fp8_format_t* fmts, int n_fmts,
                          float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags, void* workspace,
                          size_t workspace_bytes, hipStream_t stream, PlanData* P) {
    plan_clear(P, kPlanEmpty);
    if (n_tensors == 0) return AMP_OK;
    if (!d_amax || !d_scale || !d_inv || !d_flags) return AMP_ERR_INVALID_ARG;
    if (((uintptr_t)d_amax | (uintptr_t)d_scale | (uintptr_t)d_inv | (uintptr_t)d_flags) % 4) return AMP_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 256) return AMP_ERR_INVALID_ARG;
    const WsLayout L = absmax_layout(t);
    if (workspace_bytes < L.total) return AMP_ERR_WORKSPACE_TOO_SMALL;
    const WorkTable::Plan plan = t.plan(kDefaultScheduleBlock, false);
    std::vector<uint8_t> blob(t.table_bytes());
    t.fill_blob(plan, blob.data());
    const bool small = small_table(t);
    if (!small) AMP_HIP(launch_table_write(blob.data(), blob.size(), workspace, stream));
    uint8_t* ws = (uint8_t*)workspace;
    P->kind = kPlanAbsmax;
    P->ws = ws;
    P->n_fmts = n_fmts;
    P->fmt0 = (int)fmts[0];
    P->fmt1 = (int)fmts[n_fmts - 1];
    P->n_units = (uint32_t)t.units.size();
    P->n_chunks = (uint32_t)t.n_chunks;
    P->off_cb = t.units.size() * sizeof(WorkUnit);
    P->off_runits = L.runits;
    P->off_map = L.map;
    P->off_partials = L.partials;
    P->d_amax = d_amax; P->d_scale = d_scale; P->d_inv = d_inv; P->d_flags = d_flags;
    P->n_tensors = n_tensors;
    if (small) {
        AMP_HIP(launch_small_setup(blob.data(), blob.size(), ws, P->off_cb, t.schedule_offset(), P->n_units,
                                   P->n_chunks, (ResolvedUnit*)(ws + L.runits), (ChunkRef*)(ws + L.map), 0, stream));
        return AMP_OK;
    }
    AMP_HIP(launch_prepare((const WorkUnit*)ws, (const uint32_t*)(ws + P->off_cb),
                           (const UnitSchedule*)(ws + t.schedule_offset()), P->n_units, P->n_chunks,
                           (ResolvedUnit*)(ws + L.runits), (ChunkRef*)(ws + L.map), stream));
    return AMP_OK;
}

amp_status_t absmax_run(const PlanData& P, hipStream_t stream) {
    uint8_t* ws = P.ws;
    const uint32_t* d_cb = (const uint32_t*)(ws + P.off_cb);
    uint32_t* d_partial_max = (uint32_t*)(ws + P.off_partials);
    if (P.n_chunks > 0)
        AMP_HIP(launch_absmax((const ResolvedUnit*)(ws + P.off_runits), (const ChunkRef*)(ws + P.off_map), P.n_chunks,
                              d_partial_max, persistent_grid(P.n_chunks, absmax_resident(false), P.grid_limit),
                              stream));
    AMP_HIP(launch_absmax_finalize(d_cb, d_partial_max, P.n_tensors, P.n_fmts, P.fmt0, P.fmt1, P.d_amax, P.d_scale,
                                   P.d_inv, P.d_flags, stream));
    return AMP_OK;
}

// ---- set-up and run of the per-row absmax ----------------------------------------------------------

amp_status_t absmax_rows_setup(const RowPlan& R, int n_tensors, const amp_fp8_format_t* fmts, int n_fmts,
                               float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags, void* workspace,
                               size_t workspace_bytes, hipStream_t stream, PlanData* P) {
    plan_clear(P, kPlanEmpty);
    if (n_tensors == 0) return AMP_OK;
    if (!d_flags || (uintptr_t)d_flags % 4) return AMP_ERR_INVALID_ARG;
    if (R.n_rows > 0 && (!d_amax || !d_scale || !d_inv)) return AMP_ERR_INVALID_ARG;
    if (((uintptr_t)d_amax | (uintptr_t)d_scale | (uintptr_t)d_inv) % 4) return AMP_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 256) return AMP_ERR_INVALID_ARG;
    const size_t bytes = R.tensors.size() * sizeof(RowTensor);
    if (workspace_bytes < round_up(bytes, 256)) return AMP_ERR_WORKSPACE_TOO_SMALL;
    AMP_HIP(launch_table_write(R.tensors.data(), bytes, workspace, stream));
    P->kind = kPlanAbsmaxRows;
    P->ws = (uint8_t*)workspace;
    P->n_fmts = n_fmts;
    P->fmt0 = (int)fmts[0];
    P->fmt1 = (int)fmts[n_fmts - 1];
    P->n_tensors = (int32_t)R.tensors.size();
    P->n_items = (uint32_t)R.n_items;
    P->d_amax = d_amax; P->d_scale = d_scale; P->d_inv = d_inv; P->d_flags = d_flags;
    return AMP_OK;
}

amp_status_t absmax_rows_run(const PlanData& P, hipStream_t stream) {
    const uint64_t wgs = ((uint64_t)P.n_items + kWaves - 1) / kWaves;
    const int grid = persistent_grid(wgs > 0 ? wgs : 1, absmax_resident(true), P.grid_limit);
    AMP_HIP(launch_absmax_rows((const RowTensor*)P.ws, (uint32_t)P.n_tensors, P.n_items, P.n_fmts, P.fmt0, P.fmt1,
                               P.d_amax, P.d_scale, P.d_inv, P.d_flags, grid, stream));
    return AMP_OK;
}

amp_status_t run_plan(const PlanData& P, hipStream_t stream) {
    if (P.magic != kPlanMagic) return AMP_ERR_INVALID_ARG;
    switch (P.kind) {
        case kPlanEmpty: return AMP_OK;
        case kPlanAbsmax: return absmax_run(P, stream);
        case kPlanAbsmaxRows: return absmax_rows_run(P, stream);
        case kPlanSens: return sens_run(P, stream);
    }
    return AMP_ERR_INVALID_ARG;
}

// ---- the workspace of the entry point that allocates nothing -------------------------------------
// A file-scope device array stands in for the caller's workspace.  Its name is a host-side handle,
// not a device address: the address is looked up once per device (every GPU that loads the library
// holds its own copy of the array) and only that pointer is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = (size_t)AMP_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

amp_status_t static_scratch(void** out) {
    static std::mutex mu;
    static void* ptr[64];
    const int dev = device_index();
    if (dev < 0) return device_error(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mu);
    if (ptr[dev] == nullptr) {
        void* p = nullptr;
        AMP_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        if (p == nullptr || (uintptr_t)p % 256) return device_error(hipErrorInvalidSymbol);
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return AMP_OK;
}

amp_status_t build_block(const amp_linear_desc_t* linears, int n_linears, const amp_bgemm_desc_t* bgemms,
                         int n_bgemms, int n_fmts, WorkTable* t) {
    uint64_t base = 0;
    amp_status_t st = build_linear(linears, n_linears, n_fmts, t, &base);
    if (st != AMP_OK) return st;
    return build_bgemm(bgemms, n_bgemms, n_fmts, t, &base);
}

}  // namespace

extern "C" {

// ---- absmax and scales per tensor ---------------------------------------------------------------

amp_status_t amp_absmax_workspace_bytes(const amp_tensor_t* tensors, int n_tensors, size_t* bytes) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    WorkTable t;
    amp_status_t st = build_absmax(tensors, n_tensors, &t);
    if (st != AMP_OK) return st;
    *bytes = absmax_layout(t).total;
    return AMP_OK;
}

amp_status_t amp_absmax_scale_setup(const amp_tensor_t* tensors, int n_tensors, const amp_fp8_format_t* fmts,
                                    int n_fmts, float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                                    void* workspace, size_t workspace_bytes, void* stream, amp_plan_t* plan) {
    if (!plan) return AMP_ERR_INVALID_ARG;
    std::memset(plan, 0, sizeof(*plan));               // stays invalid unless the set-up succeeds
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_absmax(tensors, n_tensors, &t);
    if (st != AMP_OK) return st;
    PlanData P;
    st = absmax_setup(t, n_tensors, fmts, n_fmts, d_amax, d_scale, d_inv, d_flags, workspace, workspace_bytes,
                      (hipStream_t)stream, &P);
    if (st != AMP_OK) return st;
    std::memcpy(plan, &P, sizeof(P));
    return AMP_OK;
}

amp_status_t amp_absmax_scale(const amp_tensor_t* tensors, int n_tensors, const amp_fp8_format_t* fmts,
                              int n_fmts, float* d_amax, float* d_scale, float* d_inv,
                              uint32_t* d_flags, void* workspace, size_t workspace_bytes,
                              void* stream) {
    amp_plan_t plan;
    amp_status_t st = amp_absmax_scale_setup(tensors, n_tensors, fmts, n_fmts, d_amax, d_scale, d_inv, d_flags,
                                             workspace, workspace_bytes, stream, &plan);
    if (st != AMP_OK) return st;
    return amp_run(&plan, stream);
}

// ---- absmax and scales per row ----------------------------------------------------------------

amp_status_t amp_absmax_rows_workspace_bytes(const amp_tensor_t* tensors, int n_tensors, size_t* bytes,
                                             int64_t* n_rows) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    RowPlan R;
    amp_status_t st = build_absmax_rows(tensors, n_tensors, &R);
    if (st != AMP_OK) return st;
    *bytes = round_up(R.tensors.size() * sizeof(RowTensor), 256);
    if (n_rows) *n_rows = (int64_t)R.n_rows;
    return AMP_OK;
}

amp_status_t amp_absmax_scale_rows_setup(const amp_tensor_t* tensors, int n_tensors, const amp_fp8_format_t* fmts,
                                         int n_fmts, float* d_amax, float* d_scale, float* d_inv,
                                         uint32_t* d_flags, void* workspace, size_t workspace_bytes, void* stream,
                                         amp_plan_t* plan) {
    if (!plan) return AMP_ERR_INVALID_ARG;
    std::memset(plan, 0, sizeof(*plan));
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    RowPlan R;
    st = build_absmax_rows(tensors, n_tensors, &R);
    if (st != AMP_OK) return st;
    PlanData P;
    st = absmax_rows_setup(R, n_tensors, fmts, n_fmts, d_amax, d_scale, d_inv, d_flags, workspace, workspace_bytes,
                           (hipStream_t)stream, &P);
    if (st != AMP_OK) return st;
    std::memcpy(plan, &P, sizeof(P));
    return AMP_OK;
}

amp_status_t amp_absmax_scale_rows(const amp_tensor_t* tensors, int n_tensors, const amp_fp8_format_t* fmts,
                                   int n_fmts, float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    amp_plan_t plan;
    amp_status_t st = amp_absmax_scale_rows_setup(tensors, n_tensors, fmts, n_fmts, d_amax, d_scale, d_inv, d_flags,
                                                  workspace, workspace_bytes, stream, &plan);
    if (st != AMP_OK) return st;
    return amp_run(&plan, stream);
}

// ---- standalone fake quantisation ---------------------------------------------------------------

amp_status_t amp_fake_quant_fp8(const uint16_t* d_x, int64_t n, float scale, float inv_scale,
                                amp_fp8_format_t fmt, uint8_t* d_codes, float* d_dequant,
                                void* stream_) {
    if (!fmt_ok((int)fmt)) return AMP_ERR_BAD_FORMAT;
    if (n < 0) return AMP_ERR_INVALID_ARG;
    if (n == 0) return AMP_OK;
    if (!d_x || !d_codes || !aligned2(d_x) || (d_dequant && (uintptr_t)d_dequant % 4)) return AMP_ERR_INVALID_ARG;
    if (n > kMaxElems) return AMP_ERR_TOO_LARGE;
    const uint64_t blocks = ((uint64_t)n / kVec + kWG - 1) / kWG + 1;
    const uint64_t cap = (uint64_t)device_cus() * 8;
    AMP_HIP(launch_fake_quant(d_x, n, scale, inv_scale, (int)fmt, d_codes, d_dequant,
                              (int)(blocks < cap ? blocks : cap), (hipStream_t)stream_));
    return AMP_OK;
}

// ---- the fused sensitivity pass -------------------------------------------------------------------

amp_status_t amp_sens_linear_workspace_bytes(const amp_linear_desc_t* ops, int n_ops, int n_fmts, size_t* bytes) {
    return amp_sens_block_workspace_bytes(ops, n_ops, nullptr, 0, n_fmts, bytes);
}

amp_status_t amp_sens_linear(const amp_linear_desc_t* ops, int n_ops, const amp_fp8_format_t* fmts,
                             int n_fmts, float* d_out, void* workspace, size_t workspace_bytes,
                             void* stream) {
    return amp_sens_block(ops, n_ops, nullptr, 0, fmts, n_fmts, d_out, workspace, workspace_bytes, stream);
}

amp_status_t amp_sens_bgemm_workspace_bytes(const amp_bgemm_desc_t* ops, int n_ops, int n_fmts, size_t* bytes) {
    return amp_sens_block_workspace_bytes(nullptr, 0, ops, n_ops, n_fmts, bytes);
}

amp_status_t amp_sens_bgemm(const amp_bgemm_desc_t* ops, int n_ops, const amp_fp8_format_t* fmts,
                            int n_fmts, float* d_out, void* workspace, size_t workspace_bytes,
                            void* stream) {
    return amp_sens_block(nullptr, 0, ops, n_ops, fmts, n_fmts, d_out, workspace, workspace_bytes, stream);
}

amp_status_t amp_sens_block_workspace_bytes(const amp_linear_desc_t* linears, int n_linears,
                                            const amp_bgemm_desc_t* bgemms, int n_bgemms, int n_fmts,
                                            size_t* bytes) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    WorkTable t;
    amp_status_t st = build_block(linears, n_linears, bgemms, n_bgemms, n_fmts, &t);
    if (st != AMP_OK) return st;
    *bytes = sens_layout(t, n_fmts).total;
    return AMP_OK;
}

amp_status_t amp_sens_block_setup(const amp_linear_desc_t* linears, int n_linears, const amp_bgemm_desc_t* bgemms,
                                  int n_bgemms, const amp_fp8_format_t* fmts, int n_fmts, float* d_out,
                                  void* workspace, size_t workspace_bytes, uint32_t flags, void* stream,
                                  amp_plan_t* plan) {
    if (!plan) return AMP_ERR_INVALID_ARG;
    std::memset(plan, 0, sizeof(*plan));
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_block(linears, n_linears, bgemms, n_bgemms, n_fmts, &t);
    if (st != AMP_OK) return st;
    PlanData P;
    st = sens_setup(t, fmts, n_fmts, d_out, workspace, workspace_bytes, flags, (hipStream_t)stream, &P);
    if (st != AMP_OK) return st;
    std::memcpy(plan, &P, sizeof(P));
    return AMP_OK;
}

amp_status_t amp_sens_block(const amp_linear_desc_t* linears, int n_linears, const amp_bgemm_desc_t* bgemms,
                            int n_bgemms, const amp_fp8_format_t* fmts, int n_fmts, float* d_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_block(linears, n_linears, bgemms, n_bgemms, n_fmts, &t);
    if (st != AMP_OK) return st;
    PlanData P;
    st = sens_setup(t, fmts, n_fmts, d_out, workspace, workspace_bytes, 0u, (hipStream_t)stream, &P, true);
    if (st != AMP_OK) return st;
    return run_plan(P, (hipStream_t)stream);
}

amp_status_t amp_sens_block_static(const amp_linear_desc_t* linears, int n_linears, const amp_bgemm_desc_t* bgemms,
                                   int n_bgemms, const amp_fp8_format_t* fmts, int n_fmts, float* d_out,
                                   void* stream) {
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_block(linears, n_linears, bgemms, n_bgemms, n_fmts, &t);
    if (st != AMP_OK) return st;
    if (t.units.empty()) return AMP_OK;
    if (sens_layout(t, n_fmts).total > kStaticScratchBytes) return AMP_ERR_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    st = static_scratch(&ws);
    if (st != AMP_OK) return st;
    PlanData P;
    st = sens_setup(t, fmts, n_fmts, d_out, ws, kStaticScratchBytes, 0u, (hipStream_t)stream, &P, true);
    if (st != AMP_OK) return st;
    return run_plan(P, (hipStream_t)stream);
}

// ---- plans ------------------------------------------------------------------------------------------

amp_status_t amp_plan_limit_grid(amp_plan_t* plan, int max_workgroups) {
    if (!plan || plan_of(plan)->magic != kPlanMagic || max_workgroups < 0) return AMP_ERR_INVALID_ARG;
    plan_of(plan)->grid_limit = max_workgroups;
    return AMP_OK;
}

amp_status_t amp_run(const amp_plan_t* plan, void* stream) {
    if (!plan) return AMP_ERR_INVALID_ARG;
    PlanData P;
    std::memcpy(&P, plan, sizeof(P));
    return run_plan(P, (hipStream_t)stream);
}

// ---- optional kernel timing -----------------------------------------------------------------------

amp_status_t amp_profile_enable(int max_launches) {
    if (max_launches < 0) return AMP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_profile.mu);
    for (hipEvent_t e : g_profile.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_profile.stop) (void)hipEventDestroy(e);
    g_profile.start.clear();
    g_profile.stop.clear();
    g_profile.pairs.assign((size_t)max_launches, 0);
    g_profile.bytes.assign((size_t)max_launches, 0);
    g_profile.kinds.assign((size_t)max_launches, 0);
    g_profile.used = 0;
    for (int i = 0; i < max_launches; ++i) {
        hipEvent_t a, b;
        AMP_HIP(hipEventCreate(&a));
        g_profile.start.push_back(a);
        AMP_HIP(hipEventCreate(&b));
        g_profile.stop.push_back(b);
    }
    return AMP_OK;
}

amp_status_t amp_profile_kinds(int* kinds, int capacity, int* n_launches) {
    if (!n_launches || capacity < 0 || (capacity > 0 && !kinds)) return AMP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_profile.mu);
    if (capacity < g_profile.used) return AMP_ERR_INVALID_ARG;
    for (int i = 0; i < g_profile.used; ++i) kinds[i] = g_profile.kinds[i];
    *n_launches = g_profile.used;
    return AMP_OK;
}

amp_status_t amp_profile_read(float* ms, uint64_t* pairs, uint64_t* bytes, int capacity, int* n_launches) {
    if (!n_launches || capacity < 0 || (capacity > 0 && !ms)) return AMP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_profile.mu);
    if (capacity < g_profile.used) return AMP_ERR_INVALID_ARG;
    for (int i = 0; i < g_profile.used; ++i) {
        AMP_HIP(hipEventSynchronize(g_profile.stop[i]));
        AMP_HIP(hipEventElapsedTime(&ms[i], g_profile.start[i], g_profile.stop[i]));
        if (pairs) pairs[i] = g_profile.pairs[i];
        if (bytes) bytes[i] = g_profile.bytes[i];
    }
    *n_launches = g_profile.used;
    g_profile.used = 0;
    return AMP_OK;
}

// ---- misc -------------------------------------------------------------------------------------------

const char* amp_status_string(amp_status_t status) {
    switch (status) {
        case AMP_OK: return "ok";
        case AMP_ERR_INVALID_ARG: return "invalid argument";
        case AMP_ERR_BAD_FORMAT: return "bad FP8 format or format count";
        case AMP_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case AMP_ERR_NONFINITE_INPUT: return "non-finite input";
        case AMP_ERR_DEVICE: return "HIP runtime error";
        case AMP_ERR_INFEASIBLE: return "no configuration meets the loss-MSE budget";
        case AMP_ERR_TOO_LARGE: return "problem too large";
    }
    return "unknown status";
}

int amp_last_device_error(void) { return g_last_device_error; }

int amp_version(void) { return 200; }

}  // extern "C"
