// C-ABI layer of libampsens: argument validation, work-table construction on the host, and
// the launches.  See include/ampsens.h for the contract of every entry point.
#include "../../include/ampsens.h"
#include "internal.h"
#include "walk.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <unordered_map>
#include <vector>

using namespace ampsens;

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

constexpr int64_t kMaxDim = (int64_t)1 << 30;          // causal rows / cols
constexpr int64_t kMaxElems = (int64_t)1 << 46;        // per unit
constexpr uint64_t kMaxChunks = 0x7FFFFFFFull;

bool fmt_ok(int f) { return f == AMP_FP8_E4M3 || f == AMP_FP8_E5M2; }

// scale_flags: AMP_SCALE_POW2 may be or-ed into the formats (the absmax calls).
amp_status_t check_fmts(const amp_fp8_format_t* fmts, int n_fmts, bool scale_flags = false) {
    if (n_fmts < 1 || n_fmts > AMP_MAX_FORMATS) return AMP_ERR_BAD_FORMAT;
    if (!fmts) return AMP_ERR_INVALID_ARG;
    for (int f = 0; f < n_fmts; ++f)
        if (!fmt_ok(scale_flags ? ((int)fmts[f] & ~AMP_SCALE_POW2) : (int)fmts[f])) return AMP_ERR_BAD_FORMAT;
    return AMP_OK;
}

bool aligned2(const void* p) { return ((uintptr_t)p & 1u) == 0; }

amp_status_t check_layout(const amp_layout_t& L) {
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
uint64_t causal_valid(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    const uint64_t r = (uint64_t)rows, c = (uint64_t)cols;
    if (cols >= rows) return r * (c - r + 1) + r * (r - 1) / 2;      // lengths c-r+1 .. c
    return c * (c + 1) / 2;                                          // the last c rows: lengths 1 .. c
}

int64_t layout_span(const amp_layout_t& L) {
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
                     uint32_t group_id = 0, int64_t row_len = 0) {
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
    size_t table_bytes() const { return groups_offset() + max_groups() * sizeof(WGroup); }
    static size_t round8(size_t v) { return (v + 7) / 8 * 8; }

    uint64_t chunks_of(size_t u) const {
        return (u + 1 < units.size() ? chunk_begin[u + 1] : n_chunks) - chunk_begin[u];
    }

    // Which streaming kernel takes a unit: 0 = one scale per tensor; 1 = one scale per row with
    // rows long enough that a wave's 512 contiguous elements meet at most two of them, or an
    // aligned causal unit; 3 = short rows of a power-of-two length (a wave step covers whole rows);
    // 2 = any other unit with row scales (other short rows, rows not made of whole vectors).
    static int unit_class(const WorkUnit& u) {
        if (!(u.flags & kUnitRowScale)) return 0;
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
        uint64_t class_pos[5] = {0, 0, 0, 0, 0};     // streaming kernel of class c: positions [class_pos[c], class_pos[c+1])
        uint64_t class_pairs[4] = {0, 0, 0, 0};
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
        for (int cls = 0; cls < 4; ++cls) {
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
        P.class_pos[4] = P.n_positions;
        return P;
    }
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

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

int g_grid_cap = 0;                                    // test hook: 0 = no cap

// Persistent grid: as many workgroups as the kernel keeps resident on the device, never more
// than there are chunks.
int persistent_grid(uint64_t n_chunks, int resident) {
    uint64_t cap = resident > 0 ? (uint64_t)resident : 1;
    if (g_grid_cap > 0 && (uint64_t)g_grid_cap < cap) cap = (uint64_t)g_grid_cap;
    return (int)(n_chunks < cap ? n_chunks : cap);
}

int sens_grid(uint64_t n_chunks, int n_fmts, int f0, int f1, int rows) {
    static std::mutex mu;
    static int cached[64][2][2][2][4];
    const int dev = device_index();
    int resident;
    if (dev < 0) {
        resident = sens_resident_blocks(n_fmts, f0, f1, rows, device_cus());
    } else {
        std::lock_guard<std::mutex> lock(mu);
        int& slot = cached[dev][n_fmts - 1][f0][f1][rows];
        if (slot == 0) slot = sens_resident_blocks(n_fmts, f0, f1, rows, device_cus());
        resident = slot;
    }
    return persistent_grid(n_chunks, resident);
}

int sens_w_grid(int n_fmts, int f0, int f1, int rows) {
    static std::mutex mu;
    static int cached[64][2][2][2][2];
    const int dev = device_index();
    if (dev < 0) return sens_w_resident_blocks(n_fmts, f0, f1, rows, device_cus());
    std::lock_guard<std::mutex> lock(mu);
    int& slot = cached[dev][n_fmts - 1][f0][f1][rows];
    if (slot == 0) slot = sens_w_resident_blocks(n_fmts, f0, f1, rows, device_cus());
    return slot;
}

int absmax_grid(uint64_t n_chunks) {
    static std::mutex mu;
    static int cached[64];
    const int dev = device_index();
    int resident;
    if (dev < 0) {
        resident = absmax_resident_blocks(device_cus());
    } else {
        std::lock_guard<std::mutex> lock(mu);
        if (cached[dev] == 0) cached[dev] = absmax_resident_blocks(device_cus());
        resident = cached[dev];
    }
    return persistent_grid(n_chunks, resident);
}

// Workspace layout shared by the absmax and the sensitivity calls:
//   [ WorkUnit x n_units | chunk_begin x (n_units + 1) ]   uploaded from the host
//   [ ResolvedUnit x n_units ] [ ChunkRef x n_chunks ]       written by the prepare kernel
//   [ per-wave partials ]                                    written by the streaming kernel
struct WsLayout {
    size_t runits, map, partials, total;
};

WsLayout ws_layout(const WorkTable& t, size_t partial_bytes_per_chunk) {
    WsLayout L;
    L.runits = round_up(t.table_bytes(), 256);
    L.map = L.runits + round_up(t.units.size() * sizeof(ResolvedUnit), 256);
    L.partials = L.map + round_up((size_t)t.n_chunks * sizeof(ChunkRef), 256);
    L.total = L.partials + round_up((size_t)t.n_chunks * partial_bytes_per_chunk, 256);
    return L;
}

// Copies units + chunk_begin to the head of the workspace.
int g_schedule_block = 0;                              // test / tuning hook: 0 = default
constexpr uint32_t kDefaultScheduleBlock = 8;

int g_use_w_kernel = 1;                                // test / tuning hook

uint32_t schedule_block() { return g_schedule_block > 0 ? (uint32_t)g_schedule_block : kDefaultScheduleBlock; }

// Pinned host staging for the descriptor tables.  A table is assembled in a pinned slot and copied
// from there, so the source stays valid until the copy has run whatever the runtime does with
// pageable sources, and the copy is an ordinary asynchronous command of the stream.  Slots are host
// memory only, created on demand (at most kMaxStagingSlots per device), reused once the copy that
// read them has completed (one event per slot) and never freed.
struct StagingSlot {
    void* host = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;
    bool in_flight = false;
};
constexpr size_t kMaxStagingSlots = 32;
std::mutex g_staging_mu;
std::vector<StagingSlot> g_staging[64];                // per device

// A slot of the current device's pool with room for `bytes`, or -1 (then the caller copies from
// pageable memory).  Call with g_staging_mu held.
int staging_acquire(int dev, size_t bytes) {
    std::vector<StagingSlot>& pool = g_staging[dev];
    int busy_fit = -1;
    for (size_t i = 0; i < pool.size(); ++i) {
        if (pool[i].cap < bytes) continue;
        if (!pool[i].in_flight || hipEventQuery(pool[i].done) == hipSuccess) {
            pool[i].in_flight = false;
            return (int)i;
        }
        if (busy_fit < 0) busy_fit = (int)i;
    }
    (void)hipGetLastError();                               // hipEventQuery reports "not ready" as an error
    if (pool.size() < kMaxStagingSlots) {
        StagingSlot slot;
        slot.cap = round_up(bytes < ((size_t)64 << 10) ? ((size_t)64 << 10) : bytes, 4096);
        if (hipHostMalloc(&slot.host, slot.cap, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            return -1;
        }
        if (hipEventCreateWithFlags(&slot.done, hipEventDisableTiming) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipHostFree(slot.host);
            return -1;
        }
        pool.push_back(slot);
        return (int)pool.size() - 1;
    }
    if (busy_fit >= 0 && hipEventSynchronize(pool[busy_fit].done) == hipSuccess) {
        pool[busy_fit].in_flight = false;
        return busy_fit;
    }
    return -1;
}

// Copies `bytes` bytes, written by fill(dst), to device memory `d_dst` on `stream`.
template <class Fill>
amp_status_t staged_upload(void* d_dst, size_t bytes, hipStream_t stream, Fill fill) {
    const int dev = device_index();
    if (dev >= 0) {
        std::lock_guard<std::mutex> lock(g_staging_mu);
        const int slot = staging_acquire(dev, bytes);
        if (slot >= 0) {
            StagingSlot& sl = g_staging[dev][slot];
            fill((uint8_t*)sl.host);
            AMP_HIP(hipMemcpyAsync(d_dst, sl.host, bytes, hipMemcpyHostToDevice, stream));
            AMP_HIP(hipEventRecord(sl.done, stream));
            sl.in_flight = true;
            return AMP_OK;
        }
    }
    // No pinned slot (the pool is full and busy, or pinned memory ran out): copy from pageable
    // memory and wait, so the source outlives the copy.  The only place a device call blocks.
    std::vector<uint8_t> pageable(bytes);
    fill(pageable.data());
    AMP_HIP(hipMemcpyAsync(d_dst, pageable.data(), bytes, hipMemcpyHostToDevice, stream));
    AMP_HIP(hipStreamSynchronize(stream));
    return AMP_OK;
}

// units | chunk_begin | schedule | weight groups -> the head of the workspace
amp_status_t upload(const WorkTable& t, const WorkTable::Plan& plan, void* workspace, hipStream_t stream) {
    const size_t bytes = t.table_bytes();
    return staged_upload(workspace, bytes, stream, [&](uint8_t* blob) {
        std::memset(blob, 0, bytes);
        std::memcpy(blob, t.units.data(), t.units.size() * sizeof(WorkUnit));
        uint8_t* cb = blob + t.units.size() * sizeof(WorkUnit);
        std::memcpy(cb, t.chunk_begin.data(), t.chunk_begin.size() * 4);
        const uint32_t total = (uint32_t)t.n_chunks;
        std::memcpy(cb + t.chunk_begin.size() * 4, &total, 4);
        std::memcpy(blob + t.schedule_offset(), plan.schedule.data(), plan.schedule.size() * sizeof(UnitSchedule));
        if (!plan.wgroups.empty())
            std::memcpy(blob + t.groups_offset(), plan.wgroups.data(), plan.wgroups.size() * sizeof(WGroup));
    });
}

// ---- optional timing of the sensitivity kernel ------------------------------------------------
struct Profile {
    std::vector<hipEvent_t> start, stop;
    std::vector<uint64_t> pairs, bytes;
    int used = 0;
};
Profile g_profile;

// ---- sens: shared by linear and bgemm --------------------------------------------------------

WsLayout sens_layout(const WorkTable& t, int n_fmts) {
    return ws_layout(t, (size_t)kWaves * (n_fmts + 1) * sizeof(float));
}

amp_status_t run_sens(const WorkTable& t, const amp_fp8_format_t* fmts, int n_fmts, float* d_out,
                      void* workspace, size_t workspace_bytes, void* stream_) {
    if (t.units.empty()) return AMP_OK;
    if (!d_out || (uintptr_t)d_out % 4) return AMP_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 256) return AMP_ERR_INVALID_ARG;
    const WsLayout L = sens_layout(t, n_fmts);
    if (workspace_bytes < L.total) return AMP_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)stream_;
    const int f0 = (int)fmts[0], f1 = (int)fmts[n_fmts - 1];
    const WorkTable::Plan plan = t.plan(schedule_block(), g_use_w_kernel != 0);
    amp_status_t st = upload(t, plan, workspace, stream);
    if (st != AMP_OK) return st;
    uint8_t* ws = (uint8_t*)workspace;
    const uint32_t n_units = (uint32_t)t.units.size(), n_chunks = (uint32_t)t.n_chunks;
    const WorkUnit* d_units = (const WorkUnit*)ws;
    const uint32_t* d_cb = (const uint32_t*)(ws + t.units.size() * sizeof(WorkUnit));
    ResolvedUnit* d_runits = (ResolvedUnit*)(ws + L.runits);
    ChunkRef* d_map = (ChunkRef*)(ws + L.map);
    float* d_partials = (float*)(ws + L.partials);
    const UnitSchedule* d_sch = (const UnitSchedule*)(ws + t.schedule_offset());
    const WGroup* d_groups = (const WGroup*)(ws + t.groups_offset());
    AMP_HIP(launch_prepare(d_units, d_cb, d_sch, n_units, n_chunks, n_fmts, d_runits, d_map, stream));
    auto timed_begin = [&](uint64_t pairs, uint64_t bytes) -> hipError_t {
        if (g_profile.used >= (int)g_profile.start.size()) return hipSuccess;
        g_profile.pairs[g_profile.used] = pairs;
        g_profile.bytes[g_profile.used] = bytes;
        return hipEventRecord(g_profile.start[g_profile.used], stream);
    };
    auto timed_end = [&]() -> hipError_t {
        if (g_profile.used >= (int)g_profile.start.size()) return hipSuccess;
        return hipEventRecord(g_profile.stop[g_profile.used++], stream);
    };
    // weight kernel: groups with one scale per tensor, then groups with one per output channel
    size_t g0 = 0;
    for (int v = 0; v < 2; ++v) {
        if (plan.w_items[v] > 0) {
            const int grid = persistent_grid(plan.w_items[v], sens_w_grid(n_fmts, f0, f1, v));
            AMP_HIP(timed_begin(plan.w_pairs[v], plan.w_bytes[v]));
            AMP_HIP(launch_sens_w(d_groups + g0, (uint32_t)plan.w_groups[v], (uint32_t)plan.w_items[v], d_runits,
                                  d_cb, n_fmts, f0, f1, v, d_partials, grid, stream));
            AMP_HIP(timed_end());
        }
        g0 += plan.w_groups[v];
    }
    // streaming kernels, one launch per class of units
    for (int cls = 0; cls < 4; ++cls) {
        const uint64_t n_pos = plan.class_pos[cls + 1] - plan.class_pos[cls];
        if (n_pos == 0) continue;
        const int grid = sens_grid(n_pos, n_fmts, f0, f1, cls);
        AMP_HIP(timed_begin(plan.class_pairs[cls], plan.class_pairs[cls] * 4));
        AMP_HIP(launch_sens(d_runits, d_map + plan.class_pos[cls], (uint32_t)n_pos, n_fmts, f0, f1, cls, d_partials,
                            grid, stream));
        AMP_HIP(timed_end());
    }
    AMP_HIP(launch_sens_finalize(d_runits, d_cb, n_units, n_fmts, d_partials, d_out, stream));
    return AMP_OK;
}

// out_base (in / out): samples of the ops already in the table; this call's sums start there in d_out.
amp_status_t build_linear(const amp_linear_desc_t* ops, int n_ops, int n_fmts, WorkTable* t,
                          uint64_t* out_base = nullptr) {
    if (n_ops < 0 || (n_ops > 0 && !ops)) return AMP_ERR_INVALID_ARG;
    if (n_fmts < 1 || n_fmts > AMP_MAX_FORMATS) return AMP_ERR_BAD_FORMAT;
    uint64_t base = out_base ? *out_base : 0;
    for (int k = 0; k < n_ops; ++k) {
        const amp_linear_desc_t& op = ops[k];
        if (op.R < 0 || op.C < 0 || op.K < 0 || op.tokens < 0) return AMP_ERR_INVALID_ARG;
        if (op.scale_rows & ~(AMP_ROWS_OPERAND0 | AMP_ROWS_OPERAND1)) return AMP_ERR_INVALID_ARG;
        const bool x_rows = (op.scale_rows & AMP_ROWS_OPERAND0) != 0, w_rows = (op.scale_rows & AMP_ROWS_OPERAND1) != 0;
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
            const int64_t xs = x_rows ? r0 * n_fmts : 0;         // the sample's first token in the table
            amp_status_t st = t->add(xn ? op.x + r0 * op.C : op.x, xn ? op.dx + r0 * op.C : op.dx, Lx, 1,
                                     op.x_scale ? op.x_scale + xs : op.x_scale, op.x_inv ? op.x_inv + xs : op.x_inv,
                                     (uint32_t)o, 0u, 0u, x_rows && xn > 0 ? op.C : 0);
            if (st != AMP_OK) return st;
            st = t->add(op.w, wn ? op.dw + (int64_t)r * wn : op.dw, Lw, 1, op.w_scale, op.w_inv, (uint32_t)o + 2,
                        op.R > 1 ? kUnitKeepX : 0u, op.R > 1 ? (uint32_t)k + 1u : 0u, w_rows && wn > 0 ? op.C : 0);
            if (st != AMP_OK) return st;
        }
        base += (uint64_t)op.R;
    }
    if (out_base) *out_base = base;
    return AMP_OK;
}

// Rows of one sample's block for per-row scales: a causal block has batch * rows rows of cols
// entries; a dense block is [n_elems / cols, cols] and must say its row length in cols.
amp_status_t row_geometry(const amp_layout_t& L, int64_t* row_len, int64_t* rows) {
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

amp_status_t build_bgemm(const amp_bgemm_desc_t* ops, int n_ops, int n_fmts, WorkTable* t,
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
        if (op.scale_rows & ~(AMP_ROWS_OPERAND0 | AMP_ROWS_OPERAND1)) return AMP_ERR_INVALID_ARG;
        int64_t len0 = 0, len1 = 0, rows0 = 0, rows1 = 0;    // row length and rows per sample, 0 = one scale
        if (op.scale_rows & AMP_ROWS_OPERAND0) {
            st = row_geometry(op.layout0, &len0, &rows0);
            if (st != AMP_OK) return st;
        }
        if (op.scale_rows & AMP_ROWS_OPERAND1) {
            st = row_geometry(op.layout1, &len1, &rows1);
            if (st != AMP_OK) return st;
        }
        for (int r = 0; r < op.R; ++r) {
            const uint64_t o = (base + r) * (uint64_t)n_fmts * 4;
            if (o + 4 * n_fmts > 0xFFFFFFFFull) return AMP_ERR_TOO_LARGE;
            const int64_t s0 = r * rows0 * n_fmts, s1 = r * rows1 * n_fmts;
            st = t->add(n0 ? op.x0 + r * n0 : op.x0, n0 ? op.dx0 + r * n0 : op.dx0, op.layout0, 1,
                        op.scale0 ? op.scale0 + s0 : op.scale0, op.inv0 ? op.inv0 + s0 : op.inv0, (uint32_t)o, 0u, 0u,
                        n0 > 0 ? len0 : 0);
            if (st != AMP_OK) return st;
            st = t->add(n1 ? op.x1 + r * n1 : op.x1, n1 ? op.dx1 + r * n1 : op.dx1, op.layout1, 1,
                        op.scale1 ? op.scale1 + s1 : op.scale1, op.inv1 ? op.inv1 + s1 : op.inv1, (uint32_t)o + 2, 0u,
                        0u, n1 > 0 ? len1 : 0);
            if (st != AMP_OK) return st;
        }
        base += (uint64_t)op.R;
    }
    if (out_base) *out_base = base;
    return AMP_OK;
}

amp_status_t build_absmax(const amp_tensor_t* tensors, int n_tensors, WorkTable* t) {
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

WsLayout absmax_layout(const WorkTable& t) { return ws_layout(t, (size_t)kWaves * sizeof(uint32_t)); }

// ---- test hook (not part of the public header) ------------------------------------------------
// Replays on the host, thread by thread, the element walk the kernels perform for one unit
// and reports how often each element was touched.  counts has `span` entries (the unit's
// memory span in elements); returns the number of accesses that fell outside [0, span), plus
// the number of "full" vectors that were not 16-byte aligned.
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
    __host__ __device__ void begin_dense(int64_t e0, int le) {
        if (row_len > 0 && cursor_mode) cur.begin(e0, wave_mode ? le - lane * kVec : le, kWG * kVec, row_len);
    }
    __host__ __device__ void set_row(int64_t r) { row = r; have_row = true; }
    // a vector that starts at element s is about to be consumed
    __host__ __device__ void vector_row(int64_t s) {
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
    __host__ __device__ void touch(int64_t e) { if (e < 0 || e >= span) ++bad; else ++counts[e]; }
    template <int U> __host__ __device__ void full(int64_t eu, int le, int64_t stride) {
        for (int k = 0; k < U; ++k) {
            const int64_t s = eu + le + k * stride;
            if ((addr + 2 * (uintptr_t)s) % 16) ++bad;
            vector_row(s);
            for (int j = 0; j < kVec; ++j) touch(s + j);
        }
    }
    template <int U> __host__ __device__ void full_masked(int64_t e, int stride, int count, int tail) {
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
    __host__ __device__ void partial(int64_t e, int jlo, int jhi) {
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

amp_status_t amp_absmax_workspace_bytes(const amp_tensor_t* tensors, int n_tensors, size_t* bytes) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    WorkTable t;
    amp_status_t st = build_absmax(tensors, n_tensors, &t);
    if (st != AMP_OK) return st;
    *bytes = absmax_layout(t).total;
    return AMP_OK;
}

amp_status_t amp_absmax_scale(const amp_tensor_t* tensors, int n_tensors, const amp_fp8_format_t* fmts,
                              int n_fmts, float* d_amax, float* d_scale, float* d_inv,
                              uint32_t* d_flags, void* workspace, size_t workspace_bytes,
                              void* stream_) {
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_absmax(tensors, n_tensors, &t);
    if (st != AMP_OK) return st;
    if (n_tensors == 0) return AMP_OK;
    if (!d_amax || !d_scale || !d_inv || !d_flags) return AMP_ERR_INVALID_ARG;
    if (((uintptr_t)d_amax | (uintptr_t)d_scale | (uintptr_t)d_inv | (uintptr_t)d_flags) % 4) return AMP_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 256) return AMP_ERR_INVALID_ARG;
    const WsLayout L = absmax_layout(t);
    if (workspace_bytes < L.total) return AMP_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)stream_;
    const WorkTable::Plan plan = t.plan(schedule_block(), false);
    st = upload(t, plan, workspace, stream);
    if (st != AMP_OK) return st;
    uint8_t* ws = (uint8_t*)workspace;
    const uint32_t n_units = (uint32_t)t.units.size(), n_chunks = (uint32_t)t.n_chunks;
    const WorkUnit* d_units = (const WorkUnit*)ws;
    const uint32_t* d_cb = (const uint32_t*)(ws + t.units.size() * sizeof(WorkUnit));
    ResolvedUnit* d_runits = (ResolvedUnit*)(ws + L.runits);
    ChunkRef* d_map = (ChunkRef*)(ws + L.map);
    uint32_t* d_partial_max = (uint32_t*)(ws + L.partials);
    const UnitSchedule* d_sch = (const UnitSchedule*)(ws + t.schedule_offset());
    AMP_HIP(launch_prepare(d_units, d_cb, d_sch, n_units, n_chunks, 0, d_runits, d_map, stream));
    if (n_chunks > 0)
        AMP_HIP(launch_absmax(d_runits, d_map, n_chunks, d_partial_max, absmax_grid(n_chunks), stream));
    AMP_HIP(launch_absmax_finalize(d_cb, d_partial_max, n_tensors, n_fmts, (int)fmts[0],
                                   (int)fmts[n_fmts - 1], d_amax, d_scale, d_inv, d_flags, stream));
    return AMP_OK;
}

// ---- absmax and scales per row ----------------------------------------------------------------
namespace {
struct RowPlan {
    std::vector<RowTensor> tensors;
    uint64_t n_items = 0, n_rows = 0;
};

amp_status_t build_absmax_rows(const amp_tensor_t* tensors, int n_tensors, RowPlan* P) {
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
}  // namespace

amp_status_t amp_absmax_rows_workspace_bytes(const amp_tensor_t* tensors, int n_tensors, size_t* bytes,
                                             int64_t* n_rows) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    RowPlan P;
    amp_status_t st = build_absmax_rows(tensors, n_tensors, &P);
    if (st != AMP_OK) return st;
    *bytes = round_up(P.tensors.size() * sizeof(RowTensor), 256);
    if (n_rows) *n_rows = (int64_t)P.n_rows;
    return AMP_OK;
}

amp_status_t amp_absmax_scale_rows(const amp_tensor_t* tensors, int n_tensors, const amp_fp8_format_t* fmts,
                                   int n_fmts, float* d_amax, float* d_scale, float* d_inv, uint32_t* d_flags,
                                   void* workspace, size_t workspace_bytes, void* stream_) {
    amp_status_t st = check_fmts(fmts, n_fmts, true);
    if (st != AMP_OK) return st;
    RowPlan P;
    st = build_absmax_rows(tensors, n_tensors, &P);
    if (st != AMP_OK) return st;
    if (n_tensors == 0) return AMP_OK;
    if (!d_flags || (uintptr_t)d_flags % 4) return AMP_ERR_INVALID_ARG;
    if (P.n_rows > 0 && (!d_amax || !d_scale || !d_inv)) return AMP_ERR_INVALID_ARG;
    if (((uintptr_t)d_amax | (uintptr_t)d_scale | (uintptr_t)d_inv) % 4) return AMP_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 256) return AMP_ERR_INVALID_ARG;
    const size_t bytes = P.tensors.size() * sizeof(RowTensor);
    if (workspace_bytes < round_up(bytes, 256)) return AMP_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = (hipStream_t)stream_;
    st = staged_upload(workspace, bytes, stream,
                       [&](uint8_t* dst) { std::memcpy(dst, P.tensors.data(), bytes); });
    if (st != AMP_OK) return st;
    const uint64_t waves = P.n_items;
    const uint64_t wgs = (waves + kWaves - 1) / kWaves;
    static std::mutex mu;
    static int resident[64];
    int res;
    {
        std::lock_guard<std::mutex> lock(mu);
        const int dev = device_index();
        int& slot = resident[dev < 0 ? 0 : dev];
        if (slot == 0) slot = absmax_rows_resident_blocks(device_cus());
        res = slot;
    }
    const int grid = persistent_grid(wgs > 0 ? wgs : 1, res);
    AMP_HIP(launch_absmax_rows((const RowTensor*)workspace, (uint32_t)P.tensors.size(), (uint32_t)P.n_items,
                               n_fmts, (int)fmts[0], (int)fmts[n_fmts - 1], d_amax, d_scale, d_inv, d_flags,
                               grid, stream));
    return AMP_OK;
}

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

amp_status_t amp_sens_linear_workspace_bytes(const amp_linear_desc_t* ops, int n_ops, int n_fmts, size_t* bytes) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    WorkTable t;
    amp_status_t st = build_linear(ops, n_ops, n_fmts, &t);
    if (st != AMP_OK) return st;
    *bytes = sens_layout(t, n_fmts).total;
    return AMP_OK;
}

amp_status_t amp_sens_linear(const amp_linear_desc_t* ops, int n_ops, const amp_fp8_format_t* fmts,
                             int n_fmts, float* d_out, void* workspace, size_t workspace_bytes,
                             void* stream) {
    amp_status_t st = check_fmts(fmts, n_fmts);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_linear(ops, n_ops, n_fmts, &t);
    if (st != AMP_OK) return st;
    return run_sens(t, fmts, n_fmts, d_out, workspace, workspace_bytes, stream);
}

amp_status_t amp_sens_bgemm_workspace_bytes(const amp_bgemm_desc_t* ops, int n_ops, int n_fmts, size_t* bytes) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    WorkTable t;
    amp_status_t st = build_bgemm(ops, n_ops, n_fmts, &t);
    if (st != AMP_OK) return st;
    *bytes = sens_layout(t, n_fmts).total;
    return AMP_OK;
}

amp_status_t amp_sens_bgemm(const amp_bgemm_desc_t* ops, int n_ops, const amp_fp8_format_t* fmts,
                            int n_fmts, float* d_out, void* workspace, size_t workspace_bytes,
                            void* stream) {
    amp_status_t st = check_fmts(fmts, n_fmts);
    if (st != AMP_OK) return st;
    WorkTable t;
    st = build_bgemm(ops, n_ops, n_fmts, &t);
    if (st != AMP_OK) return st;
    return run_sens(t, fmts, n_fmts, d_out, workspace, workspace_bytes, stream);
}

amp_status_t amp_sens_block_workspace_bytes(const amp_linear_desc_t* linears, int n_linears,
                                            const amp_bgemm_desc_t* bgemms, int n_bgemms, int n_fmts,
                                            size_t* bytes) {
    if (!bytes) return AMP_ERR_INVALID_ARG;
    WorkTable t;
    uint64_t base = 0;
    amp_status_t st = build_linear(linears, n_linears, n_fmts, &t, &base);
    if (st != AMP_OK) return st;
    st = build_bgemm(bgemms, n_bgemms, n_fmts, &t, &base);
    if (st != AMP_OK) return st;
    *bytes = sens_layout(t, n_fmts).total;
    return AMP_OK;
}

amp_status_t amp_sens_block(const amp_linear_desc_t* linears, int n_linears, const amp_bgemm_desc_t* bgemms,
                            int n_bgemms, const amp_fp8_format_t* fmts, int n_fmts, float* d_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
    amp_status_t st = check_fmts(fmts, n_fmts);
    if (st != AMP_OK) return st;
    WorkTable t;
    uint64_t base = 0;
    st = build_linear(linears, n_linears, n_fmts, &t, &base);
    if (st != AMP_OK) return st;
    st = build_bgemm(bgemms, n_bgemms, n_fmts, &t, &base);
    if (st != AMP_OK) return st;
    return run_sens(t, fmts, n_fmts, d_out, workspace, workspace_bytes, stream);
}

amp_status_t amp_profile_enable(int max_launches) {
    if (max_launches < 0) return AMP_ERR_INVALID_ARG;
    for (hipEvent_t e : g_profile.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_profile.stop) (void)hipEventDestroy(e);
    g_profile.start.clear();
    g_profile.stop.clear();
    g_profile.pairs.assign((size_t)max_launches, 0);
    g_profile.bytes.assign((size_t)max_launches, 0);
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

amp_status_t amp_profile_read(float* ms, uint64_t* pairs, uint64_t* bytes, int capacity, int* n_launches) {
    if (!n_launches || capacity < 0 || (capacity > 0 && !ms)) return AMP_ERR_INVALID_ARG;
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

int amp_version(void) { return 100; }

// Test hook: checks on the host that the schedule of a linear call is a permutation of its
// chunks; returns the number of positions that are out of range, hit twice or never hit, and
// reports the number of chunks and how many units are interleaved with others.
int64_t ampsens_debug_check_linear_schedule(const amp_linear_desc_t* ops, int n_ops, int n_fmts,
                                            uint64_t* n_chunks_out, uint64_t* interleaved_units) {
    WorkTable t;
    if (build_linear(ops, n_ops, n_fmts, &t) != AMP_OK) return -1;
    const WorkTable::Plan plan = t.plan(schedule_block(), g_use_w_kernel != 0);
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
    if (n_chunks_out) *n_chunks_out = t.n_chunks;
    if (interleaved_units) *interleaved_units = inter;
    return bad;
}

// Test / tuning hook: 0 sends weights through the streaming kernel like everything else.
void ampsens_debug_set_w_kernel(int on) { g_use_w_kernel = on; }

// Test / tuning hook: chunks of one member that sit next to each other in the schedule (0 = default).
void ampsens_debug_set_schedule_block(int block) { g_schedule_block = block; }

// Test hook: cap the persistent grid (0 = default) to show that results do not depend on it.
void ampsens_debug_set_grid_cap(int cap) { g_grid_cap = cap; }

// row_len != 0 also replays the row tracking of a unit with one scale per row and counts every
// vector whose tracked row differs from (element index / row_len), or that straddles two rows.
int64_t ampsens_debug_replay_unit_rows(uint64_t x_addr, uint64_t dx_addr, const amp_layout_t* layout,
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

int64_t ampsens_debug_replay_unit(uint64_t x_addr, uint64_t dx_addr, const amp_layout_t* layout,
                                  int64_t batch_mul, int32_t* counts, int64_t span, uint64_t* n_chunks_out) {
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
