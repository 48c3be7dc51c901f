// Host-side driver for the sanitizer test: calls every entry point of the library that does its work
// on the host (validation, table building, schedule planning, the walk replay, partition, selection)
// on seeded random inputs.  Built by tests/test_host_sanitizers.py with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code; the launchers are stubbed, no GPU is touched.
#include "../include/ampsens.h"
#include "../paper_2505_13060_amd/csrc/internal.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

namespace ampsens {      // the kernels' launchers: never reached from the calls below
int sens_resident_blocks(int, int, int, int, int cus) { return 8 * cus; }
int absmax_resident_blocks(int cus) { return 8 * cus; }
int absmax_rows_resident_blocks(int cus) { return 8 * cus; }
int sens_w_resident_blocks(int, int, int, int, int cus) { return 4 * cus; }
hipError_t launch_table_write(const void*, size_t, void*, hipStream_t) { std::abort(); }
hipError_t launch_table_runs(const TableRun*, size_t, void*, size_t, hipStream_t) { std::abort(); }
hipError_t launch_table_literals(const TableLiteral*, size_t, void*, size_t, hipStream_t) { std::abort(); }
hipError_t launch_small_setup(const void*, size_t, void*, size_t, size_t, uint32_t, uint32_t, ResolvedUnit*, ChunkRef*,
                              int, hipStream_t) { std::abort(); }
hipError_t launch_prepare(const WorkUnit*, const uint32_t*, const UnitSchedule*, uint32_t, uint32_t,
                          ResolvedUnit*, ChunkRef*, hipStream_t) { std::abort(); }
hipError_t launch_resolve(const WorkUnit*, uint32_t, int, ResolvedUnit*, hipStream_t) { std::abort(); }
hipError_t launch_absmax(const ResolvedUnit*, const ChunkRef*, uint32_t, uint32_t*, int, hipStream_t) { std::abort(); }
hipError_t launch_absmax_finalize(const uint32_t*, const uint32_t*, int, int, int, int, float*, float*, float*,
                                  uint32_t*, hipStream_t) { std::abort(); }
hipError_t launch_fake_quant(const uint16_t*, int64_t, float, float, int, uint8_t*, float*, int, hipStream_t) { std::abort(); }
hipError_t launch_sens(const ResolvedUnit*, const ChunkRef*, uint32_t, int, int, int, int, float*, int, hipStream_t) { std::abort(); }
hipError_t launch_sens_w(const WGroup*, uint32_t, uint32_t, const ResolvedUnit*, const uint32_t*, int, int, int, int,
                         float*, int, hipStream_t) { std::abort(); }
hipError_t launch_absmax_rows(const RowTensor*, uint32_t, uint32_t, int, int, int, float*, float*, float*, uint32_t*,
                              int, hipStream_t) { std::abort(); }
hipError_t launch_sens_finalize(const ResolvedUnit*, const uint32_t*, uint32_t, int, const float*, float*,
                                hipStream_t) { std::abort(); }
}  // namespace ampsens

extern "C" {
// tests/host_hooks.cpp, compiled along
int64_t hooks_check_linear_schedule(const amp_linear_desc_t*, int, int, int, int, uint64_t*, uint64_t*);
int64_t hooks_replay_unit(uint64_t, uint64_t, const amp_layout_t*, int64_t, int32_t*, int64_t, uint64_t*);
int64_t hooks_replay_unit_rows(uint64_t, uint64_t, const amp_layout_t*, int64_t, int64_t, int32_t*, int64_t,
                               uint64_t*);
}

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("CHECK failed at line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main() {
    std::mt19937_64 rng(20250513);
    auto uni = [&](int64_t lo, int64_t hi) { return (int64_t)(lo + rng() % (uint64_t)(hi - lo + 1)); };
    const uint16_t* fake = (const uint16_t*)(uintptr_t)0x10000000;       // never dereferenced on the host
    const float* fakef = (const float*)(uintptr_t)0x20000000;

    // table building, workspace sizes and schedules of random linear / BGEMM calls
    for (int it = 0; it < 200; ++it) {
        const int n_ops = (int)uni(0, 6), nf = (int)uni(1, 2);
        std::vector<amp_linear_desc_t> lin(n_ops);
        std::vector<std::vector<int64_t>> offs(n_ops);
        for (int k = 0; k < n_ops; ++k) {
            amp_linear_desc_t& d = lin[k];
            std::memset(&d, 0, sizeof(d));
            d.x = d.dx = d.w = fake;
            d.dw = fake + uni(0, 9);
            d.C = uni(1, 700); d.K = uni(1, 300); d.R = (int32_t)uni(0, 19);
            d.x_scale = d.x_inv = d.w_scale = d.w_inv = fakef;
            d.scale_rows = (int32_t)uni(0, 3);
            if (uni(0, 1)) {
                offs[k].assign((size_t)d.R + 1, 0);
                for (int r = 0; r < d.R; ++r) offs[k][r + 1] = offs[k][r] + uni(0, 40);
                d.sample_row_offsets = offs[k].data();
            } else {
                d.tokens = uni(0, 64);
            }
        }
        size_t bytes = 0;
        const amp_status_t st = amp_sens_linear_workspace_bytes(lin.data(), n_ops, nf, &bytes);
        CHECK(st == AMP_OK);
        uint64_t chunks = 0, inter = 0;
        CHECK(hooks_check_linear_schedule(lin.data(), n_ops, nf, (int)uni(0, 9), (int)uni(0, 1), &chunks, &inter) == 0);
        std::vector<amp_bgemm_desc_t> bg((size_t)uni(0, 4));
        for (amp_bgemm_desc_t& b : bg) {
            std::memset(&b, 0, sizeof(b));
            b.x0 = b.dx0 = b.x1 = b.dx1 = fake;
            b.scale0 = b.inv0 = b.scale1 = b.inv1 = fakef;
            b.R = (int32_t)uni(0, 5);
            b.layout0.n_elems = uni(0, 50) * 16; b.layout0.cols = 16;
            b.layout1.causal = 1; b.layout1.batch = uni(0, 3); b.layout1.rows = uni(0, 70); b.layout1.cols = uni(0, 70);
            b.scale_rows = (int32_t)uni(0, 3);
        }
        size_t bytes2 = 0;
        CHECK(amp_sens_block_workspace_bytes(lin.data(), n_ops, bg.data(), (int)bg.size(), nf, &bytes2) == AMP_OK);
        CHECK(bytes2 >= bytes || bg.empty());
        std::vector<amp_tensor_t> ts(bg.size());
        for (size_t i = 0; i < bg.size(); ++i) { ts[i].data = fake; ts[i].layout = bg[i].layout1; ts[i].n_samples = bg[i].R; }
        size_t b3 = 0; int64_t rows = 0;
        CHECK(amp_absmax_workspace_bytes(ts.data(), (int)ts.size(), &b3) == AMP_OK);
        CHECK(amp_absmax_rows_workspace_bytes(ts.data(), (int)ts.size(), &b3, &rows) == AMP_OK);
    }

    // plans: every error path of the set-up calls answers on the host, and a plan that was never set up does not run
    {
        amp_plan_t plan;
        std::memset(&plan, 0xAB, sizeof(plan));
        CHECK(amp_run(&plan, nullptr) == AMP_ERR_INVALID_ARG);
        CHECK(amp_run(nullptr, nullptr) == AMP_ERR_INVALID_ARG);
        const amp_fp8_format_t fm[2] = {AMP_FP8_E4M3, AMP_FP8_E5M2};
        CHECK(amp_sens_block_setup(nullptr, 0, nullptr, 0, fm, 2, nullptr, nullptr, 0, 0u, nullptr, nullptr) == AMP_ERR_INVALID_ARG);
        CHECK(amp_sens_block_setup(nullptr, 0, nullptr, 0, fm, 2, nullptr, nullptr, 0, 2u, nullptr, &plan) == AMP_ERR_INVALID_ARG);
        CHECK(amp_run(&plan, nullptr) == AMP_ERR_INVALID_ARG);
        CHECK(amp_sens_block_setup(nullptr, 0, nullptr, 0, fm, 2, nullptr, nullptr, 0, 0u, nullptr, &plan) == AMP_OK);
        CHECK(amp_run(&plan, nullptr) == AMP_OK);                       // nothing to do, nothing launched
        CHECK(amp_plan_limit_grid(&plan, 7) == AMP_OK && amp_plan_limit_grid(&plan, -1) == AMP_ERR_INVALID_ARG);
        CHECK(amp_absmax_scale_setup(nullptr, 0, fm, 2, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, &plan) == AMP_OK);
        CHECK(amp_run(&plan, nullptr) == AMP_OK);
        CHECK(amp_absmax_scale_rows_setup(nullptr, 0, fm, 3, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, &plan) == AMP_ERR_BAD_FORMAT);
        CHECK(amp_run(&plan, nullptr) == AMP_ERR_INVALID_ARG);
    }

    // the walk replay: every element of a unit exactly once, no access outside it
    for (int it = 0; it < 60; ++it) {
        amp_layout_t L;
        std::memset(&L, 0, sizeof(L));
        int64_t span, row_len = 0;
        const bool causal = uni(0, 2) == 0;
        if (causal) {
            L.causal = 1; L.batch = uni(1, 3); L.rows = uni(1, 80); L.cols = uni(1, 12) * 8;
            span = L.batch * L.rows * L.cols;
            if (uni(0, 1)) row_len = L.cols;
        } else {
            const int64_t rl = uni(1, 40) * (uni(0, 1) ? 8 : 3);
            L.n_elems = rl * uni(1, 3000);
            span = L.n_elems;
            if (uni(0, 1)) row_len = rl;
        }
        const uint64_t addr = 0x40000000ull + 2 * (uint64_t)uni(0, 7);
        std::vector<int32_t> counts((size_t)span, 0);
        uint64_t nch = 0;
        const int64_t bad = row_len ? hooks_replay_unit_rows(addr, addr, &L, 1, row_len, counts.data(), span, &nch)
                                    : hooks_replay_unit(addr, addr, &L, 1, counts.data(), span, &nch);
        CHECK(bad == 0);
        if (!causal)
            for (int64_t e = 0; e < span; ++e) if (counts[(size_t)e] != 1) { CHECK(counts[(size_t)e] == 1); break; }
    }

    // selection (eq. (ip)), ordered baselines, group tables, partition
    for (int it = 0; it < 300; ++it) {
        const int J = (int)uni(0, 40);
        std::vector<int32_t> nc(J), choice(J), choice2(J);
        std::vector<double> gain, mse;
        std::uniform_real_distribution<double> u01(0.0, 1.0);
        double dmax = 0;
        for (int j = 0; j < J; ++j) {
            nc[j] = (int32_t)uni(1, 9);
            for (int p = 0; p < nc[j]; ++p) {
                gain.push_back(p == 0 ? 0.0 : u01(rng) * 10);
                mse.push_back(p == 0 ? 0.0 : u01(rng));
            }
            dmax += 1.0;
        }
        const double budget = u01(rng) * dmax * 0.3;
        double tg = 0, td = 0, tg2 = 0, td2 = 0;
        CHECK(amp_select_subgraphs(J, nc.data(), gain.data(), mse.data(), budget, choice.data(), &tg, &td) == AMP_OK);
        CHECK(td <= budget + 1e-9);
        CHECK(amp_select_ordered(J, nc.data(), gain.data(), mse.data(), budget, nullptr, choice2.data(), &tg2, &td2) == AMP_OK);
        CHECK(tg2 <= tg + 1e-9 && td2 <= budget + 1e-9);
        CHECK(amp_select_subgraphs(J, nc.data(), gain.data(), mse.data(), -1.0, choice.data(), &tg, &td) == AMP_ERR_INFEASIBLE);
    }
    for (int it = 0; it < 100; ++it) {
        const int n_layers = (int)uni(0, 6), F = (int)uni(1, 3);
        size_t ncol = 1;
        for (int l = 0; l < n_layers; ++l) ncol *= (size_t)F;
        std::vector<double> lm((size_t)n_layers * F + 1, 0.5), lg((size_t)n_layers * F + 1, 2.0), d(ncol), c(ncol);
        CHECK(amp_group_tables(n_layers, F, lm.data(), lg.data(), d.data(), c.data()) == AMP_OK);
        CHECK(d[ncol - 1] == 0.5 * n_layers && c[0] == 2.0 * n_layers);
    }
    for (int it = 0; it < 200; ++it) {
        // a random layered DAG with one source and one sink
        const int layers = (int)uni(1, 7);
        std::vector<std::vector<int32_t>> lv((size_t)layers + 2);
        int n = 0;
        lv[0].push_back(n++);
        for (int l = 1; l <= layers; ++l) for (int k = (int)uni(1, 3); k > 0; --k) lv[(size_t)l].push_back(n++);
        lv[(size_t)layers + 1].push_back(n++);
        std::vector<int32_t> src, dst;
        for (size_t l = 0; l + 1 < lv.size(); ++l) {
            for (int32_t a : lv[l]) { src.push_back(a); dst.push_back(lv[l + 1][(size_t)uni(0, (int64_t)lv[l + 1].size() - 1)]); }
            for (int32_t b : lv[l + 1]) { src.push_back(lv[l][(size_t)uni(0, (int64_t)lv[l].size() - 1)]); dst.push_back(b); }
        }
        std::vector<uint8_t> q((size_t)n);
        for (uint8_t& v : q) v = (uint8_t)uni(0, 1);
        std::vector<int32_t> group((size_t)n, -7);
        int32_t ng = -1;
        const amp_status_t st = amp_partition_sequential(n, (int)src.size(), src.data(), dst.data(), q.data(), group.data(), &ng);
        CHECK(st == AMP_OK);
        for (int v = 0; v < n; ++v) CHECK(group[(size_t)v] >= -1 && group[(size_t)v] < ng);
    }
    std::printf("host_sanitize: %d failures\n", failures);
    return failures ? 1 : 0;
}
