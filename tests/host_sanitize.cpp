// Host-only stress driver for the cost model and the tuner, meant to be built with
// -fsanitize=address,undefined (see tests/test_host_sanitizers.py).  It checks no numbers against
// the oracle (the Python tests do that); it only has to run clean under the sanitizers and to see
// every error path return its code instead of crashing.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "lagom.h"

struct Tab { std::vector<std::vector<lagom_table_entry>> e; std::vector<lagom_comm_table> t; };

static int profile_cb(void* user, const lagom_cfg* cfgs, int n, double* x, double* Y) {
    int* calls = static_cast<int*>(user);
    ++*calls;
    if (*calls == 1000003) return 1;
    double y = 50.0;
    for (int j = 0; j < n; ++j) { x[j] = 300.0 / cfgs[j].nc + 1e-6 * (double)cfgs[j].chunk_bytes / cfgs[j].nt + 0.3 * cfgs[j].nc; y += 2.0 * cfgs[j].nc; }
    *Y = y;
    return 0;
}
static int failing_cb(void*, const lagom_cfg*, int, double*, double*) { return 7; }

int main() {
    std::mt19937 rng(12345);
    int bad = 0;
    for (int rep = 0; rep < 400; ++rep) {
        const int N = 1 + rng() % 6, M = 1 + rng() % 5;
        std::vector<int32_t> nc = {1, 2, 4, 8, 16, 32};
        std::vector<int32_t> nt = {128, 256, 512};
        std::vector<int64_t> ch = {32768, 65536, 131072, 262144};
        nc.resize(1 + rng() % nc.size()); nt.resize(1 + rng() % nt.size()); ch.resize(1 + rng() % ch.size());
        Tab tab; tab.e.resize(N); tab.t.resize(N);
        for (int j = 0; j < N; ++j) {
            for (int32_t a : nc) for (int32_t b : nt) for (int64_t c : ch)
                tab.e[j].push_back(lagom_table_entry{lagom_cfg{a, b, c}, 10.0 + (rng() % 1000) / 3.0, (double)(rng() % 7000000)});
            tab.t[j] = lagom_comm_table{tab.e[j].data(), (int32_t)tab.e[j].size()};
        }
        std::vector<lagom_comp_model> comps(M);
        for (auto& c : comps) c = lagom_comp_model{(int64_t)(rng() % 3000), (int32_t)(1 + rng() % 2), (double)(rng() % 5000000), (rng() % 100) / 4.0};
        std::vector<int32_t> cac(M), cap(N);
        for (int i = 0; i < M; ++i) cac[i] = (int)(rng() % (std::min(i + 1, N) + 1)) - 1;
        for (int j = 0; j < N; ++j) cap[j] = j == 0 ? -1 : (int)(rng() % (std::min(j, M) + 1)) - 1;
        const bool dep = rep & 1;
        lagom_model m{256, 8.0e6, comps.data(), M, tab.t.data(), N, dep ? cac.data() : nullptr, dep ? cap.data() : nullptr, (rep % 3 == 0) ? 0.0 : 0.125 * (double)(rep % 9)};
        std::vector<lagom_cfg> cfgs(N);
        for (auto& c : cfgs) c = lagom_cfg{nc[rng() % nc.size()], nt[rng() % nt.size()], ch[rng() % ch.size()]};
        std::vector<double> x(N), y(M);
        std::vector<int32_t> g((size_t)M * (N + 1));
        lagom_pred p{0, 0, 0, x.data(), y.data(), g.data()};
        if (lagom_cost_model(&m, cfgs.data(), N, &p) != LAGOM_OK) { std::printf("cost model failed: %s\n", lagom_last_error()); ++bad; }
        if (!(p.Z_us >= p.X_us - 1e-9) || !std::isfinite(p.Y_us)) ++bad;
        lagom_pred q{0, 0, 0, nullptr, nullptr, nullptr};
        if (lagom_cost_model(&m, cfgs.data(), N, &q) != LAGOM_OK) ++bad;
        // error paths
        lagom_cfg missing = cfgs[0]; missing.nc = 3;
        std::vector<lagom_cfg> wrong = cfgs; wrong[0] = missing;
        if (lagom_cost_model(&m, wrong.data(), N, &p) != LAGOM_EINVAL) ++bad;
        if (lagom_cost_model(&m, cfgs.data(), N + 1, &p) != LAGOM_EINVAL) ++bad;
        if (lagom_cost_model(nullptr, cfgs.data(), N, &p) != LAGOM_EINVAL) ++bad;

        std::vector<lagom_tune_space> sp(N, lagom_tune_space{nc.data(), (int32_t)nc.size(), nt.data(), (int32_t)nt.size(), ch.data(), (int32_t)ch.size()});
        std::vector<lagom_cfg> out(N);
        std::vector<lagom_trace_step> steps(8 * N + 4);
        std::vector<int32_t> lev(N);
        for (int mode : {LAGOM_PRIORITY, LAGOM_COMM_OPTIMAL, LAGOM_EXHAUSTIVE, LAGOM_HIDE_COMM, LAGOM_EXHAUSTIVE_HIDE, LAGOM_PRIORITY_FREE}) {
            if ((mode == LAGOM_EXHAUSTIVE || mode == LAGOM_EXHAUSTIVE_HIDE) && N > 3) continue;
            int calls = 0;
            lagom_trace tr{steps.data(), (int32_t)steps.size(), 0, 0, 0, 0, 0, lev.data()};
            if (lagom_tune(sp.data(), N, profile_cb, &calls, mode, out.data(), &tr) != LAGOM_OK) { std::printf("tune mode %d failed: %s\n", mode, lagom_last_error()); ++bad; }
            if (tr.calls != calls) ++bad;
            if (lagom_tune(sp.data(), N, profile_cb, &calls, mode, out.data(), nullptr) != LAGOM_OK) ++bad;
            // model-driven profile through the library's own callback (only ladder levels are in the table when grids are full products)
            if (lagom_tune(sp.data(), N, lagom_model_profile, &m, mode, out.data(), &tr) != LAGOM_OK) ++bad;
        }
        lagom_trace tiny{steps.data(), 1, 0, 0, 0, 0, 0, nullptr};
        int calls = 0;
        const int rc = lagom_tune(sp.data(), N, profile_cb, &calls, LAGOM_PRIORITY, out.data(), &tiny);
        if (rc != LAGOM_OK && rc != LAGOM_EINVAL) ++bad;                    // a too-small trace is an error, never an overrun
        if (lagom_tune(sp.data(), N, failing_cb, nullptr, LAGOM_PRIORITY, out.data(), nullptr) != LAGOM_ECALLBACK) ++bad;
        if (lagom_tune(sp.data(), 0, profile_cb, &calls, LAGOM_PRIORITY, out.data(), nullptr) != LAGOM_EINVAL) ++bad;
        if (lagom_tune(sp.data(), N, profile_cb, &calls, 9, out.data(), nullptr) != LAGOM_EINVAL) ++bad;

        // model fill, calibration and the ladder helper on a synthetic sweep over the same grids
        std::vector<lagom_sweep_point> pts;
        for (int32_t a : nc) for (int32_t b : nt) for (int64_t c : ch)
            pts.push_back(lagom_sweep_point{lagom_cfg{a, b, c}, 5.0 + rng() % 300, 5.0 + rng() % 300, 100.0 + rng() % 500, 100.0 + rng() % 700,
                                            100.0 + rng() % 900, (double)(rng() % 9000000), (double)(rng() % 9000000)});
        const int P = (int)pts.size();
        std::vector<uint8_t> held(P);
        for (int i = 0; i < P; ++i) held[i] = i & 1;
        std::vector<double> nbytes(N);
        for (auto& b : nbytes) b = 1.0 + rng() % 100000000;
        lagom_fill_desc fd{256, 8.0e6, (int64_t)(1 + rng() % 3000), (int32_t)(1 + rng() % 2), (double)(rng() % 5000000), M, N, nbytes.data(), 0.0};
        std::vector<lagom_table_entry> fe((size_t)N * P);
        std::vector<lagom_comm_table> ft(N);
        std::vector<lagom_comp_model> fc(M);
        double t_alone = 0.0;
        if (lagom_model_fill(pts.data(), P, held.data(), &fd, fe.data(), ft.data(), fc.data(), &t_alone) != LAGOM_OK) { std::printf("fill failed: %s\n", lagom_last_error()); ++bad; }
        if (lagom_model_fill(pts.data(), P, nullptr, &fd, fe.data(), ft.data(), fc.data(), nullptr) != LAGOM_OK) ++bad;
        const lagom_penalty fixed_pen[2] = {{nt[0], 0.05}, {nt.back(), 0.2}};
        lagom_model fm{256, 8.0e6, fc.data(), M, ft.data(), N, nullptr, nullptr, 0.25, fixed_pen, 2};
        if (lagom_tune(sp.data(), N, lagom_model_profile, &fm, LAGOM_HIDE_COMM, out.data(), nullptr) != LAGOM_OK) ++bad;
        const double sig[3] = {0.0, 0.5, 1.0};
        lagom_calibration cal{};
        if (lagom_model_calibrate(pts.data(), P, held.data(), &fd, dep ? cac.data() : nullptr, dep ? cap.data() : nullptr, sig, 3, nullptr, 0, nullptr, 0, &cal) != LAGOM_OK) { std::printf("calibrate failed: %s\n", lagom_last_error()); ++bad; }
        if (cal.n_fit + cal.n_held != P) ++bad;
        const double rho[3] = {0.0, 0.1, 0.3};
        std::vector<lagom_penalty> pen(nt.size());
        if (lagom_model_calibrate(pts.data(), P, held.data(), &fd, dep ? cac.data() : nullptr, dep ? cap.data() : nullptr, sig, 3, rho, 3, pen.data(), (int)pen.size(), &cal) != LAGOM_OK) { std::printf("calibrate with penalties failed: %s\n", lagom_last_error()); ++bad; }
        if (cal.npenalty < 1 || cal.npenalty > (int)nt.size()) ++bad;
        if (nt.size() > 1 && lagom_model_calibrate(pts.data(), P, nullptr, &fd, nullptr, nullptr, sig, 3, rho, 3, pen.data(), 1, &cal) != LAGOM_EINVAL) ++bad;
        if (lagom_model_calibrate(pts.data(), P, held.data(), &fd, nullptr, nullptr, sig, 0, nullptr, 0, nullptr, 0, &cal) != LAGOM_EINVAL) ++bad;
        std::vector<uint8_t> all_held(P, 1);
        if (lagom_model_fill(pts.data(), P, all_held.data(), &fd, fe.data(), ft.data(), fc.data(), nullptr) != LAGOM_EINVAL) ++bad;
        if (lagom_model_fill(pts.data(), 0, nullptr, &fd, fe.data(), ft.data(), fc.data(), nullptr) != LAGOM_EINVAL) ++bad;
        std::vector<int64_t> lc(ch.size());
        int32_t ln = 0;
        for (int kind : {LAGOM_LADDER_FULL, LAGOM_LADDER_CUT, LAGOM_LADDER_FIXED_CHUNK}) {
            if (lagom_ladder_chunks(ch.data(), (int)ch.size(), nc.back(), nt[0], (int64_t)(rng() % 4000000), kind, pts.data(), P, lc.data(), &ln) != LAGOM_OK) ++bad;
            if (ln < 1 || ln > (int32_t)ch.size()) ++bad;
        }
        if (lagom_ladder_chunks(ch.data(), (int)ch.size(), 77, nt[0], 100, LAGOM_LADDER_FIXED_CHUNK, pts.data(), P, lc.data(), &ln) != LAGOM_EINVAL) ++bad;
    }
    std::printf("host sanitize driver: %d problems\n", bad);
    return bad ? 1 : 0;
}
