// Priority-based parameter search (metric H of Eq. 7, Alg. 1 driving Alg. 2) and the
// exhaustive search over the same ladder space.  Host only; measuring is the callback's.
// Compiled with floating-point contraction off.
#include <array>
#include <cmath>
#include <limits>
#include <vector>
#include "common.h"

namespace {

constexpr double kHInit = 0.01;  // Alg. 1: every H starts at 0.01

struct Ladder {
    const lagom_tune_space* sp;
    int K;
    lagom_cfg cfg(int level) const {
        auto at = [level](int n) { return level < n - 1 ? level : n - 1; };
        return lagom_cfg{sp->nc[at(sp->n_nc)], sp->nt[at(sp->n_nt)], sp->chunk[at(sp->n_chunk)]};
    }
};

template <class T>
bool ascending(const T* g, int n) {
    if (!g || n < 1) return false;
    for (int i = 1; i < n; ++i)
        if (!(g[i] > g[i - 1])) return false;
    return true;
}

// Alg. 2's parameter increase on the ladder: the lowest level above `level` at which every
// parameter has reached min(p * (1 + lr), p_max); one level when no lr is known yet.
int next_level(const Ladder& L, int level, bool has_lr, double lr) {
    const int top = L.K - 1;
    if (level >= top) return top;
    if (!has_lr) return level + 1;
    const lagom_cfg cur = L.cfg(level);
    const double tgt[3] = {(double)cur.nc * (1.0 + lr), (double)cur.nt * (1.0 + lr), (double)cur.chunk_bytes * (1.0 + lr)};
    for (int cand = level + 1; cand <= top; ++cand) {
        const lagom_cfg c = L.cfg(cand);
        const bool ok_nc = (double)c.nc >= tgt[0] || c.nc == L.sp->nc[L.sp->n_nc - 1];
        const bool ok_nt = (double)c.nt >= tgt[1] || c.nt == L.sp->nt[L.sp->n_nt - 1];
        const bool ok_c = (double)c.chunk_bytes >= tgt[2] || c.chunk_bytes == L.sp->chunk[L.sp->n_chunk - 1];
        if (ok_nc && ok_nt && ok_c) return cand;
    }
    return top;
}

struct Measurement {
    std::vector<double> x;
    double X = 0, Y = 0, Z = 0;
};

// One ProfileTime call; X is the sum of the x_j in index order.
int measure(lagom_profile_fn profile, void* user, const std::vector<Ladder>& L, const std::vector<int>& lev,
            std::vector<lagom_cfg>& scratch, Measurement* m) {
    const int N = (int)L.size();
    for (int j = 0; j < N; ++j) scratch[j] = L[j].cfg(lev[j]);
    m->x.assign(N, 0.0);
    double Y = 0.0;
    if (profile(user, scratch.data(), N, m->x.data(), &Y) != 0) return LAGOM_ECALLBACK;
    double X = 0.0;
    for (int j = 0; j < N; ++j) {
        if (!(m->x[j] >= 0.0) || !std::isfinite(m->x[j])) return LAGOM_ECALLBACK;
        X = X + m->x[j];
    }
    if (!(Y >= 0.0) || !std::isfinite(Y)) return LAGOM_ECALLBACK;
    m->X = X; m->Y = Y; m->Z = X > Y ? X : Y;
    return LAGOM_OK;
}

void emit(const std::vector<Ladder>& L, const std::vector<int>& lev, const Measurement* m, int calls,
          lagom_cfg* out_cfgs, lagom_trace* tr) {
    for (size_t j = 0; j < L.size(); ++j) out_cfgs[j] = L[j].cfg(lev[j]);
    if (!tr) return;
    tr->calls = calls;
    if (m) { tr->X = m->X; tr->Y = m->Y; tr->Z = m->Z; }
    if (tr->levels) for (size_t j = 0; j < L.size(); ++j) tr->levels[j] = lev[j];
}

int push(lagom_trace* tr, const lagom_trace_step& s) {
    if (!tr || !tr->steps) return LAGOM_OK;
    if (tr->n >= tr->capacity) return lagom::fail(LAGOM_EINVAL, "trace capacity %d too small", tr->capacity);
    tr->steps[tr->n++] = s;
    return LAGOM_OK;
}

// free_steps: a hidden step that also lowered Y (H of Eq. 7 negative: it cost the computation nothing) does not end the
// communication; it is accepted like any other step.
// hide = false: Alg. 1 driving Alg. 2.  hide = true: the same walk for the computation-bound objective (least Y
// subject to X <= Y): it ends, for every communication, at the first vector with X <= Y, which is kept.
int priority(const std::vector<Ladder>& L, lagom_profile_fn profile, void* user, lagom_cfg* out_cfgs, lagom_trace* tr, bool hide, bool free_steps) {
    const int N = (int)L.size();
    const double nan = std::numeric_limits<double>::quiet_NaN();
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<int> lev(N, 0);
    std::vector<double> H(N, kHInit), lr(N, nan);
    std::vector<char> has_lr(N, 0), done(N, 0);
    std::vector<lagom_cfg> scratch(N);
    int ndone = 0;
    for (int j = 0; j < N; ++j)
        if (L[j].K == 1) { done[j] = 1; ++ndone; }

    Measurement cur;
    int calls = 0;
    int rc = measure(profile, user, L, lev, scratch, &cur);
    if (rc) { emit(L, lev, nullptr, calls, out_cfgs, tr); return lagom::fail(rc, "baseline profile failed"); }
    calls = 1;
    if (hide ? cur.X <= cur.Y : cur.X < cur.Y) {   // optimality condition 1: minimum resources already hide X
        for (int j = 0; j < N; ++j) done[j] = 1;
        ndone = N;
    }
    if ((rc = push(tr, lagom_trace_step{-1, 0, 0, 1, ndone == N, nan, nan, cur.X, cur.Y, cur.Z, kHInit, nan}))) return rc;

    Measurement trial;
    std::vector<int> tl(N);
    while (ndone < N) {
        int j = -1;
        for (int i = 0; i < N; ++i)            // Alg. 1: smallest H among the unfinished, ties to the lowest index
            if (!done[i] && (j < 0 || H[i] < H[j])) j = i;
        const int to = next_level(L[j], lev[j], has_lr[j], lr[j]);
        tl = lev; tl[j] = to;
        rc = measure(profile, user, L, tl, scratch, &trial);
        if (rc) { emit(L, lev, &cur, calls, out_cfgs, tr); return lagom::fail(rc, "profile call %d failed", calls + 1); }
        ++calls;
        bool accepted;
        if (trial.x[j] - cur.x[j] > 0.0) {     // Alg. 2: the communication itself got slower
            done[j] = 1; accepted = false;
        } else if (hide && trial.X <= trial.Y) {   // hidden: keep it; nothing else needs raising
            accepted = true;
            for (int i = 0; i < N; ++i) done[i] = 1;
            ndone = N - 1;                          // the step's own bookkeeping below adds the last one
        } else if (!hide && trial.X < trial.Y && !(free_steps && trial.Y < cur.Y)) {   // Alg. 2: all communication is hidden
            done[j] = 1; accepted = trial.Z < cur.Z;
        } else {
            accepted = true;
            const double den = cur.x[j] - trial.x[j];
            H[j] = den == 0.0 ? inf : (trial.Y - cur.Y) / den;      // Eq. 7
            lr[j] = trial.x[j] == 0.0 ? inf : den / trial.x[j];
            has_lr[j] = 1;
            if (to == L[j].K - 1) done[j] = 1;
        }
        if (done[j]) ++ndone;
        if ((rc = push(tr, lagom_trace_step{j, lev[j], to, accepted ? 1 : 0, done[j] ? 1 : 0, cur.x[j], trial.x[j],
                                            trial.X, trial.Y, trial.Z, H[j], has_lr[j] ? lr[j] : nan}))) return rc;
        if (accepted) { lev = tl; std::swap(cur, trial); }
    }
    emit(L, lev, &cur, calls, out_cfgs, tr);
    return LAGOM_OK;
}

// hide = true: among the vectors with X <= Y the smallest Y wins; the smallest Z only if there is none.
int exhaustive(const std::vector<Ladder>& L, lagom_profile_fn profile, void* user, lagom_cfg* out_cfgs, lagom_trace* tr, bool hide) {
    const int N = (int)L.size();
    double total = 1.0;
    for (const Ladder& l : L) total *= l.K;
    if (total > 1048576.0) return lagom::fail(LAGOM_EINVAL, "exhaustive search over %.0f vectors refused", total);
    std::vector<int> lev(N, 0), best_lev(N, 0), hid_lev(N, 0);
    std::vector<lagom_cfg> scratch(N);
    Measurement m, best, hid;
    long best_sum = 0, hid_sum = 0;
    bool have = false, have_hid = false;
    int calls = 0;
    for (;;) {                                  // lexicographic order, last index fastest
        int rc = measure(profile, user, L, lev, scratch, &m);
        if (rc) { emit(L, best_lev, have ? &best : nullptr, calls, out_cfgs, tr); return lagom::fail(rc, "profile call %d failed", calls + 1); }
        ++calls;
        long sum = 0;
        for (int v : lev) sum += v;
        // visiting order is lexicographic, so "strictly better" keeps the lexicographically smallest on full ties
        if (!have || m.Z < best.Z || (m.Z == best.Z && sum < best_sum)) { best = m; best_lev = lev; best_sum = sum; have = true; }
        if (hide && m.X <= m.Y && (!have_hid || m.Y < hid.Y || (m.Y == hid.Y && sum < hid_sum))) { hid = m; hid_lev = lev; hid_sum = sum; have_hid = true; }
        int d = N - 1;
        while (d >= 0 && ++lev[d] == L[d].K) lev[d--] = 0;
        if (d < 0) break;
    }
    if (have_hid) emit(L, hid_lev, &hid, calls, out_cfgs, tr);
    else emit(L, best_lev, &best, calls, out_cfgs, tr);
    return LAGOM_OK;
}


// Communication-bound regime (Eq. 2): Z is the sum of the x_j and separates per communication, so
// each x_j is minimised on its own over the full (NC, NT, C) product by coordinate descent with
// measured feedback.  Communications in index order, the others staying where they are; for one
// communication start at the minimum of every grid and sweep the coordinates NC, C, NT: one grid
// step up while x_j falls strictly, and if the first step up did not help, down while x_j falls
// strictly; repeat the sweeps until one changes nothing.  Every probe is one profile call.
int comm_optimal(const std::vector<Ladder>& L, lagom_profile_fn profile, void* user, lagom_cfg* out_cfgs, lagom_trace* tr) {
    const int N = (int)L.size();
    std::vector<std::array<int, 3>> idx(N, std::array<int, 3>{0, 0, 0});
    std::vector<lagom_cfg> cfgs(N);
    std::vector<double> x(N), x2(N);
    double Y = 0.0, Y2 = 0.0;
    int calls = 0;
    auto size_of = [&](int j, int p) { return p == 0 ? L[j].sp->n_nc : (p == 1 ? L[j].sp->n_nt : L[j].sp->n_chunk); };
    auto fill = [&]() {
        for (int j = 0; j < N; ++j)
            cfgs[j] = lagom_cfg{L[j].sp->nc[idx[j][0]], L[j].sp->nt[idx[j][1]], L[j].sp->chunk[idx[j][2]]};
    };
    auto finish = [&](int rc) {
        fill();
        for (int j = 0; j < N; ++j) out_cfgs[j] = cfgs[j];
        if (tr) {
            tr->calls = calls;
            double X = 0.0;
            for (int j = 0; j < N; ++j) X = X + x[j];
            tr->X = X; tr->Y = Y; tr->Z = X > Y ? X : Y;
            if (tr->levels) for (int j = 0; j < N; ++j) tr->levels[j] = idx[j][0];
        }
        return rc;
    };
    auto probe = [&](std::vector<double>& xs, double* y) -> int {
        fill();
        if (profile(user, cfgs.data(), N, xs.data(), y) != 0) return LAGOM_ECALLBACK;
        for (int j = 0; j < N; ++j)
            if (!(xs[j] >= 0.0) || !std::isfinite(xs[j])) return LAGOM_ECALLBACK;
        if (!(*y >= 0.0) || !std::isfinite(*y)) return LAGOM_ECALLBACK;
        ++calls;
        return LAGOM_OK;
    };
    if (int rc = probe(x, &Y)) return finish(lagom::fail(rc, "baseline profile failed"));
    static const int order[3] = {0, 2, 1};   // NC, C, NT
    for (int j = 0; j < N; ++j) {
        double best = x[j];
        bool changed = true;
        while (changed) {
            changed = false;
            for (int p : order) {
                bool moved_up = false;
                while (idx[j][p] + 1 < size_of(j, p)) {
                    idx[j][p] += 1;
                    if (int rc = probe(x2, &Y2)) { idx[j][p] -= 1; return finish(lagom::fail(rc, "profile call %d failed", calls + 1)); }
                    if (x2[j] < best) { best = x2[j]; x = x2; Y = Y2; moved_up = true; changed = true; }
                    else { idx[j][p] -= 1; break; }
                }
                if (moved_up) continue;
                while (idx[j][p] - 1 >= 0) {
                    idx[j][p] -= 1;
                    if (int rc = probe(x2, &Y2)) { idx[j][p] += 1; return finish(lagom::fail(rc, "profile call %d failed", calls + 1)); }
                    if (x2[j] < best) { best = x2[j]; x = x2; Y = Y2; changed = true; }
                    else { idx[j][p] += 1; break; }
                }
            }
        }
    }
    return finish(LAGOM_OK);
}

}  // namespace

extern "C" int lagom_tune(const lagom_tune_space* spaces, int ncomm, lagom_profile_fn profile, void* user,
                          int mode, lagom_cfg* out_cfgs, lagom_trace* trace) {
    if (!spaces || !profile || !out_cfgs) return lagom::fail(LAGOM_EINVAL, "null argument");
    if (ncomm < 1 || ncomm > LAGOM_MAX_COMMS) return lagom::fail(LAGOM_EINVAL, "ncomm=%d outside 1..%d", ncomm, LAGOM_MAX_COMMS);
    if (mode < LAGOM_PRIORITY || mode > LAGOM_PRIORITY_FREE) return lagom::fail(LAGOM_EINVAL, "unknown mode %d", mode);
    std::vector<Ladder> L(ncomm);
    for (int j = 0; j < ncomm; ++j) {
        const lagom_tune_space& s = spaces[j];
        if (!ascending(s.nc, s.n_nc) || !ascending(s.nt, s.n_nt) || !ascending(s.chunk, s.n_chunk))
            return lagom::fail(LAGOM_EINVAL, "communication %d: grids must be non-empty and strictly ascending", j);
        int K = s.n_nc > s.n_nt ? s.n_nc : s.n_nt;
        L[j] = Ladder{&s, K > s.n_chunk ? K : s.n_chunk};
    }
    if (trace) {
        trace->n = 0; trace->calls = 0;
        if (trace->steps && trace->capacity < 0) return lagom::fail(LAGOM_EINVAL, "negative trace capacity");
    }
    if (mode == LAGOM_PRIORITY || mode == LAGOM_HIDE_COMM || mode == LAGOM_PRIORITY_FREE)
        return priority(L, profile, user, out_cfgs, trace, mode == LAGOM_HIDE_COMM, mode == LAGOM_PRIORITY_FREE);
    if (mode == LAGOM_EXHAUSTIVE || mode == LAGOM_EXHAUSTIVE_HIDE) return exhaustive(L, profile, user, out_cfgs, trace, mode == LAGOM_EXHAUSTIVE_HIDE);
    return comm_optimal(L, profile, user, out_cfgs, trace);
}

extern "C" int lagom_ladder_chunks(const int64_t* chunk_grid, int n_chunk, int32_t nc_max, int32_t nt_ref, int64_t bytes_per_source,
                                   int kind, const lagom_sweep_point* pts, int npts, int64_t* out_chunks, int32_t* out_n) {
    if (!out_chunks || !out_n) return lagom::fail(LAGOM_EINVAL, "null output");
    if (!ascending(chunk_grid, n_chunk)) return lagom::fail(LAGOM_EINVAL, "the chunk grid must be non-empty and strictly ascending");
    if (nc_max < 1 || bytes_per_source < 0) return lagom::fail(LAGOM_EINVAL, "nc_max >= 1 and bytes_per_source >= 0 required");
    int n = 0;
    if (kind == LAGOM_LADDER_FULL) {
        for (int i = 0; i < n_chunk; ++i) out_chunks[n++] = chunk_grid[i];
    } else if (kind == LAGOM_LADDER_CUT) {
        for (int i = 0; i < n_chunk; ++i)
            if (chunk_grid[i] * (int64_t)nc_max <= bytes_per_source) out_chunks[n++] = chunk_grid[i];
        if (n == 0) out_chunks[n++] = chunk_grid[0];
    } else if (kind == LAGOM_LADDER_FIXED_CHUNK) {
        if (!pts || npts < 1) return lagom::fail(LAGOM_EINVAL, "a fixed-chunk ladder needs sweep points");
        bool have = false;
        double best = 0.0;
        for (int i = 0; i < n_chunk; ++i)
            for (int p = 0; p < npts; ++p) {
                const lagom_sweep_point& s = pts[p];
                if (s.cfg.nc != nc_max || s.cfg.nt != nt_ref || s.cfg.chunk_bytes != chunk_grid[i]) continue;
                if (!have || s.comm_alone_us < best) { best = s.comm_alone_us; out_chunks[0] = chunk_grid[i]; have = true; }
                break;
            }
        if (!have) return lagom::fail(LAGOM_EINVAL, "no sweep point at nc=%d, nt=%d", nc_max, nt_ref);
        n = 1;
    } else {
        return lagom::fail(LAGOM_EINVAL, "unknown ladder kind %d", kind);
    }
    *out_n = n;
    return LAGOM_OK;
}
