// lagom_model_fill, lagom_model_calibrate: the contention wave model (Eq. 4-6) filled from a
// profiler sweep.  The paper measures x_j and names theta and V(NC, C) without saying how they are
// obtained; here theta is Eq. 6 solved for the standalone run and V the measured co-run rate.
// Host only.  Compiled with floating-point contraction off; expression order is part of the contract.
#include <algorithm>
#include <cmath>
#include <vector>
#include "common.h"

namespace {

int check_desc(const lagom_fill_desc* d) {
    if (!d) return lagom::fail(LAGOM_EINVAL, "null description");
    if (d->lambda < 1 || !(d->bw_peak > 0.0)) return lagom::fail(LAGOM_EINVAL, "lambda and peak bandwidth must be positive");
    if (d->mu < 1 || d->tb < 1 || !(d->d_bytes >= 0.0)) return lagom::fail(LAGOM_EINVAL, "bad computation geometry");
    if (d->ncomp < 1 || d->ncomp > LAGOM_MAX_LAUNCHES) return lagom::fail(LAGOM_EINVAL, "ncomp=%d outside 1..%d", d->ncomp, LAGOM_MAX_LAUNCHES);
    if (d->ncomm < 1 || d->ncomm > LAGOM_MAX_COMMS || !d->comm_bytes) return lagom::fail(LAGOM_EINVAL, "ncomm=%d outside 1..%d or null byte counts", d->ncomm, LAGOM_MAX_COMMS);
    if (!(d->v_cap_frac >= 0.0 && d->v_cap_frac < 1.0)) return lagom::fail(LAGOM_EINVAL, "v_cap_frac must lie in [0, 1)");
    return LAGOM_OK;
}

double median_of(std::vector<double> v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n & 1 ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
}

// theta of Eq. 6 from the standalone time: g0 = ceil(mu / (lambda*TB)) waves (Eq. 5 with NC = 0), each
// theta + lambda*TB*D/B long.
double fit_theta(double t_alone, const lagom_fill_desc* d) {
    const int64_t cap = (int64_t)d->lambda * d->tb;
    const int64_t g0 = (d->mu + cap - 1) / cap;
    const double theta = t_alone / (double)g0 - ((double)cap * d->d_bytes) / d->bw_peak;
    return theta > 0.0 ? theta : 0.0;
}

int fill_tables(const lagom_sweep_point* pts, int npts, const lagom_fill_desc* d, lagom_table_entry* entries, lagom_comm_table* tables) {
    double total = 0.0;
    for (int j = 0; j < d->ncomm; ++j) {
        if (!(d->comm_bytes[j] >= 0.0)) return lagom::fail(LAGOM_EINVAL, "communication %d: negative byte count", j);
        total = total + d->comm_bytes[j];
    }
    if (!(total > 0.0)) return lagom::fail(LAGOM_EINVAL, "the communications move no bytes");
    const double cap = d->v_cap_frac > 0.0 ? d->v_cap_frac : 0.99;
    const double vmax = cap * d->bw_peak;
    for (int j = 0; j < d->ncomm; ++j) {
        const double share = d->comm_bytes[j] / total;
        lagom_table_entry* e = entries + (int64_t)j * npts;
        for (int p = 0; p < npts; ++p) {
            e[p].cfg = pts[p].cfg;
            e[p].x_us = share * pts[p].comm_corun_us;
            e[p].v = pts[p].v_corun < vmax ? pts[p].v_corun : vmax;
        }
        tables[j].entries = e;
        tables[j].n = npts;
    }
    return LAGOM_OK;
}

}  // namespace

extern "C" int lagom_model_fill(const lagom_sweep_point* pts, int npts, const uint8_t* held_out, const lagom_fill_desc* d,
                                lagom_table_entry* entries, lagom_comm_table* tables, lagom_comp_model* comps, double* t_alone_us) {
    if (!pts || npts < 1 || !entries || !tables || !comps) return lagom::fail(LAGOM_EINVAL, "null argument or no sweep points");
    if (int rc = check_desc(d)) return rc;
    std::vector<double> alone;
    for (int p = 0; p < npts; ++p) {
        if (!(pts[p].comm_corun_us >= 0.0) || !(pts[p].comp_alone_us >= 0.0) || !(pts[p].v_corun >= 0.0))
            return lagom::fail(LAGOM_EINVAL, "sweep point %d holds a negative or non-finite time", p);
        if (!held_out || !held_out[p]) alone.push_back(pts[p].comp_alone_us);
    }
    if (alone.empty()) return lagom::fail(LAGOM_EINVAL, "every sweep point is held out");
    const double t_alone = median_of(alone) / (double)d->ncomp;
    const double theta = fit_theta(t_alone, d);
    for (int i = 0; i < d->ncomp; ++i) comps[i] = lagom_comp_model{d->mu, d->tb, d->d_bytes, theta};
    if (t_alone_us) *t_alone_us = t_alone;
    return fill_tables(pts, npts, d, entries, tables);
}

extern "C" int lagom_model_calibrate(const lagom_sweep_point* pts, int npts, const uint8_t* held_out, const lagom_fill_desc* d,
                                     const int32_t* comp_after_comm, const int32_t* comm_after_comp,
                                     const double* sigmas, int nsigma,
                                     const double* rhos, int nrho, lagom_penalty* penalty_out, int penalty_capacity,
                                     lagom_calibration* out) {
    if (!out || !sigmas || nsigma < 1) return lagom::fail(LAGOM_EINVAL, "null output or no candidate sigma");
    if (nrho < 0 || (nrho > 0 && (!rhos || !penalty_out))) return lagom::fail(LAGOM_EINVAL, "candidate penalties without an array for them or for the result");
    if (!pts || npts < 1) return lagom::fail(LAGOM_EINVAL, "no sweep points");
    if (int rc = check_desc(d)) return rc;
    std::vector<lagom_table_entry> entries((size_t)d->ncomm * npts);
    std::vector<lagom_comm_table> tables(d->ncomm);
    std::vector<lagom_comp_model> comps(d->ncomp);
    if (int rc = lagom_model_fill(pts, npts, held_out, d, entries.data(), tables.data(), comps.data(), nullptr)) return rc;
    lagom_model m{};
    m.lambda = d->lambda; m.bw_peak = d->bw_peak;
    m.comps = comps.data(); m.ncomp = d->ncomp;
    m.tables = tables.data(); m.ncomm = d->ncomm;
    m.comp_after_comm = comp_after_comm; m.comm_after_comp = comm_after_comp;
    std::vector<lagom_cfg> cfgs(d->ncomm);
    // mean and maximum of |Y_model - Y_measured| / Y_measured over the points with held_out == which
    // (and, for only_nt > 0, with that thread count)
    auto errors = [&](int which, double* mean, double* worst, int* count, int only_nt = 0) -> int {
        double total = 0.0, w = 0.0;
        int n = 0;
        for (int p = 0; p < npts; ++p) {
            const int h = held_out && held_out[p] ? 1 : 0;
            if (h != which) continue;
            if (only_nt > 0 && pts[p].cfg.nt != only_nt) continue;
            if (!(pts[p].comp_corun_us > 0.0)) return lagom::fail(LAGOM_EINVAL, "sweep point %d: co-run computation time must be positive", p);
            std::fill(cfgs.begin(), cfgs.end(), pts[p].cfg);
            lagom_pred pr{};
            if (int rc = lagom_cost_model(&m, cfgs.data(), d->ncomm, &pr)) return rc;
            const double e = std::fabs(pr.Y_us - pts[p].comp_corun_us) / pts[p].comp_corun_us;
            total = total + e;
            w = e > w ? e : w;
            ++n;
        }
        *mean = n ? total / (double)n : 0.0;
        *worst = w;
        *count = n;
        return LAGOM_OK;
    };
    bool have = false;
    lagom_calibration best{};
    for (int s = 0; s < nsigma; ++s) {
        if (!(sigmas[s] >= 0.0 && sigmas[s] <= 1.0)) return lagom::fail(LAGOM_EINVAL, "candidate sigma %d outside [0, 1]", s);
        m.corun_share = sigmas[s];
        double mean, worst; int n;
        if (int rc = errors(0, &mean, &worst, &n)) return rc;
        if (!have || mean < best.fit_mean) { best.sigma = sigmas[s]; best.fit_mean = mean; best.fit_max = worst; best.n_fit = n; have = true; }
    }
    m.corun_share = best.sigma;
    if (nrho > 0) {
        // the thread counts among the fitted points, ascending
        std::vector<int> nts;
        for (int p = 0; p < npts; ++p)
            if (!(held_out && held_out[p])) nts.push_back(pts[p].cfg.nt);
        std::sort(nts.begin(), nts.end());
        nts.erase(std::unique(nts.begin(), nts.end()), nts.end());
        if ((int)nts.size() > penalty_capacity) return lagom::fail(LAGOM_EINVAL, "%d thread counts, room for %d penalties", (int)nts.size(), penalty_capacity);
        m.penalty = penalty_out;
        m.npenalty = 0;
        for (int nt : nts) {
            const int slot = m.npenalty;
            m.npenalty = slot + 1;
            penalty_out[slot].nt = nt;
            bool have_rho = false;
            double best_mean = 0.0, best_rho = 0.0;
            for (int r = 0; r < nrho; ++r) {
                if (!(rhos[r] >= 0.0)) return lagom::fail(LAGOM_EINVAL, "candidate rho %d is negative", r);
                penalty_out[slot].rho = rhos[r];
                double mean, worst; int n;
                if (int rc = errors(0, &mean, &worst, &n, nt)) return rc;
                if (!have_rho || mean < best_mean) { best_mean = mean; best_rho = rhos[r]; have_rho = true; }
            }
            penalty_out[slot].rho = best_rho;
        }
        best.npenalty = m.npenalty;
        if (int rc = errors(0, &best.fit_mean, &best.fit_max, &best.n_fit)) return rc;
    }
    if (int rc = errors(1, &best.held_mean, &best.held_max, &best.n_held)) return rc;
    best.theta_us = comps[0].theta_us;
    *out = best;
    return LAGOM_OK;
}
