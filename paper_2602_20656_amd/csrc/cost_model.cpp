// Unified overlap cost model (Eq. 1) over the contention wave model (Eq. 4-6, Table 1).
// Host only.  Compiled with floating-point contraction off: every product and sum below
// is rounded separately, in the order written.
#include <cmath>
#include <vector>
#include "common.h"

namespace {

struct CommPoint { double x, v; int nc; double pf; };   // pf = 1 + rho of the communication's thread count

int lookup(const lagom_comm_table& t, const lagom_cfg& c, int j, CommPoint* out) {
    if (t.n < 0 || (t.n > 0 && !t.entries)) return lagom::fail(LAGOM_EINVAL, "communication %d: bad table", j);
    for (int e = 0; e < t.n; ++e) {
        const lagom_table_entry& te = t.entries[e];
        if (te.cfg.nc == c.nc && te.cfg.nt == c.nt && te.cfg.chunk_bytes == c.chunk_bytes) {
            out->x = te.x_us; out->v = te.v; out->nc = c.nc;
            return LAGOM_OK;
        }
    }
    return lagom::fail(LAGOM_EINVAL, "communication %d: configuration (nc=%d, nt=%d, chunk=%lld) is not in its table",
                       j, c.nc, c.nt, (long long)c.chunk_bytes);
}

// Workgroups in flight under a communication of NC channels (Eq. 5's divisor): (lambda - NC) * TB, or
// with a share sigma of every channel's compute unit left to the computation
// floor((lambda - NC * (1 - sigma)) * TB).
inline int64_t in_flight(int lambda, int nc, int tb, double sigma) {
    if (sigma == 0.0) return (int64_t)(lambda - nc) * tb;
    const double avail = (double)lambda - (double)nc * (1.0 - sigma);
    return (int64_t)std::floor(avail * (double)tb);
}

// Eq. 6 with cap = (lambda - NC) * TB workgroups in flight.
inline double wave_time(double theta, int64_t cap, double d_bytes, double bw_peak, double v) {
    return theta + ((double)cap * d_bytes) / (bw_peak - v);
}

}  // namespace

extern "C" int lagom_cost_model(const lagom_model* m, const lagom_cfg* cfgs, int ncomm, lagom_pred* out) {
    if (!m || !out || (ncomm > 0 && !cfgs)) return lagom::fail(LAGOM_EINVAL, "null argument");
    if (ncomm != m->ncomm || ncomm < 0 || ncomm > LAGOM_MAX_COMMS)
        return lagom::fail(LAGOM_EINVAL, "ncomm=%d does not match the model's %d (max %d)", ncomm, m->ncomm, LAGOM_MAX_COMMS);
    if (m->ncomp < 0 || (m->ncomp > 0 && !m->comps) || (ncomm > 0 && !m->tables))
        return lagom::fail(LAGOM_EINVAL, "bad model arrays");
    if (m->lambda < 1 || !(m->bw_peak > 0.0)) return lagom::fail(LAGOM_EINVAL, "lambda and peak bandwidth must be positive");
    if (!(m->corun_share >= 0.0 && m->corun_share <= 1.0)) return lagom::fail(LAGOM_EINVAL, "corun_share must lie in [0, 1]");

    if (m->npenalty < 0 || (m->npenalty > 0 && !m->penalty)) return lagom::fail(LAGOM_EINVAL, "bad penalty array");
    for (int e = 0; e < m->npenalty; ++e)
        if (!(m->penalty[e].rho >= 0.0)) return lagom::fail(LAGOM_EINVAL, "penalty %d: rho must be non-negative", e);
    const int N = ncomm;
    std::vector<CommPoint> c(N);
    for (int j = 0; j < N; ++j) {
        if (int rc = lookup(m->tables[j], cfgs[j], j, &c[j])) return rc;
        c[j].pf = 1.0;
        for (int e = 0; e < m->npenalty; ++e)
            if (m->penalty[e].nt == cfgs[j].nt) { c[j].pf = 1.0 + m->penalty[e].rho; break; }
        if (c[j].nc < 1 || c[j].nc >= m->lambda)
            return lagom::fail(LAGOM_EINVAL, "communication %d: NC=%d outside 1..lambda-1", j, c[j].nc);
        if (!(c[j].v >= 0.0 && c[j].v < m->bw_peak))
            return lagom::fail(LAGOM_EINVAL, "communication %d: V outside [0, peak bandwidth)", j);
        if (!(c[j].x >= 0.0) || !std::isfinite(c[j].x))
            return lagom::fail(LAGOM_EINVAL, "communication %d: x must be finite and non-negative", j);
    }
    for (int i = 0; i < m->ncomp; ++i) {
        const lagom_comp_model& cp = m->comps[i];
        if (cp.mu < 0 || cp.tb < 1 || !(cp.d_bytes >= 0.0) || !std::isfinite(cp.theta_us))
            return lagom::fail(LAGOM_EINVAL, "computation %d: bad description", i);
    }
    const int M = m->ncomp;
    double X = 0.0, Y = 0.0, Z = 0.0;
    for (int j = 0; j < N; ++j) X = X + c[j].x;
    std::vector<double> f(N + 1);
    std::vector<int32_t> g(N + 1);

    if (!m->comp_after_comm && !m->comm_after_comp) {
        // communication j is active on [T[j], T[j+1])
        std::vector<double> T(N + 1, 0.0);
        for (int j = 0; j < N; ++j) T[j + 1] = T[j] + c[j].x;
        double t0 = 0.0;
        for (int i = 0; i < M; ++i) {
            const lagom_comp_model& cp = m->comps[i];
            for (int s = 0; s <= N; ++s) { f[s] = 0.0; g[s] = 0; }
            int64_t rem = cp.mu;
            double t = t0, y = 0.0;
            while (rem > 0) {
                int slot = N;
                for (int j = 0; j < N; ++j)
                    if (t < T[j + 1]) { slot = j; break; }
                int64_t cap;
                if (slot < N) {
                    cap = in_flight(m->lambda, c[slot].nc, cp.tb, m->corun_share);
                    f[slot] = wave_time(cp.theta_us, cap, cp.d_bytes, m->bw_peak, c[slot].v);
                    if (c[slot].pf != 1.0) f[slot] = f[slot] * c[slot].pf;
                } else {
                    cap = (int64_t)m->lambda * cp.tb;
                    f[slot] = wave_time(cp.theta_us, cap, cp.d_bytes, m->bw_peak, 0.0);
                }
                g[slot] += 1;
                rem -= rem < cap ? rem : cap;
                y = 0.0;
                for (int s = 0; s <= N; ++s)            // Eq. 4, terms in ascending j
                    if (g[s] > 0) y = y + f[s] * (double)g[s];
                t = t0 + y;
            }
            if (out->y_us) out->y_us[i] = y;
            if (out->g) for (int s = 0; s <= N; ++s) out->g[(int64_t)i * (N + 1) + s] = g[s];
            t0 = t0 + y;
            Y = Y + y;
        }
        Z = T[N] > Y ? T[N] : Y;
    } else {
        // dependent chains: both streams advance together; a communication is placed as soon as its
        // predecessor on the stream and the computation it waits for have ended, a computation is
        // stepped wave by wave against the communications placed so far
        std::vector<int> cac(M, -1), cap_dep(N, -1);
        for (int i = 0; i < M && m->comp_after_comm; ++i) cac[i] = m->comp_after_comm[i];
        for (int j = 0; j < N && m->comm_after_comp; ++j) cap_dep[j] = m->comm_after_comp[j];
        for (int i = 0; i < M; ++i) if (cac[i] < -1 || cac[i] >= N) return lagom::fail(LAGOM_EINVAL, "computation %d waits for communication %d", i, cac[i]);
        for (int j = 0; j < N; ++j) if (cap_dep[j] < -1 || cap_dep[j] >= M) return lagom::fail(LAGOM_EINVAL, "communication %d waits for computation %d", j, cap_dep[j]);
        std::vector<double> cs(N, 0.0), ce(N, 0.0), pe(M, 0.0), ys(M, 0.0);
        std::vector<char> c_known(N, 0), p_known(M, 0);
        std::vector<int32_t> gall((size_t)M * (N + 1), 0);
        int jn = 0, in = 0;
        double tc = 0.0, ty = 0.0, t0 = 0.0;
        bool running = false;
        int64_t rem = 0;
        while (jn < N || in < M) {
            bool progressed = false;
            while (jn < N && (cap_dep[jn] < 0 || p_known[cap_dep[jn]])) {
                const int dep = cap_dep[jn];
                const double start = dep < 0 ? tc : (tc > pe[dep] ? tc : pe[dep]);
                cs[jn] = start; ce[jn] = start + c[jn].x; c_known[jn] = 1;
                tc = ce[jn];
                ++jn;
                progressed = true;
            }
            if (in < M) {
                const lagom_comp_model& cp = m->comps[in];
                if (!running) {
                    const int dep = cac[in];
                    if (dep < 0 || c_known[dep]) {
                        t0 = dep < 0 ? ty : (ty > ce[dep] ? ty : ce[dep]);
                        running = true; rem = cp.mu;
                        for (int s = 0; s <= N; ++s) f[s] = 0.0;
                        progressed = true;
                    }
                }
                if (running) {
                    int32_t* gi = &gall[(size_t)in * (N + 1)];
                    double y = 0.0;
                    for (int s = 0; s <= N; ++s)
                        if (gi[s] > 0) y = y + f[s] * (double)gi[s];
                    if (rem > 0) {
                        const double t = t0 + y;
                        int slot = N;
                        for (int j = 0; j < N; ++j)
                            if (c_known[j] && cs[j] <= t && t < ce[j]) { slot = j; break; }
                        int64_t cap;
                        if (slot < N) {
                            cap = in_flight(m->lambda, c[slot].nc, cp.tb, m->corun_share);
                            f[slot] = wave_time(cp.theta_us, cap, cp.d_bytes, m->bw_peak, c[slot].v);
                            if (c[slot].pf != 1.0) f[slot] = f[slot] * c[slot].pf;
                        } else {
                            cap = (int64_t)m->lambda * cp.tb;
                            f[slot] = wave_time(cp.theta_us, cap, cp.d_bytes, m->bw_peak, 0.0);
                        }
                        gi[slot] += 1;
                        rem -= rem < cap ? rem : cap;
                    } else {
                        ys[in] = y;
                        pe[in] = t0 + y; p_known[in] = 1;
                        ty = pe[in];
                        running = false;
                        ++in;
                    }
                    progressed = true;
                }
            }
            if (!progressed) return lagom::fail(LAGOM_EINVAL, "the dependencies form a cycle");
        }
        for (int i = 0; i < M; ++i) {
            Y = Y + ys[i];
            if (out->y_us) out->y_us[i] = ys[i];
        }
        if (out->g) for (size_t k = 0; k < gall.size(); ++k) out->g[k] = gall[k];
        const double end_comm = N ? tc : 0.0, end_comp = M ? ty : 0.0;
        Z = end_comm > end_comp ? end_comm : end_comp;
    }
    if (out->x_us) for (int j = 0; j < N; ++j) out->x_us[j] = c[j].x;
    out->X_us = X;
    out->Y_us = Y;
    out->Z_us = Z;
    return LAGOM_OK;
}

extern "C" int lagom_model_profile(void* user, const lagom_cfg* cfgs, int ncomm, double* x_us, double* Y_us) {
    if (!user || !x_us || !Y_us) return lagom::fail(LAGOM_EINVAL, "null argument");
    lagom_pred p{};
    p.x_us = x_us;
    int rc = lagom_cost_model(static_cast<const lagom_model*>(user), cfgs, ncomm, &p);
    if (rc) return rc;
    *Y_us = p.Y_us;
    return LAGOM_OK;
}
