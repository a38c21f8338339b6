"""Oracle: filling the contention wave model from a profiler sweep -- TEST INFRASTRUCTURE ONLY.

The paper measures x_j and uses Eq. 4-6 for the computations (Sec. 3.2); it prints neither how
theta nor how V(NC, C) is obtained.  The reading taken here, step by step:

* t_alone = median over the sweep points of (standalone computation time) / (number of
  computations): every computation of a group has the same geometry.
* theta (Eq. 6 solved for theta with no communication active: NC = 0, V = 0):
      g0    = ceil(mu / (lambda * TB))                       (Eq. 5)
      theta = t_alone / g0 - lambda * TB * D / B             (Eq. 6), floored at 0
  so that, whenever the floor is not hit, the filled model returns exactly t_alone for a
  computation that no communication overlaps.
* Tables, one entry per swept configuration and communication j: the sweep times the
  communication stream as a whole, and communication j's part of it is its part of the bytes:
      share_j = bytes_j / sum(bytes),   x_j = share_j * X_corun,
      V       = min(bytes / X_corun, cap * B)                (Eq. 6 needs V < B; cap = 0.99)
  (bytes_j / x_j = bytes / X_corun for every j).
* Calibration of the co-run share sigma (the extension of oracle.cost_model): theta is fitted on
  the points that are not held out, every candidate sigma is scored by the mean of
  |Y_model - Y_measured| / Y_measured over those points, the first smallest wins; the same error
  is reported over the held-out points.  x and V of every point stay in the tables -- they are
  measured inputs of the model (Eq. 1), not predictions.

* Calibration of the resident penalty rho(NT) (the second extension of oracle.cost_model), after sigma: for every thread
  count NT among the points that are not held out, in ascending order, every candidate rho is scored by the mean error
  over the fitted points *with that NT* (the penalties chosen for smaller NT already in place -- they do not touch
  these points, a point's communications all have its NT), the first smallest wins.  Errors are then reported over all
  fitted and all held-out points with sigma and every rho in place.

Every function is pinned in tests/test_oracle_model_fill.py by pencil-worked numbers, by the
round trip "filled model without communication == t_alone", and by recovering a planted sigma.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

from . import cost_model as cm

Cfg = Tuple[int, int, int]


@dataclass
class SweepPoint:
    cfg: Cfg
    comm_corun_us: float     # X of the co-run, all communications of the group at `cfg`
    comp_alone_us: float     # Y of the computations alone
    comp_corun_us: float     # Y of the co-run
    v_corun: float           # algorithmic bytes / X_corun, bytes per microsecond


@dataclass
class Geometry:
    mu: int
    tb: int
    d_bytes: float


def median(values: Sequence[float]) -> float:
    v = sorted(float(x) for x in values)
    n = len(v)
    if n == 0:
        raise ValueError("median of nothing")
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def t_alone(points: Sequence[SweepPoint], ncomp: int) -> float:
    return median([p.comp_alone_us for p in points]) / float(ncomp)


def fit_theta(t_alone_us: float, geo: Geometry, lam: int, bw_peak: float) -> float:
    g0 = -(-geo.mu // (lam * geo.tb))
    if g0 < 1:
        raise ValueError("a computation needs at least one workgroup")
    theta = t_alone_us / float(g0) - (float(lam * geo.tb) * geo.d_bytes) / bw_peak
    return theta if theta > 0.0 else 0.0


def shares(comm_bytes: Sequence[float]) -> List[float]:
    total = 0.0
    for b in comm_bytes:
        total = total + float(b)
    if not total > 0.0:
        raise ValueError("the communications move no bytes")
    return [float(b) / total for b in comm_bytes]


def fill_tables(points: Sequence[SweepPoint], comm_bytes: Sequence[float], bw_peak: float, cap: float = 0.99):
    sh = shares(comm_bytes)
    vmax = cap * bw_peak
    tables = []
    for s in sh:
        tables.append({tuple(p.cfg): (s * p.comm_corun_us, p.v_corun if p.v_corun < vmax else vmax) for p in points})
    return tables


def fill(points: Sequence[SweepPoint], geo: Geometry, ncomp: int, comm_bytes: Sequence[float], lam: int, bw_peak: float,
         sigma: float = 0.0, theta_points: Optional[Sequence[SweepPoint]] = None, penalty=None) -> cm.Model:
    """The model of one overlap group.  theta is fitted on `theta_points` (default: all points)."""
    theta = fit_theta(t_alone(theta_points if theta_points is not None else points, ncomp), geo, lam, bw_peak)
    comps = [cm.Comp(geo.mu, geo.tb, geo.d_bytes, theta) for _ in range(ncomp)]
    return cm.Model(lam, bw_peak, comps, fill_tables(points, comm_bytes, bw_peak), corun_share=sigma,
                    resident_penalty=dict(penalty) if penalty else {})


def y_errors(model: cm.Model, points: Sequence[SweepPoint], comp_after_comm=None, comm_after_comp=None) -> Tuple[float, float]:
    """Mean and maximum of |Y_model - Y_measured| / Y_measured over `points` (all communications at the point's cfg)."""
    n = len(model.tables)
    total, worst = 0.0, 0.0
    for p in points:
        y = cm.predict(model, [tuple(p.cfg)] * n, comp_after_comm, comm_after_comp).Y
        e = abs(y - p.comp_corun_us) / p.comp_corun_us
        total = total + e
        worst = e if e > worst else worst
    return (total / float(len(points)) if points else 0.0), worst


@dataclass
class Calibration:
    sigma: float
    fit_mean: float
    fit_max: float
    held_mean: float
    held_max: float
    n_fit: int
    n_held: int
    penalty: Optional[dict] = None      # NT -> rho, when rhos were given


def calibrate(points: Sequence[SweepPoint], held_out: Optional[Sequence[bool]], geo: Geometry, ncomp: int,
              comm_bytes: Sequence[float], lam: int, bw_peak: float, sigmas: Sequence[float],
              comp_after_comm=None, comm_after_comp=None, rhos: Optional[Sequence[float]] = None) -> Calibration:
    held = [bool(h) for h in held_out] if held_out is not None else [False] * len(points)
    fit_pts = [p for p, h in zip(points, held) if not h]
    held_pts = [p for p, h in zip(points, held) if h]
    if not fit_pts or not sigmas:
        raise ValueError("nothing to fit on")
    best = None
    for s in sigmas:
        model = fill(points, geo, ncomp, comm_bytes, lam, bw_peak, s, theta_points=fit_pts)
        mean, worst = y_errors(model, fit_pts, comp_after_comm, comm_after_comp)
        if best is None or mean < best[0]:
            best = (mean, worst, s, model)
    mean, worst, s, model = best
    penalty = None
    if rhos:
        penalty = {}
        for nt in sorted(set(int(p.cfg[1]) for p in fit_pts)):
            with_nt = [p for p in fit_pts if int(p.cfg[1]) == nt]
            pick = None
            for rho in rhos:
                model.resident_penalty = dict(penalty)
                model.resident_penalty[nt] = float(rho)
                m, _ = y_errors(model, with_nt, comp_after_comm, comm_after_comp)
                if pick is None or m < pick[0]:
                    pick = (m, float(rho))
            penalty[nt] = pick[1]
        model.resident_penalty = dict(penalty)
        mean, worst = y_errors(model, fit_pts, comp_after_comm, comm_after_comp)
    h_mean, h_max = y_errors(model, held_pts, comp_after_comm, comm_after_comp)
    return Calibration(s, mean, worst, h_mean, h_max, len(fit_pts), len(held_pts), penalty)
