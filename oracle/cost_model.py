"""Oracle: the unified overlap cost model -- TEST INFRASTRUCTURE ONLY.

Follows the paper's Eq. 1 (Z = max(Y, X) with Y = sum_i y_i, X = sum_j x_j) and the
contention wave model of Eq. 4-6 in the paper's notation (Table 1):

    y_i  = sum_{j=l..k} f_ij * g_ij                                   (Eq. 4)
    g_ij = ceil( mu_i / ((lambda - NC_j) * TB_i) )                    (Eq. 5)
    f_ij = theta_i + (lambda - NC_j) * TB_i * D_i / (B - V(NC_j,C_j)) (Eq. 6)

Readings taken where the text leaves a choice:

* mu_i is the total number of workgroups of computation i, TB_i the number resident
  per compute unit, lambda the number of compute units (Eq. 5's prose).
* x_j is not modelled by the paper (it is measured); here it comes from a table
  keyed by the configuration (NC, NT, C), and so does V(NC, C).
* When one computation overlaps several communications, the two serialized queues
  are stepped wave by wave: communication j is active on [sum_{<j} x, sum_{<=j} x);
  a wave that starts while j is active (or after the last one ended: NC = 0, V = 0)
  retires min(remaining, (lambda - NC_j) * TB_i) workgroups and lasts f_ij, and g_ij
  counts the waves issued under j.  With a single communication covering the whole
  computation this is exactly Eq. 4-6 as printed.
* The last, partial wave costs a full f_ij (Eq. 6 is used literally).
* Eq. 1 has no cross-stream dependencies, and none are assumed by default.  The overlap
  patterns of Sec. 2.1 do have them (FSDP: a layer's GEMM needs its all-gathered weights;
  TP with batch pipelining: a batch's all-reduce needs that batch's GEMM), so they can be
  given: computation i may name a communication that must have ended before it starts and
  communication j a computation likewise.  Each stream is then still serial, an operator
  starts at the later of its stream being free and its dependency having ended, the wave
  stepping is unchanged, and the makespan is the later of the two stream ends (without
  dependencies that is max(X, Y) again).

* Not in the paper (an adaptation to a part where a communication workgroup can run beside
  the computation's workgroups on one compute unit): Model.corun_share = sigma in [0, 1] is the
  fraction of a compute unit that stays available to the computation while a channel runs on
  it.  The workgroups in flight of Eq. 5 and Eq. 6 become floor((lambda - NC*(1-sigma)) * TB);
  sigma = 0 (the default) is the paper's model, sigma = 1 leaves only the bandwidth term V.
  Every pin of the printed model runs with sigma = 0; the extension has pins of its own (three
  pencil-worked cases, the closed forms at both ends).

* Not in the paper either (default off): Model.resident_penalty maps a thread count NT to rho >= 0.  A wave of the
  computation that is issued while a communication with NT threads per channel is active lasts f_ij * (1 + rho(NT)).
  Reason: on the part this build targets the computation is slowed for as long as channels are resident, by an amount that
  depends on how heavy one channel is (its thread count) and hardly on how many there are -- neither (lambda - NC) nor
  B - V of Eq. 5-6 can express that.  An NT without an entry has rho = 0; with an empty map the model is unchanged bit for bit.

Units: time in microseconds, bandwidth in bytes per microsecond, D_i in bytes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

Cfg = Tuple[int, int, int]  # (NC, NT, C bytes)


@dataclass
class Comp:
    mu: int          # total workgroups of the computation
    tb: int          # workgroups resident per compute unit
    d_bytes: float   # bytes moved per workgroup
    theta: float     # compute time of one wave, microseconds


@dataclass
class Model:
    lam: int                       # number of compute units
    bw_peak: float                 # peak global-memory bandwidth, bytes / microsecond
    comps: List[Comp]
    # one table per communication: cfg -> (x microseconds, V bytes/microsecond)
    tables: List[Dict[Cfg, Tuple[float, float]]] = field(default_factory=list)
    corun_share: float = 0.0       # sigma; 0 = Eq. 5-6 as printed
    resident_penalty: Dict[int, float] = field(default_factory=dict)   # NT -> rho; empty = Eq. 6 as printed


@dataclass
class Prediction:
    x: List[float]
    y: List[float]
    g: List[List[int]]   # g[i][j], j = N is "no communication active"
    X: float
    Y: float
    Z: float


def workgroups_in_flight(lam: int, nc: int, tb: int, share: float = 0.0) -> int:
    """The divisor of Eq. 5, (lambda - NC) * TB; with a co-run share sigma, floor((lambda - NC*(1-sigma)) * TB)."""
    if not 0.0 <= share <= 1.0:
        raise ValueError("co-run share outside [0, 1]")
    if share == 0.0:
        return (lam - nc) * tb
    return int(math.floor((float(lam) - float(nc) * (1.0 - share)) * float(tb)))


def wave_count(mu: int, lam: int, nc: int, tb: int, share: float = 0.0) -> int:
    """Eq. 5."""
    cap = workgroups_in_flight(lam, nc, tb, share)
    if cap <= 0:
        raise ValueError("communication leaves no compute unit free")
    return -(-mu // cap)


def wave_time(theta: float, lam: int, nc: int, tb: int, d_bytes: float, bw_peak: float, v: float, share: float = 0.0) -> float:
    """Eq. 6."""
    if not v < bw_peak:
        raise ValueError("communication bandwidth reaches the peak")
    cap = workgroups_in_flight(lam, nc, tb, share)
    return theta + (cap * d_bytes) / (bw_peak - v)


def penalty_factor(model: Model, nt: int) -> float:
    """1 + rho(NT); exactly 1.0 where the map has no entry."""
    rho = model.resident_penalty.get(int(nt))
    if rho is None:
        return 1.0
    if not rho >= 0.0:
        raise ValueError("negative resident penalty")
    return 1.0 + rho


def predict(model: Model, cfgs: Sequence[Cfg], comp_after_comm=None, comm_after_comp=None) -> Prediction:
    """Eq. 1 over Eq. 4-6 for the whole overlap group.

    comp_after_comm[i] = j (or -1): computation i starts only after communication j has ended;
    comm_after_comp[j] = i (or -1): communication j starts only after computation i has ended.
    """
    if comp_after_comm is not None or comm_after_comp is not None:
        return _predict_dependent(model, cfgs, comp_after_comm, comm_after_comp)
    N = len(model.tables)
    if len(cfgs) != N:
        raise ValueError("one configuration per communication")
    x, v, nc, pf = [], [], [], []
    for j, cfg in enumerate(cfgs):
        key = (int(cfg[0]), int(cfg[1]), int(cfg[2]))
        if key not in model.tables[j]:
            raise KeyError(f"communication {j}: configuration {key} not in its table")
        xj, vj = model.tables[j][key]
        if key[0] >= model.lam or key[0] < 1:
            raise ValueError("NC out of range")
        if not (0.0 <= vj < model.bw_peak) or not xj >= 0.0:
            raise ValueError("table entry out of range")
        x.append(float(xj)); v.append(float(vj)); nc.append(key[0]); pf.append(penalty_factor(model, key[1]))
    # communication j is active on [T[j], T[j+1])
    T = [0.0]
    for xj in x:
        T.append(T[-1] + xj)
    X = T[N]

    y_all, g_all = [], []
    t0 = 0.0
    for comp in model.comps:
        if comp.mu < 0 or comp.tb < 1:
            raise ValueError("bad computation description")
        g = [0] * (N + 1)
        f = [0.0] * (N + 1)
        rem = comp.mu
        t = t0
        y = 0.0
        while rem > 0:
            slot = N
            for j in range(N):
                if t < T[j + 1]:
                    slot = j
                    break
            if slot < N:
                cap = workgroups_in_flight(model.lam, nc[slot], comp.tb, model.corun_share)
                f[slot] = wave_time(comp.theta, model.lam, nc[slot], comp.tb, comp.d_bytes, model.bw_peak, v[slot], model.corun_share)
                if pf[slot] != 1.0:
                    f[slot] = f[slot] * pf[slot]
            else:
                cap = model.lam * comp.tb
                f[slot] = wave_time(comp.theta, model.lam, 0, comp.tb, comp.d_bytes, model.bw_peak, 0.0)
            g[slot] += 1
            rem -= min(rem, cap)
            y = 0.0
            for s in range(N + 1):          # Eq. 4, terms in ascending j
                if g[s] > 0:
                    y = y + f[s] * g[s]
            t = t0 + y
        y_all.append(y)
        g_all.append(g)
        t0 = t0 + y
    Y = 0.0
    for yi in y_all:
        Y = Y + yi
    return Prediction(x=x, y=y_all, g=g_all, X=X, Y=Y, Z=max(X, Y))


def _predict_dependent(model: Model, cfgs: Sequence[Cfg], comp_after_comm, comm_after_comp) -> Prediction:
    N, M = len(model.tables), len(model.comps)
    free = predict(model, cfgs)                       # validates the inputs; x_j do not depend on the timeline
    x = free.x
    nc = [int(c[0]) for c in cfgs]
    pf = [penalty_factor(model, int(c[1])) for c in cfgs]
    v = [model.tables[j][(int(c[0]), int(c[1]), int(c[2]))][1] for j, c in enumerate(cfgs)]
    cac = list(comp_after_comm) if comp_after_comm is not None else [-1] * M
    cap_ = list(comm_after_comp) if comm_after_comp is not None else [-1] * N
    if len(cac) != M or len(cap_) != N or any(not -1 <= d < N for d in cac) or any(not -1 <= d < M for d in cap_):
        raise ValueError("bad dependency arrays")
    comm_start, comm_end, comp_end = [None] * N, [None] * N, [None] * M
    y_all, g_all = [0.0] * M, [[0] * (N + 1) for _ in range(M)]
    j_next, i_next = 0, 0
    tc, ty = 0.0, 0.0                                 # when each stream becomes free
    # state of the computation in progress
    running, rem, t0, f = False, 0, 0.0, [0.0] * (N + 1)
    while j_next < N or i_next < M:
        progressed = False
        # start every communication whose turn and dependency have come
        while j_next < N and (cap_[j_next] < 0 or comp_end[cap_[j_next]] is not None):
            dep = cap_[j_next]
            start = tc if dep < 0 else max(tc, comp_end[dep])
            comm_start[j_next], comm_end[j_next] = start, start + x[j_next]
            tc = comm_end[j_next]
            j_next += 1
            progressed = True
        if i_next < M:
            comp = model.comps[i_next]
            if not running:
                dep = cac[i_next]
                if dep < 0 or comm_end[dep] is not None:
                    t0 = ty if dep < 0 else max(ty, comm_end[dep])
                    running, rem, f = True, comp.mu, [0.0] * (N + 1)
                    progressed = True
            if running:
                g = g_all[i_next]
                y = 0.0
                for s in range(N + 1):
                    if g[s] > 0:
                        y = y + f[s] * g[s]
                if rem > 0:
                    t = t0 + y
                    slot = N
                    for j in range(N):
                        if comm_start[j] is not None and comm_start[j] <= t < comm_end[j]:
                            slot = j
                            break
                    if slot < N:
                        cap = workgroups_in_flight(model.lam, nc[slot], comp.tb, model.corun_share)
                        f[slot] = wave_time(comp.theta, model.lam, nc[slot], comp.tb, comp.d_bytes, model.bw_peak, v[slot], model.corun_share)
                        if pf[slot] != 1.0:
                            f[slot] = f[slot] * pf[slot]
                    else:
                        cap = model.lam * comp.tb
                        f[slot] = wave_time(comp.theta, model.lam, 0, comp.tb, comp.d_bytes, model.bw_peak, 0.0)
                    g[slot] += 1
                    rem -= min(rem, cap)
                    progressed = True
                else:
                    y_all[i_next] = y
                    comp_end[i_next] = t0 + y
                    ty = comp_end[i_next]
                    running = False
                    i_next += 1
                    progressed = True
        if not progressed:
            raise ValueError("the dependencies form a cycle")
    X = 0.0
    for xj in x:
        X = X + xj
    Y = 0.0
    for yi in y_all:
        Y = Y + yi
    end_comm = tc if N else 0.0
    end_comp = ty if M else 0.0
    return Prediction(x=x, y=y_all, g=g_all, X=X, Y=Y, Z=max(end_comm, end_comp))
