"""Oracle: priority-based parameter search and brute force -- TEST INFRASTRUCTURE ONLY.

Follows the paper's Sec. 3.3-3.4: the priority metric H (Eq. 7), the
cost-effectiveness loop (Alg. 1) and resource-efficient tuning (Alg. 2), in the
paper's order and notation, with these readings where the text leaves a choice or
is garbled:

* Search space.  Alg. 2 raises NC, NT and C together, so each communication j moves
  on a one-dimensional ladder of levels 0..K_j-1: level l stands for
  (G_NC[min(l,|G_NC|-1)], G_NT[min(l,|G_NT|-1)], G_C[min(l,|G_C|-1)]) over ascending
  grids, K_j = the longest grid.  Brute force ranges over the product of the ladders.
* Initial state.  Every communication starts at level 0 (the minimum values of
  Alg. 2) and one baseline profile measures all of them; if X < Y there, every
  communication is done (optimality condition 1).
* Learning rate.  As printed lr is negative exactly when a step helped and is added
  to integers; read as lr = (x - x') / x' >= 0, and a step goes to the lowest level
  above the current one at which every parameter has reached min(p * (1 + lr), p_max);
  the first step of a communication (no lr yet) is one level.  A communication at
  its top level is done.
* Which configuration is kept at "done".  If the trial made x_j worse, the previous
  level is kept.  If the trial hid all communication (X' < Y'), whichever of previous
  and trial has the smaller makespan Z is kept, ties to the previous (fewer resources).
* H.  H_j = (Y' - Y) / (x_j - x_j') in double, exactly that expression; a zero
  denominator gives +inf; H stays 0.01 until the communication has an accepted step;
  the smallest H wins, ties to the lowest index.
* ProfileTime returns every x_j and Y; X is their sum in index order; measurements of
  the accepted configuration vector are the "before" values of the next step.
"""
from __future__ import annotations

import itertools
import math
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

Cfg = Tuple[int, int, int]
ProfileFn = Callable[[Sequence[Cfg]], Tuple[Sequence[float], float]]

H_INIT = 0.01  # Alg. 1: "Initialize all H to 0.01"


@dataclass
class Space:
    nc: List[int]
    nt: List[int]
    chunk: List[int]

    def __post_init__(self):
        for g in (self.nc, self.nt, self.chunk):
            if len(g) < 1 or any(b <= a for a, b in zip(g, g[1:])):
                raise ValueError("grids must be non-empty and strictly ascending")

    @property
    def K(self) -> int:
        return max(len(self.nc), len(self.nt), len(self.chunk))

    def cfg(self, level: int) -> Cfg:
        if not 0 <= level < self.K:
            raise ValueError("level out of range")
        pick = lambda g: g[min(level, len(g) - 1)]
        return (pick(self.nc), pick(self.nt), pick(self.chunk))


@dataclass
class Step:
    comm: int              # -1 for the baseline profile
    level_from: int
    level_to: int
    accepted: bool
    done: bool
    xj_prev: float
    xj_new: float
    X: float
    Y: float
    Z: float
    H: float               # H of `comm` after this step
    lr: float              # learning rate of `comm` after this step (nan if none yet)


@dataclass
class Result:
    levels: List[int]
    cfgs: List[Cfg]
    x: List[float]
    X: float
    Y: float
    Z: float
    calls: int
    trace: List[Step] = field(default_factory=list)


def _sum(xs: Sequence[float]) -> float:
    s = 0.0
    for v in xs:
        s = s + v
    return s


def priority_metric(Y_before: float, Y_after: float, x_before: float, x_after: float) -> float:
    """Eq. 7."""
    den = x_before - x_after
    if den == 0.0:
        return math.inf
    return (Y_after - Y_before) / den


def next_level(space: Space, level: int, lr: Optional[float]) -> int:
    """Alg. 2's parameter increase, on the ladder."""
    top = space.K - 1
    if level >= top:
        return top
    if lr is None:
        return level + 1
    cur = space.cfg(level)
    grids = (space.nc, space.nt, space.chunk)
    for cand in range(level + 1, top + 1):
        c = space.cfg(cand)
        ok = True
        for p in range(3):
            target = float(cur[p]) * (1.0 + lr)
            if not (float(c[p]) >= target or c[p] == grids[p][-1]):
                ok = False
                break
        if ok:
            return cand
    return top


def priority_search(spaces: Sequence[Space], profile: ProfileFn, free_steps: bool = False) -> Result:
    """Alg. 1 driving Alg. 2.

    free_steps (default off = the algorithm as printed).  Alg. 2 ends a communication at "X' < Y'" because, by the paper's
    contention analysis (Sec. 3.2), any further resource can only lengthen the computation.  Where a step makes the
    communication faster *and* the computation faster (H of Eq. 7 negative: the step costs nothing), that reason does
    not apply; with free_steps such a step is accepted like any other and the communication stays in the search.  A
    hidden step that does not lower Y ends the communication exactly as printed.
    """
    N = len(spaces)
    lev = [0] * N
    H = [H_INIT] * N
    lr: List[Optional[float]] = [None] * N
    done = [sp.K == 1 for sp in spaces]
    trace: List[Step] = []

    x, Y = profile([sp.cfg(l) for sp, l in zip(spaces, lev)])
    x = [float(v) for v in x]; Y = float(Y)
    X = _sum(x); Z = max(X, Y)
    calls = 1
    if X < Y:                      # optimality condition 1
        done = [True] * N
    trace.append(Step(-1, 0, 0, True, all(done), math.nan, math.nan, X, Y, Z, H_INIT, math.nan))

    while not all(done):
        j = -1
        for i in range(N):          # Alg. 1: not-done communication with the smallest H
            if not done[i] and (j < 0 or H[i] < H[j]):
                j = i
        new = next_level(spaces[j], lev[j], lr[j])
        trial = list(lev); trial[j] = new
        x2, Y2 = profile([sp.cfg(l) for sp, l in zip(spaces, trial)])
        x2 = [float(v) for v in x2]; Y2 = float(Y2)
        X2 = _sum(x2); Z2 = max(X2, Y2)
        calls += 1
        if x2[j] - x[j] > 0.0:      # Alg. 2: the communication itself got slower
            done[j] = True
            accepted = False
        elif X2 < Y2 and not (free_steps and Y2 < Y):   # Alg. 2: all communication is hidden
            done[j] = True
            accepted = Z2 < Z
        else:
            accepted = True
            H[j] = priority_metric(Y, Y2, x[j], x2[j])
            den = x[j] - x2[j]
            lr[j] = math.inf if x2[j] == 0.0 else den / x2[j]
            if new == spaces[j].K - 1:
                done[j] = True
        trace.append(Step(j, lev[j], new, accepted, done[j], x[j], x2[j], X2, Y2, Z2, H[j],
                          math.nan if lr[j] is None else lr[j]))
        if accepted:
            lev, x, Y, X, Z = trial, x2, Y2, X2, Z2
    return Result(levels=lev, cfgs=[sp.cfg(l) for sp, l in zip(spaces, lev)],
                  x=x, X=X, Y=Y, Z=Z, calls=calls, trace=trace)


def brute_force(spaces: Sequence[Space], profile: ProfileFn) -> Result:
    """Exhaustive search over the product of the ladders.

    argmin Z; ties go to the smallest sum of levels, then to the lexicographically
    smallest level vector (the minimal resource-related parameters).
    """
    best = None
    calls = 0
    for levels in itertools.product(*[range(sp.K) for sp in spaces]):
        x, Y = profile([sp.cfg(l) for sp, l in zip(spaces, levels)])
        x = [float(v) for v in x]; Y = float(Y)
        X = _sum(x); Z = max(X, Y)
        calls += 1
        key = (Z, sum(levels), tuple(levels))
        if best is None or key < best[0]:
            best = (key, list(levels), x, X, Y, Z)
    _, levels, x, X, Y, Z = best
    return Result(levels=levels, cfgs=[sp.cfg(l) for sp, l in zip(spaces, levels)],
                  x=x, X=X, Y=Y, Z=Z, calls=calls)


def brute_force_full_product(spaces: Sequence[Space], profile: ProfileFn):
    """Exhaustive search over every (NC, NT, C) combination of every communication.

    Only for reporting what the diagonal ladder gives up (tiny N).  Returns
    (cfgs, Z, calls); ties go to the first combination in product order.
    """
    per_comm = [list(itertools.product(sp.nc, sp.nt, sp.chunk)) for sp in spaces]
    best = None
    calls = 0
    for cfgs in itertools.product(*per_comm):
        x, Y = profile(list(cfgs))
        Z = max(_sum([float(v) for v in x]), float(Y))
        calls += 1
        if best is None or Z < best[1]:
            best = (list(cfgs), Z)
    return best[0], best[1], calls


def coordinate_descent(spaces: Sequence[Space], profile: ProfileFn) -> Result:
    """Communication-bound regime (Eq. 2): the makespan is the sum of the x_j and separates per
    communication, so each x_j is minimised on its own over the full (NC, NT, C) product.

    The paper only names the method of its predecessor for this regime (coordinate descent over the
    resource parameters with measured feedback) and gives no steps; this build's definition:
    communications are taken in index order, the others staying where they are (the grid minimum
    until they have been tuned); for one communication, starting from the minimum of every grid,
    sweep the coordinates in the order NC, C, NT; along a coordinate go one grid step up while x_j
    falls strictly, and if the first step up did not help go down while x_j falls strictly; repeat
    the sweeps until one changes nothing.  Every probe is one profile call.
    """
    N = len(spaces)
    idx = [[0, 0, 0] for _ in range(N)]               # indices into (nc, nt, chunk)
    grids = [(sp.nc, sp.nt, sp.chunk) for sp in spaces]
    calls = 0

    def cfgs_of(ix):
        return [(g[0][i[0]], g[1][i[1]], g[2][i[2]]) for g, i in zip(grids, ix)]

    def probe(ix):
        nonlocal calls
        x, Y = profile(cfgs_of(ix))
        calls += 1
        return [float(v) for v in x], float(Y)

    x, Y = probe(idx)
    for j in range(N):
        best = x[j]
        changed = True
        while changed:
            changed = False
            for p in (0, 2, 1):                       # NC, C, NT
                moved_up = False
                while idx[j][p] + 1 < len(grids[j][p]):
                    idx[j][p] += 1
                    x2, Y2 = probe(idx)
                    if x2[j] < best:
                        best, x, Y, moved_up, changed = x2[j], x2, Y2, True, True
                    else:
                        idx[j][p] -= 1
                        break
                if moved_up:
                    continue
                while idx[j][p] - 1 >= 0:
                    idx[j][p] -= 1
                    x2, Y2 = probe(idx)
                    if x2[j] < best:
                        best, x, Y, changed = x2[j], x2, Y2, True
                    else:
                        idx[j][p] += 1
                        break
    X = _sum(x)
    return Result(levels=[i[0] for i in idx], cfgs=cfgs_of(idx), x=x, X=X, Y=Y, Z=max(X, Y), calls=calls)


def hide_search(spaces: Sequence[Space], profile: ProfileFn) -> Result:
    """The computation-bound objective (Sec. 3.1, Eq. 3): once the communication is hidden the makespan is
    Y, and Y grows with the resources the communications hold (Sec. 3.2), so the goal is the least Y
    subject to X <= Y.  The paper's own loop (Alg. 1 driving Alg. 2) already walks up from the minimum
    resources and stops at "X' < Y'"; this variant keeps exactly that walk and changes only what happens
    at the stop: the baseline ends the search when X <= Y, and the first trial with X' <= Y' is kept and
    ends the search for every communication (the lowest resources on the path that hide the
    communication -- anything raised further can only add contention).  If no visited vector hides the
    communication, the walk ends as Alg. 1/2 ends and its last accepted vector is returned.
    """
    N = len(spaces)
    lev = [0] * N
    H = [H_INIT] * N
    lr: List[Optional[float]] = [None] * N
    done = [sp.K == 1 for sp in spaces]
    trace: List[Step] = []

    x, Y = profile([sp.cfg(l) for sp, l in zip(spaces, lev)])
    x = [float(v) for v in x]; Y = float(Y)
    X = _sum(x); Z = max(X, Y)
    calls = 1
    if X <= Y:
        done = [True] * N
    trace.append(Step(-1, 0, 0, True, all(done), math.nan, math.nan, X, Y, Z, H_INIT, math.nan))

    while not all(done):
        j = -1
        for i in range(N):
            if not done[i] and (j < 0 or H[i] < H[j]):
                j = i
        new = next_level(spaces[j], lev[j], lr[j])
        trial = list(lev); trial[j] = new
        x2, Y2 = profile([sp.cfg(l) for sp, l in zip(spaces, trial)])
        x2 = [float(v) for v in x2]; Y2 = float(Y2)
        X2 = _sum(x2); Z2 = max(X2, Y2)
        calls += 1
        if x2[j] - x[j] > 0.0:
            done[j] = True
            accepted = False
        elif X2 <= Y2:              # hidden: keep it, and nothing else needs raising
            accepted = True
            done = [True] * N
        else:
            accepted = True
            H[j] = priority_metric(Y, Y2, x[j], x2[j])
            den = x[j] - x2[j]
            lr[j] = math.inf if x2[j] == 0.0 else den / x2[j]
            if new == spaces[j].K - 1:
                done[j] = True
        trace.append(Step(j, lev[j], new, accepted, done[j], x[j], x2[j], X2, Y2, Z2, H[j],
                          math.nan if lr[j] is None else lr[j]))
        if accepted:
            lev, x, Y, X, Z = trial, x2, Y2, X2, Z2
    return Result(levels=lev, cfgs=[sp.cfg(l) for sp, l in zip(spaces, lev)],
                  x=x, X=X, Y=Y, Z=Z, calls=calls, trace=trace)


def brute_force_hide(spaces: Sequence[Space], profile: ProfileFn) -> Result:
    """Exhaustive counterpart of hide_search: among the level vectors with X <= Y the smallest Y (ties:
    smallest level sum, then lexicographic); if no vector hides the communication, the smallest Z with
    the same tie-breaks (which is brute_force's answer)."""
    best_hidden = None
    best_any = None
    calls = 0
    for levels in itertools.product(*[range(sp.K) for sp in spaces]):
        x, Y = profile([sp.cfg(l) for sp, l in zip(spaces, levels)])
        x = [float(v) for v in x]; Y = float(Y)
        X = _sum(x); Z = max(X, Y)
        calls += 1
        rec = (list(levels), x, X, Y, Z)
        key_any = (Z, sum(levels), tuple(levels))
        if best_any is None or key_any < best_any[0]:
            best_any = (key_any, rec)
        if X <= Y:
            key_h = (Y, sum(levels), tuple(levels))
            if best_hidden is None or key_h < best_hidden[0]:
                best_hidden = (key_h, rec)
    levels, x, X, Y, Z = (best_hidden or best_any)[1]
    return Result(levels=levels, cfgs=[sp.cfg(l) for sp, l in zip(spaces, levels)],
                  x=x, X=X, Y=Y, Z=Z, calls=calls)


LADDER_FULL, LADDER_CUT, LADDER_FIXED_CHUNK = 0, 1, 2


def ladder_chunks(chunk_grid: Sequence[int], nc_max: int, nt_ref: int, bytes_per_source: int, kind: int,
                  alone_us=None) -> List[int]:
    """The chunk grid a ladder is built from.  Chunk g of a launch goes to channel g mod NC (Sec. 3.2: NC
    blocks move data at granularity C), so when chunk * nc_max exceeds the bytes a launch moves per source
    some channels have nothing to move.  FULL: the grid; CUT: the chunks with chunk * nc_max <=
    bytes_per_source (at least the smallest); FIXED_CHUNK: the single chunk with the smallest standalone
    communication time at (nc_max, nt_ref), first smallest in grid order -- `alone_us` maps
    (nc, nt, chunk) to that time."""
    grid = list(chunk_grid)
    if kind == LADDER_FULL:
        return grid
    if kind == LADDER_CUT:
        kept = [c for c in grid if c * nc_max <= bytes_per_source]
        return kept if kept else [grid[0]]
    if kind == LADDER_FIXED_CHUNK:
        best = None
        for c in grid:
            t = alone_us.get((nc_max, nt_ref, c))
            if t is not None and (best is None or t < best[0]):
                best = (t, c)
        if best is None:
            raise ValueError("no sweep point at (nc_max, nt_ref)")
        return [best[1]]
    raise ValueError("unknown ladder kind")
