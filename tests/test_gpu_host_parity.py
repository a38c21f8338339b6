"""GPU record of the host rows against the oracle.  The searches run inside the library with the measured
ProfileTime (lagom_overlap_profile); what every call measured is logged by the library, and the same sequence of
measurements is then replayed to oracle.search, whose result and full trace must equal the library's.  The cost model is
filled from a sweep measured in this run by the library and by the oracle, and both must predict the same numbers."""
import math

import numpy as np
import pytest
import torch

from oracle import cost_model as ocm, model_fill as omf, search as osr
from paper_2602_20656_amd import binding as lg, inputs
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def chain():
    """Three all-gather copies (8 shards of 256 Ki bf16 -> 4 MiB) against three 1024 x 2048 x 2048 GEMMs."""
    n, P, N3 = 1 << 18, 8, 3
    s1, s2 = lg.overlapping_streams()
    keep, launches, comps = [], [], []
    A = dev(inputs.normal_bf16(2, (1024, 2048)))
    for j in range(N3):
        shards = [dev(inputs.normal_bf16(100 * j + p, n, 0.02)) for p in range(P)]
        full = dev(np.zeros(P * n, np.uint16))
        B = dev(inputs.normal_bf16(3 + j, (2048, 2048), 0.02))
        Cm = dev(np.zeros((1024, 2048), np.uint16))
        keep += [shards, full, B, Cm]
        launches.append(lg.CommLaunch(lg.LAGOM_GATHER_COPY, lg.LAGOM_BF16, shards, [full], n, j))
        comps.append(lg.GemmDesc(A, B, Cm, 1024, 2048, 2048))
    torch.cuda.synchronize()
    return dict(s1=s1, s2=s2, launches=launches, comps=comps, keep=keep + [A], ncomm=N3)


def _replay(log):
    """A ProfileTime that hands out the logged measurements in call order and insists on the logged configurations."""
    state = {"k": 0}

    def profile(cfgs):
        e = log[state["k"]]
        assert [tuple(c) for c in cfgs] == [tuple(c) for c in e["cfgs"]], f"call {state['k']}: the oracle asks for another configuration"
        state["k"] += 1
        return e["x"], e["Y"]
    return profile, state


def _same_trace(lib_trace, oracle_trace):
    assert len(lib_trace) == len(oracle_trace)
    for a, b in zip(lib_trace, oracle_trace):
        assert (a.comm, a.level_from, a.level_to, a.accepted, a.done) == (b.comm, b.level_from, b.level_to, b.accepted, b.done)
        for u, v in [(a.xj_prev, b.xj_prev), (a.xj_new, b.xj_new), (a.X, b.X), (a.Y, b.Y), (a.Z, b.Z), (a.H, b.H), (a.lr, b.lr)]:
            assert (math.isnan(u) and math.isnan(v)) or u == v


NC, NT, CH = [1, 4, 16, 64], [256], [32 << 10, 128 << 10]
MODES = [(lg.LAGOM_PRIORITY, osr.priority_search, True), (lg.LAGOM_HIDE_COMM, osr.hide_search, True),
         (lg.LAGOM_PRIORITY_FREE, lambda sp, pr: osr.priority_search(sp, pr, free_steps=True), True),
         (lg.LAGOM_COMM_OPTIMAL, osr.coordinate_descent, False), (lg.LAGOM_EXHAUSTIVE, osr.brute_force, False),
         (lg.LAGOM_EXHAUSTIVE_HIDE, osr.brute_force_hide, False)]


@pytest.mark.parametrize("mode,oracle_fn,has_trace", MODES, ids=["priority", "hide_comm", "priority_free", "comm_optimal", "exhaustive", "exhaustive_hide"])
def test_measured_search_replayed_through_the_oracle(chain, mode, oracle_fn, has_trace):
    sl = [lg.Space(NC, NT, CH) for _ in range(chain["ncomm"])]
    so = [osr.Space(NC, NT, CH) for _ in range(chain["ncomm"])]
    prof = lg.OverlapProfile(chain["launches"], chain["comps"], chain["s1"], chain["s2"], 1, 3, log_capacity=400)
    rl = lg.lagom_tune(sl, prof, mode)
    assert len(prof.log) == rl.calls and rl.calls >= 1
    replay, state = _replay(prof.log)
    ro = oracle_fn(so, replay)
    assert state["k"] == len(prof.log) == ro.calls              # the oracle made exactly the same calls
    assert rl.cfgs == ro.cfgs and (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)
    if mode != lg.LAGOM_COMM_OPTIMAL:
        assert rl.levels == ro.levels
    if has_trace:
        _same_trace(rl.trace, ro.trace)
        assert rl.calls <= 1 + sum(sp.K for sp in so)           # linear in the number of communications (Sec. 4.4)
    # what was measured is a real co-run: every x_j and Y positive, spreads reported
    for e in prof.log:
        assert all(x > 0 for x in e["x"]) and e["Y"] > 0 and e["Z"] >= max(sum(e["x"]), e["Y"]) * 0.5 and e["iters"] >= 3


def test_short_groups_are_measured_for_longer(chain):
    sl = [lg.Space([4], NT, [32 << 10]) for _ in range(chain["ncomm"])]
    prof = lg.OverlapProfile(chain["launches"], chain["comps"], chain["s1"], chain["s2"], 1, 3, min_total_us=5000.0, max_iters=40, log_capacity=4)
    lg.lagom_tune(sl, prof, lg.LAGOM_PRIORITY)
    e = prof.log[0]
    assert 3 < e["iters"] <= 40 and e["iters"] * e["Z"] >= 5000.0 * 0.5


def test_model_filled_from_a_measured_sweep_equals_the_oracle(chain):
    """lagom_contention_sweep -> lagom_model_fill / lagom_model_calibrate -> lagom_cost_model, against the oracle fed the
    same measured points: tables, theta, calibration and every prediction equal bit for bit."""
    ncomm, ncomp = chain["ncomm"], len(chain["comps"])
    points = [(nc, 256, c) for nc in NC for c in CH]
    sweep = lg.lagom_contention_sweep(chain["launches"], ncomm, chain["comps"], points, chain["s1"], chain["s2"], 1, 3)
    assert all(p.comm_alone_us > 0 and p.comm_corun_us > 0 and p.comp_corun_us > 0 and p.z_corun_us > 0 for p in sweep)
    nbytes = [float(lg.lagom_comm_bytes(l.op, l.dtype, len(l.srcs), len(l.dsts), l.count)) for l in chain["launches"]]
    # V = algorithmic bytes / X, as the header defines it
    for p in sweep:
        assert p.v_corun == sum(nbytes) / p.comm_corun_us and p.v_alone == sum(nbytes) / p.comm_alone_us
    geo = lg.lagom_gemm_describe(1024, 2048, 2048)
    lam, bw = 256, 8.0e6
    held = [i % 2 == 1 for i in range(len(sweep))]
    sigmas = [i / 8 for i in range(9)]
    opts = [omf.SweepPoint(p.cfg, p.comm_corun_us, p.comp_alone_us, p.comp_corun_us, p.v_corun) for p in sweep]
    ogeo = omf.Geometry(geo.mu, geo.tb, geo.d_bytes_past_l2)
    rhos = [0.0, 0.02, 0.05, 0.1, 0.2, 0.4]
    for use_rhos in (None, rhos):
        co = omf.calibrate(opts, held, ogeo, ncomp, nbytes, lam, bw, sigmas, rhos=use_rhos)
        cl = lg.lagom_model_calibrate(sweep, lam, bw, geo.mu, geo.tb, geo.d_bytes_past_l2, ncomp, nbytes, sigmas, held, rhos=use_rhos)
        assert (cl.sigma, cl.fit_mean, cl.fit_max, cl.held_mean, cl.held_max, cl.n_fit, cl.n_held, cl.penalty) == \
            (co.sigma, co.fit_mean, co.fit_max, co.held_mean, co.held_max, co.n_fit, co.n_held, co.penalty)
    ml, t_alone = lg.lagom_model_fill(sweep, lam, bw, geo.mu, geo.tb, geo.d_bytes_past_l2, ncomp, nbytes, corun_share=cl.sigma,
                                      resident_penalty=cl.penalty)
    mo = omf.fill(opts, ogeo, ncomp, nbytes, lam, bw, co.sigma, penalty=co.penalty)
    assert ml.tables == mo.tables and [c.theta_us for c in ml.comps] == [c.theta for c in mo.comps]
    rng = np.random.default_rng(5)
    for _ in range(50):
        cfgs = [points[int(rng.integers(0, len(points)))] for _ in range(ncomm)]
        pl, po = lg.lagom_cost_model(ml, cfgs), ocm.predict(mo, cfgs)
        assert pl.x_us == po.x and pl.y_us == po.y and pl.g == po.g and (pl.X_us, pl.Y_us, pl.Z_us) == (po.X, po.Y, po.Z)
    # and the search driven by that model, library against oracle on the oracle's own model
    sl = [lg.Space(NC, NT, CH) for _ in range(ncomm)]
    so = [osr.Space(NC, NT, CH) for _ in range(ncomm)]
    oprof = lambda cfgs: (lambda p: (p.x, p.Y))(ocm.predict(mo, cfgs))
    for mode, fn in [(lg.LAGOM_PRIORITY, osr.priority_search), (lg.LAGOM_EXHAUSTIVE, osr.brute_force), (lg.LAGOM_HIDE_COMM, osr.hide_search)]:
        rl, ro = lg.lagom_tune(sl, ml, mode), fn(so, oprof)
        assert rl.cfgs == ro.cfgs and (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z) and rl.calls == ro.calls
