"""Pins for oracle/cost_model.py: hand-worked fixtures, closed forms and invariants of
the paper's Eq. 1-6."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import cost_model as cm


def _model(lam, bw, comps, comms):
    tables = [{(c["nc"], 256, 65536): (c["x"], c["v"])} for c in comms]
    return cm.Model(lam=lam, bw_peak=bw, comps=[cm.Comp(**c) for c in comps], tables=tables), \
        [(c["nc"], 256, 65536) for c in comms]


def test_hand_worked_fixture(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["cases"]:
        model, cfgs = _model(fx["lambda"], fx["bw_peak"], case["comps"], case["comms"])
        p = cm.predict(model, cfgs)
        assert p.y == case["y"], case["name"]
        assert p.g == case["g"], case["name"]
        assert (p.X, p.Y, p.Z) == (case["X"], case["Y"], case["Z"]), case["name"]


def test_single_comm_reduces_to_eq_4_5_6():
    lam, bw = 256, 8.0e6
    for nc, v, mu, tb in itertools.product([1, 8, 32, 200], [0.0, 1.0e6, 7.9e6], [1, 255, 1024, 5000], [1, 2]):
        theta, d = 12.5, 3.0e6
        g = math.ceil(mu / ((lam - nc) * tb))                              # Eq. 5
        f = theta + (lam - nc) * tb * d / (bw - v)                         # Eq. 6
        model = cm.Model(lam, bw, [cm.Comp(mu, tb, d, theta)], [{(nc, 256, 4096): (1e12, v)}])
        p = cm.predict(model, [(nc, 256, 4096)])
        assert p.g[0][0] == g and p.g[0][1] == 0
        assert p.y[0] == pytest.approx(f * g, rel=1e-15)                   # Eq. 4
        assert cm.wave_count(mu, lam, nc, tb) == g
        assert p.Z == 1e12 and p.X == 1e12                                 # Eq. 1, communication-bound


def test_no_comm_is_textbook_wave_quantisation():
    lam, bw = 256, 8.0e6
    for mu, tb in [(1, 1), (256, 1), (257, 1), (1024, 2), (1025, 2)]:
        model = cm.Model(lam, bw, [cm.Comp(mu, tb, 1.0e6, 3.0)], [])
        p = cm.predict(model, [])
        want = math.ceil(mu / (lam * tb)) * (3.0 + lam * tb * 1.0e6 / bw)
        assert p.Y == pytest.approx(want, rel=1e-15) and p.X == 0.0 and p.Z == p.Y


def test_eq1_and_monotone_invariants():
    lam, bw = 64, 1000.0
    comps = [cm.Comp(300, 2, 50.0, 2.0), cm.Comp(100, 1, 80.0, 1.0)]
    ncs, vs = [1, 2, 4, 8, 16, 32], [0.0, 100.0, 400.0, 900.0]
    for nc in ncs:
        prev = None
        for v in vs:
            table = {(nc, 64, 1024): (1e9, v)}
            p = cm.predict(cm.Model(lam, bw, comps, [table]), [(nc, 64, 1024)])
            assert p.Z == max(p.X, p.Y) and p.Y == sum(p.y)       # Eq. 1
            if prev is not None:
                assert p.Y > prev                                 # strictly slower as V grows (Eq. 6)
            prev = p.Y
    # In NC the printed Eq. 6 charges every wave, also the partial last one, the bytes of a full wave,
    # so y is monotone in NC only without a partial wave: mu a multiple of every (lambda - NC) * TB.
    comps = [cm.Comp(192, 1, 50.0, 2.0)]
    prev = cm.predict(cm.Model(lam, bw, comps, []), []).Y
    for nc in (16, 32, 48):
        table = {(nc, 64, 1024): (1e9, 100.0)}
        p = cm.predict(cm.Model(lam, bw, comps, [table]), [(nc, 64, 1024)])
        assert p.Y > prev
        prev = p.Y


def test_eq2_separability_when_communication_bound():
    # if X >= Y for every configuration, the best Z is the sum of the per-communication minima (Eq. 2)
    lam, bw = 32, 1000.0
    comps = [cm.Comp(10, 1, 1.0, 0.5)]
    cfgs = [(1, 64, 1024), (2, 64, 1024), (4, 64, 1024)]
    t0 = {cfgs[0]: (900.0, 10.0), cfgs[1]: (500.0, 20.0), cfgs[2]: (650.0, 30.0)}
    t1 = {cfgs[0]: (800.0, 10.0), cfgs[1]: (700.0, 20.0), cfgs[2]: (300.0, 30.0)}
    model = cm.Model(lam, bw, comps, [t0, t1])
    best = min(cm.predict(model, [a, b]).Z for a in cfgs for b in cfgs)
    assert best == min(x for x, _ in t0.values()) + min(x for x, _ in t1.values())


def test_rejects_out_of_range_inputs():
    comps = [cm.Comp(10, 1, 1.0, 0.5)]
    with pytest.raises(ValueError):
        cm.predict(cm.Model(8, 100.0, comps, [{(8, 64, 64): (1.0, 1.0)}]), [(8, 64, 64)])     # NC >= lambda
    with pytest.raises(ValueError):
        cm.predict(cm.Model(8, 100.0, comps, [{(2, 64, 64): (1.0, 100.0)}]), [(2, 64, 64)])   # V >= B
    with pytest.raises(KeyError):
        cm.predict(cm.Model(8, 100.0, comps, [{(2, 64, 64): (1.0, 1.0)}]), [(4, 64, 64)])     # not in the table


# ------------------------------------------------------------ dependent chains (Sec. 2.1 patterns)
def test_dependent_chains_hand_worked_fixture(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["dependent_cases"]:
        model, cfgs = _model(fx["lambda"], fx["bw_peak"], case["comps"], case["comms"])
        p = cm.predict(model, cfgs, case["comp_after_comm"], case["comm_after_comp"])
        assert p.y == case["y"] and p.g == case["g"], case["name"]
        assert (p.X, p.Y, p.Z) == (case["X"], case["Y"], case["Z"]), case["name"]


def test_dependencies_that_bind_nothing_change_nothing_and_real_ones_never_shorten_the_makespan():
    import numpy as np
    rng = np.random.default_rng(5)
    for _ in range(200):
        N, M = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        lam, bw = 64, 1000.0
        comps = [cm.Comp(int(rng.integers(1, 400)), int(rng.integers(1, 3)), float(rng.uniform(1, 200)), float(rng.uniform(0, 5))) for _ in range(M)]
        tables = [{(int(rng.choice([1, 4, 16])), 64, 1024): (float(rng.uniform(1, 300)), float(rng.uniform(0, 900)))} for _ in range(N)]
        model = cm.Model(lam, bw, comps, tables)
        cfgs = [next(iter(t)) for t in tables]
        free = cm.predict(model, cfgs)
        none = cm.predict(model, cfgs, [-1] * M, [-1] * N)
        assert (none.y, none.g, none.X, none.Y, none.Z) == (free.y, free.g, free.X, free.Y, free.Z)
        cac = [int(rng.integers(-1, min(i + 1, N))) for i in range(M)]          # comp i may wait for comm <= i
        cap = [int(rng.integers(-1, min(j, M))) if j > 0 else -1 for j in range(N)]   # comm j may wait for comp < j
        dep = cm.predict(model, cfgs, cac, cap)
        assert dep.X == free.X                                   # x_j are table values
        assert dep.Z >= max(dep.X, dep.Y) - 1e-9                 # waiting only adds idle time
        assert dep.Z >= min(free.Z, dep.Z)                       # and every wave count is still Eq. 5's
        for i, comp in enumerate(comps):
            assert sum(dep.g[i]) >= math.ceil(comp.mu / (lam * comp.tb))


def test_dependency_cycle_is_rejected():
    model = cm.Model(8, 100.0, [cm.Comp(10, 1, 1.0, 0.5)], [{(2, 64, 64): (5.0, 1.0)}])
    with pytest.raises(ValueError):
        cm.predict(model, [(2, 64, 64)], [0], [0])       # each waits for the other


# ------------------------------------------------------------------ co-run share (not in the paper)
def test_corun_share_hand_worked_fixture(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["corun_share_cases"]:
        model, cfgs = _model(fx["lambda"], fx["bw_peak"], case["comps"], case["comms"])
        model.corun_share = case["corun_share"]
        p = cm.predict(model, cfgs)
        assert p.y == case["y"] and p.g == case["g"], case["name"]
        assert (p.X, p.Y, p.Z) == (case["X"], case["Y"], case["Z"]), case["name"]


def test_corun_share_zero_is_the_printed_model_and_one_removes_the_channel_count():
    lam, bw = 256, 8.0e6
    for nc, v, mu, tb in itertools.product([1, 8, 32, 200], [0.0, 1.0e6, 7.9e6], [1, 255, 1024, 5000], [1, 2]):
        comp = cm.Comp(mu, tb, 3.0e6, 12.5)
        table = {(nc, 256, 4096): (1e12, v)}
        printed = cm.predict(cm.Model(lam, bw, [comp], [table]), [(nc, 256, 4096)])
        zero = cm.predict(cm.Model(lam, bw, [comp], [table], corun_share=0.0), [(nc, 256, 4096)])
        assert (zero.y, zero.g) == (printed.y, printed.g)
        one = cm.predict(cm.Model(lam, bw, [comp], [table], corun_share=1.0), [(nc, 256, 4096)])
        g = math.ceil(mu / (lam * tb))                                      # Eq. 5 with no compute unit taken
        f = 12.5 + lam * tb * 3.0e6 / (bw - v)                              # Eq. 6, bandwidth term only
        assert one.g[0][0] == g and one.y[0] == pytest.approx(f * g, rel=1e-15)
        assert cm.workgroups_in_flight(lam, nc, tb, 1.0) == lam * tb
        # in between, the workgroups in flight grow with the share and stay within the two ends
        caps = [cm.workgroups_in_flight(lam, nc, tb, s / 8) for s in range(9)]
        assert caps == sorted(caps) and caps[0] == (lam - nc) * tb and caps[-1] == lam * tb


def test_corun_share_out_of_range_is_rejected():
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(ValueError):
            cm.predict(cm.Model(8, 100.0, [cm.Comp(10, 1, 1.0, 1.0)], [{(2, 64, 64): (1.0, 1.0)}], corun_share=bad), [(2, 64, 64)])


def test_resident_penalty_pencil_cases_and_neutral_element(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["resident_penalty_cases"]:
        model, cfgs = _model(fx["lambda"], fx["bw_peak"], case["comps"], case["comms"])
        model.corun_share = case["corun_share"]
        model.resident_penalty = {int(k): v for k, v in case["penalty"].items()}
        p = cm.predict(model, cfgs)
        assert p.y == case["y"] and p.g == case["g"], case["name"]
        assert (p.X, p.Y, p.Z) == (case["X"], case["Y"], case["Z"]), case["name"]
    # rho = 0 and an empty map are the printed model bit for bit; Y grows with rho; waves after the last communication never pay
    rng = np.random.default_rng(5)
    for _ in range(100):
        lam, bw = 64, float(rng.uniform(1e3, 1e6))
        comps = [cm.Comp(int(rng.integers(1, 900)), 1, float(rng.uniform(1e2, 1e5)), float(rng.uniform(1, 50))) for _ in range(int(rng.integers(1, 4)))]
        tables = [{(4, 256, 64): (float(rng.uniform(0, 300)), float(rng.uniform(0, 0.5 * bw)))} for _ in range(int(rng.integers(1, 4)))]
        cfgs = [(4, 256, 64)] * len(tables)
        base = cm.predict(cm.Model(lam, bw, comps, tables), cfgs)
        zero = cm.predict(cm.Model(lam, bw, comps, tables, resident_penalty={256: 0.0}), cfgs)
        assert (zero.y, zero.g, zero.Z) == (base.y, base.g, base.Z)
        # under one communication that outlasts everything every wave pays: Y scales by exactly 1 + rho up to rounding.
        # (With communications that end inside a computation Y is not monotone in rho: longer waves shift later ones
        # past the end of a communication, where more workgroups fit in a wave.)
        long_tables = [{(4, 256, 64): (1e12, tables[0][(4, 256, 64)][1])}]
        b1 = cm.predict(cm.Model(lam, bw, comps, long_tables), cfgs[:1])
        s1 = cm.predict(cm.Model(lam, bw, comps, long_tables, resident_penalty={256: 0.25}), cfgs[:1])
        assert s1.g == b1.g and s1.Y == pytest.approx(1.25 * b1.Y, rel=1e-12)
        never = cm.predict(cm.Model(lam, bw, comps, [{(4, 256, 64): (0.0, 0.0)} for _ in tables], resident_penalty={256: 0.25}), cfgs)
        alone = cm.predict(cm.Model(lam, bw, comps, [{(4, 256, 64): (0.0, 0.0)} for _ in tables]), cfgs)
        assert never.y == alone.y                      # communications of no duration: no wave is issued under one
    with pytest.raises(ValueError):
        cm.predict(cm.Model(64, 1e3, [cm.Comp(10, 1, 1.0, 1.0)], [{(4, 256, 64): (5.0, 1.0)}], resident_penalty={256: -0.1}), [(4, 256, 64)])
