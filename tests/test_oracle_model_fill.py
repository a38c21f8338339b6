"""Pins for oracle/model_fill.py: pencil-worked numbers for theta (Eq. 5-6 solved for the standalone run), the tables
and the choice of the co-run share; the round trip "a filled model predicts the standalone time it was fitted to";
a planted share recovered.  The paper prints no numbers for these steps; the pencil work is in the comments."""
import math

import numpy as np
import pytest

from oracle import cost_model as cm, model_fill as mf

GEO = mf.Geometry(mu=20, tb=2, d_bytes=1000.0)     # lambda = 4 below: 8 workgroups in flight, 3 waves
LAM, BW = 4, 100.0                                  # lambda * TB * D / B = 8 * 1000 / 100 = 80 us per wave of traffic


def _pt(cfg, xc, alone, corun, v):
    return mf.SweepPoint(cfg, xc, alone, corun, v)


def test_median_and_standalone_time():
    assert mf.median([330.0, 300.0, 360.0]) == 330.0
    assert mf.median([300.0, 400.0, 330.0, 360.0]) == 345.0
    pts = [_pt((1, 64, 16), 1.0, a, 1.0, 1.0) for a in (990.0, 900.0, 1080.0)]
    assert mf.t_alone(pts, 3) == 330.0
    with pytest.raises(ValueError):
        mf.median([])


def test_theta_pencil_cases():
    # g0 = ceil(20 / 8) = 3 waves; 330 / 3 = 110 per wave; minus 80 of traffic -> theta = 30
    assert mf.fit_theta(330.0, GEO, LAM, BW) == 30.0
    # 150 / 3 = 50 < 80: the traffic term alone exceeds the measured wave -> floored at 0
    assert mf.fit_theta(150.0, GEO, LAM, BW) == 0.0
    # one wave exactly: mu = 8 -> g0 = 1 -> theta = 200 - 80
    assert mf.fit_theta(200.0, mf.Geometry(8, 2, 1000.0), LAM, BW) == 120.0
    # mu = 9 spills into a second wave: g0 = 2 -> theta = 100 - 80
    assert mf.fit_theta(200.0, mf.Geometry(9, 2, 1000.0), LAM, BW) == 20.0


def test_tables_pencil_cases():
    pts = [_pt((2, 64, 16), 40.0, 330.0, 350.0, 10.0), _pt((4, 64, 32), 20.0, 330.0, 380.0, 120.0)]
    assert mf.shares([300.0, 100.0]) == [0.75, 0.25]
    t = mf.fill_tables(pts, [300.0, 100.0], BW)
    assert t[0][(2, 64, 16)] == (30.0, 10.0) and t[1][(2, 64, 16)] == (10.0, 10.0)
    # V = 120 >= B: capped at 0.99 * B so that Eq. 6's denominator stays positive
    assert t[0][(4, 64, 32)] == (15.0, 99.0) and t[1][(4, 64, 32)] == (5.0, 99.0)
    for p in pts:                                           # the parts add up to the measured whole
        assert t[0][p.cfg][0] + t[1][p.cfg][0] == p.comm_corun_us
    with pytest.raises(ValueError):
        mf.shares([0.0, 0.0])


def test_filled_model_returns_the_standalone_time_it_was_fitted_to():
    rng = np.random.default_rng(9)
    for _ in range(200):
        lam = int(rng.integers(2, 300)); tb = int(rng.integers(1, 4))
        geo = mf.Geometry(int(rng.integers(1, 5000)), tb, float(rng.uniform(1e3, 1e6)))
        bw = float(rng.uniform(1e5, 8e6))
        ncomp = int(rng.integers(1, 5))
        alone = float(rng.uniform(50.0, 5000.0)) * ncomp
        # the communication lasts no time at all, so every wave runs without it
        pts = [_pt((1, 64, 16), 0.0, alone, alone, 0.0)]
        model = mf.fill(pts, geo, ncomp, [1.0], lam, bw)
        pred = cm.predict(model, [(1, 64, 16)])
        if model.comps[0].theta > 0.0:
            assert pred.Y == pytest.approx(alone, rel=1e-12)
        else:                                               # floored: the traffic term alone is already longer
            assert pred.Y >= alone * (1 - 1e-12)


def test_calibration_pencil_case():
    # One fitted point: the communication (NC = 2, V = 10) covers the whole computation (x = 1000 us); theta = 30 from 330.
    #   sigma 0   : 4 in flight -> 5 waves of 30 + 4000/90 = 74.444 -> 372.22; |.-400|/400 = 0.069444
    #   sigma 0.5 : floor((4 - 1) * 2) = 6 -> waves 6,6,6,2 -> 4 of 30 + 6000/90 = 96.667 -> 386.667; error 0.033333
    #   sigma 1   : 8 in flight -> 3 waves of 30 + 8000/90 = 118.889 -> 356.667; error 0.108333
    fit = _pt((2, 64, 16), 1000.0, 330.0, 400.0, 10.0)
    # Held out (its standalone time must not move theta): NC = 1, V = 20, sigma 0.5 -> floor(3.5 * 2) = 7 -> waves 7,7,6
    # -> 3 of 30 + 7000/80 = 117.5 -> 352.5; measured 350 -> 2.5/350
    held = _pt((1, 64, 16), 1000.0, 500.0, 350.0, 20.0)
    c = mf.calibrate([fit, held], [False, True], GEO, 1, [4000.0], LAM, BW, [0.0, 0.5, 1.0])
    assert c.sigma == 0.5 and (c.n_fit, c.n_held) == (1, 1)
    assert c.fit_mean == pytest.approx(1.0 / 30.0, rel=1e-12) and c.fit_max == c.fit_mean
    assert c.held_mean == pytest.approx(2.5 / 350.0, rel=1e-12) and c.held_max == c.held_mean
    errs = [mf.y_errors(mf.fill([fit, held], GEO, 1, [4000.0], LAM, BW, s, theta_points=[fit]), [fit])[0] for s in (0.0, 0.5, 1.0)]
    assert errs == pytest.approx([0.0694444444444, 0.0333333333333, 0.1083333333333], rel=1e-9)
    # ties go to the first candidate; nothing held out reports zeros there
    same = mf.calibrate([fit], None, GEO, 1, [4000.0], LAM, BW, [0.5, 0.5, 0.0])
    assert same.sigma == 0.5 and (same.held_mean, same.held_max, same.n_held) == (0.0, 0.0, 0)
    with pytest.raises(ValueError):
        mf.calibrate([fit], [True], GEO, 1, [4000.0], LAM, BW, [0.0])


def test_calibration_recovers_a_planted_share():
    rng = np.random.default_rng(31)
    sigmas = [i / 8 for i in range(9)]
    found = 0
    for _ in range(40):
        planted = float(rng.choice(sigmas))
        lam, geo, bw = 256, mf.Geometry(int(rng.integers(300, 1500)), 1, float(rng.uniform(2e5, 1e6))), 8e6
        theta = float(rng.uniform(20.0, 100.0))
        g0 = -(-geo.mu // lam)
        alone = g0 * (theta + lam * geo.d_bytes / bw)
        truth = cm.Model(lam, bw, [cm.Comp(geo.mu, 1, geo.d_bytes, theta)], [{}], corun_share=planted)
        pts = []
        for nc in (8, 32, 64, 128):
            for c in (1 << 16, 1 << 18):
                cfg, v, xc = (nc, 256, c), float(rng.uniform(1e5, 4e6)), 1e9
                truth.tables[0][cfg] = (xc, v)
                pts.append(_pt(cfg, xc, alone, cm.predict(truth, [cfg]).Y, v))
        held = [i % 2 == 1 for i in range(len(pts))]
        c = mf.calibrate(pts, held, geo, 1, [1.0], lam, bw, sigmas)
        assert c.fit_mean <= 1e-9 and c.held_mean <= 1e-9      # the planted share (or one that gives the same waves) fits exactly
        truth.corun_share = c.sigma
        assert all(cm.predict(truth, [p.cfg]).Y == pytest.approx(p.comp_corun_us, rel=1e-9) for p in pts)
        found += c.sigma == planted
    assert found >= 20                                          # distinct shares can give identical wave counts; most are identified


def test_penalty_calibration_pencil_case_and_planted_values():
    # The pencil case of the share calibration, continued: with sigma = 0.5 the fitted point predicts 386.667 against 400
    # measured.  rho candidates 0, 0.05, 0.1: 386.667 -> error 1/30; 386.667 * 1.05 = 406 -> 6/400 = 0.015; * 1.1 = 425.33 ->
    # 0.0633.  rho(64) = 0.05.  The held-out point (NT 64 too): 352.5 * 1.05 = 370.125 against 350 -> 0.0575.
    fit = _pt((2, 64, 16), 1000.0, 330.0, 400.0, 10.0)
    held = _pt((1, 64, 16), 1000.0, 500.0, 350.0, 20.0)
    c = mf.calibrate([fit, held], [False, True], GEO, 1, [4000.0], LAM, BW, [0.0, 0.5, 1.0], rhos=[0.0, 0.05, 0.1])
    assert c.sigma == 0.5 and c.penalty == {64: 0.05}
    assert c.fit_mean == pytest.approx(6.0 / 400.0, rel=1e-9) and c.held_mean == pytest.approx(20.125 / 350.0, rel=1e-9)
    # planted: two thread counts with different penalties, recovered exactly from points the planted model produced
    rng = np.random.default_rng(77)
    rhos = [i / 50 for i in range(16)]
    for _ in range(20):
        lam, geo, bw = 256, mf.Geometry(int(rng.integers(300, 1500)), 1, float(rng.uniform(2e5, 1e6))), 8e6
        theta = float(rng.uniform(20.0, 100.0))
        alone = -(-geo.mu // lam) * (theta + lam * geo.d_bytes / bw)
        planted = {128: float(rng.choice(rhos)), 256: float(rng.choice(rhos))}
        truth = cm.Model(lam, bw, [cm.Comp(geo.mu, 1, geo.d_bytes, theta)], [{}], corun_share=1.0, resident_penalty=planted)
        pts = []
        for nt in (128, 256):
            for nc in (8, 32, 128):
                cfg, v, xc = (nc, nt, 1 << 16), float(rng.uniform(1e5, 4e6)), 1e9
                truth.tables[0][cfg] = (xc, v)
                pts.append(_pt(cfg, xc, alone, cm.predict(truth, [cfg]).Y, v))
        c = mf.calibrate(pts, [i % 3 == 2 for i in range(len(pts))], geo, 1, [1.0], lam, bw, [1.0], rhos=rhos)
        assert c.penalty == planted and c.fit_mean <= 1e-9 and c.held_mean <= 1e-9
    # without candidates nothing changes
    assert mf.calibrate([fit], None, GEO, 1, [4000.0], LAM, BW, [0.5]).penalty is None
