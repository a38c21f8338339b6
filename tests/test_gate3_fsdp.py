"""The tuner's choice against brute force on the first three pairs of the FSDP chain, driven by the cost model filled
from a recorded sweep of that chain (tests/golden/fsdp_chain_sweep.json: timings, input data).  Library and oracle are
run side by side from the same table; the comparison with brute force is asserted where it holds and bounded and
printed where it does not (the search is a heuristic for N >= 2: Sec. 3.3-3.4 make no optimality claim beyond "can find
the optimal configuration", Sec. 4.4)."""
import json
import os

import pytest

from oracle import cost_model as ocm, model_fill as omf, search as osr
from paper_2602_20656_amd import binding as lg


@pytest.fixture(scope="module")
def table(golden_dir):
    t = json.load(open(os.path.join(golden_dir, "fsdp_chain_sweep.json")))
    total = float(sum(t["bytes_per_comm"]))
    for p in t["points"]:
        p["v_corun"] = total / p["comm_corun_us"]
        p["v_alone"] = total / p["comm_alone_us"]
    return t


def _models(t, d_key, sigmas, rhos=None):
    geo, lam, bw = t["geometry"], t["lambda"], t["bw_peak_bytes_per_us"]
    usable = [p for p in t["points"] if p["cfg"][0] < lam]
    lpts = [lg.SweepPoint(tuple(p["cfg"]), p["comm_alone_us"], p["comm_corun_us"], p["comp_alone_us"], p["comp_corun_us"],
                          p["z_corun_us"], p["v_alone"], p["v_corun"]) for p in usable]
    opts = [omf.SweepPoint(tuple(p["cfg"]), p["comm_corun_us"], p["comp_alone_us"], p["comp_corun_us"], p["v_corun"]) for p in usable]
    ogeo = omf.Geometry(geo["mu"], geo["tb"], geo[d_key])
    cl = lg.lagom_model_calibrate(lpts, lam, bw, geo["mu"], geo["tb"], geo[d_key], t["ncomp"], t["bytes_per_comm"], sigmas,
                                  rhos=rhos)
    co = omf.calibrate(opts, None, ogeo, t["ncomp"], t["bytes_per_comm"], lam, bw, sigmas, rhos=rhos)
    assert (cl.sigma, cl.fit_mean, cl.fit_max, cl.penalty) == (co.sigma, co.fit_mean, co.fit_max, co.penalty)
    ml, _ = lg.lagom_model_fill(lpts, lam, bw, geo["mu"], geo["tb"], geo[d_key], t["ncomp"], t["bytes_per_comm"], corun_share=cl.sigma,
                                resident_penalty=cl.penalty)
    mo = omf.fill(opts, ogeo, t["ncomp"], t["bytes_per_comm"], lam, bw, co.sigma, penalty=co.penalty)
    assert ml.tables == mo.tables
    # the first three pairs
    ml3 = lg.Model(ml.lam, ml.bw_peak, ml.comps[:3], ml.tables[:3], corun_share=ml.corun_share, resident_penalty=ml.resident_penalty)
    mo3 = ocm.Model(mo.lam, mo.bw_peak, mo.comps[:3], mo.tables[:3], corun_share=mo.corun_share, resident_penalty=mo.resident_penalty)
    return ml3, mo3, cl


def _ladder(t):
    per_src = t["per_src_bytes"][0]
    chunks = lg.lagom_ladder_chunks(t["chunk_grid"], max(t["nc_grid"]), 256, per_src, lg.LAGOM_LADDER_CUT)
    assert chunks == osr.ladder_chunks(t["chunk_grid"], max(t["nc_grid"]), 256, per_src, osr.LADDER_CUT)
    return t["nc_grid"][:6], chunks[:6]


@pytest.mark.parametrize("which", ["calibrated", "calibrated_with_penalty", "as_printed"])
def test_priority_against_brute_force_on_the_first_three_pairs(table, which):
    sigmas = [i / 8 for i in range(9)] if which != "as_printed" else [0.0]
    rhos = [0.0, 0.02, 0.05, 0.1, 0.15, 0.2, 0.3] if which == "calibrated_with_penalty" else None
    ml3, mo3, cal = _models(table, "d_bytes_past_l2" if which != "as_printed" else "d_bytes", sigmas, rhos)
    nc, chunks = _ladder(table)
    sl = [lg.Space(nc, [256], chunks) for _ in range(3)]
    so = [osr.Space(nc, [256], chunks) for _ in range(3)]
    oprof = lambda cfgs: (lambda p: (p.x, p.Y))(ocm.predict(mo3, cfgs))
    res = {}
    for name, mode, fn in [("priority", lg.LAGOM_PRIORITY, osr.priority_search), ("exhaustive", lg.LAGOM_EXHAUSTIVE, osr.brute_force),
                           ("priority_free", lg.LAGOM_PRIORITY_FREE, lambda s, p: osr.priority_search(s, p, free_steps=True))]:
        rl, ro = lg.lagom_tune(sl, ml3, mode), fn(so, oprof)
        # Gates 1 and 2 on real data: the library's search is the oracle's search
        assert rl.cfgs == ro.cfgs and rl.levels == ro.levels and rl.calls == ro.calls and (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)
        res[name] = rl
    pr, ex, fr = res["priority"], res["exhaustive"], res["priority_free"]
    assert ex.calls == 6 ** 3 and pr.calls <= 1 + 3 * 6 and fr.calls <= 1 + 3 * 6
    assert ex.Z <= pr.Z and ex.Z <= fr.Z                       # brute force is the lower bound
    gap, gap_free = pr.Z / ex.Z - 1.0, fr.Z / ex.Z - 1.0
    same = sorted(pr.cfgs) == sorted(ex.cfgs)                  # the three pairs are identical: order is immaterial
    print(f"\n[{which}, sigma {cal.sigma}, penalty {cal.penalty}, mean Y error {cal.fit_mean:.4f}] priority {pr.cfgs} Z={pr.Z:.2f} us ({pr.calls} calls) | exhaustive {ex.cfgs} "
          f"Z={ex.Z:.2f} us ({ex.calls} calls) | gap {100 * gap:.2f} % | same up to order: {same} | "
          f"free steps {fr.cfgs} Z={fr.Z:.2f} us, gap {100 * gap_free:.2f} %")
    # Gate 3 on this chain is not an identity: under the model filled from the recorded sweep the heuristic stops as soon
    # as the communication is hidden, while the model (like the hardware it was filled from) still rewards faster
    # communication with a shorter computation.  What holds with the calibrated model, and is asserted: it ends within
    # 2 % of the optimum with at most 19 of 216 calls.  With the model as printed (every byte of a workgroup charged to
    # HBM, a channel taking a whole compute unit) the predicted computation is so long that the walk stops almost at
    # once; the gap (30 % on the recorded table) is printed, not gated.  With the resident penalty calibrated as well
    # the model follows the recorded Y four times more closely (mean error 0.029 against 0.115), and the closer it
    # follows it the more the early stop costs: 8.8 % on the recorded table, printed, not gated -- the same order as
    # the gap measured on the hardware between the priority search and the exhaustive search over this ladder.
    if which == "calibrated":
        assert gap <= 0.02 and gap_free <= 0.02
    if gap == 0.0:
        assert same


def test_resident_penalty_on_the_recorded_extended_sweep(golden_dir):
    """The recorded sweep with channels of 128 and of 256 threads and up to 256 of them: sigma, then rho per thread count,
    fitted on every second point and scored on the others, library and oracle side by side.  On these recorded timings
    the penalty cuts the held-out error of Y to less than half, the heavier channel gets the larger penalty, and the
    model's choice among the swept points moves from a mid-field point to one within 2 % of the best measured one."""
    t = json.load(open(os.path.join(golden_dir, "fsdp_chain_sweep_extended.json")))
    total = float(sum(t["bytes_per_comm"]))
    geo, lam, bw, ncomp, nbytes = t["geometry"], t["lambda"], t["bw_peak_bytes_per_us"], t["ncomp"], t["bytes_per_comm"]
    usable = [p for p in t["points"] if p["cfg"][0] < lam]
    lpts = [lg.SweepPoint(tuple(p["cfg"]), p["comm_alone_us"], p["comm_corun_us"], p["comp_alone_us"], p["comp_corun_us"],
                          p["z_corun_us"], total / p["comm_alone_us"], total / p["comm_corun_us"]) for p in usable]
    opts = [omf.SweepPoint(p.cfg, p.comm_corun_us, p.comp_alone_us, p.comp_corun_us, p.v_corun) for p in lpts]
    ogeo = omf.Geometry(geo["mu"], geo["tb"], geo["d_bytes_past_l2"])
    held = [i % 2 == 1 for i in range(len(lpts))]
    sigmas = [i / 8 for i in range(9)]
    rhos = [0.0, 0.01, 0.02, 0.03, 0.04, 0.05, 0.06, 0.08, 0.1, 0.125, 0.15, 0.2, 0.25, 0.3, 0.4, 0.5]
    res = {}
    for label, use in (("sigma", None), ("sigma_rho", rhos)):
        cl = lg.lagom_model_calibrate(lpts, lam, bw, geo["mu"], geo["tb"], geo["d_bytes_past_l2"], ncomp, nbytes, sigmas, held, rhos=use)
        co = omf.calibrate(opts, held, ogeo, ncomp, nbytes, lam, bw, sigmas, rhos=use)
        assert (cl.sigma, cl.fit_mean, cl.fit_max, cl.held_mean, cl.held_max, cl.penalty) == \
            (co.sigma, co.fit_mean, co.fit_max, co.held_mean, co.held_max, co.penalty)
        model, _ = lg.lagom_model_fill(lpts, lam, bw, geo["mu"], geo["tb"], geo["d_bytes_past_l2"], ncomp, nbytes,
                                       corun_share=cl.sigma, resident_penalty=cl.penalty)
        z = {p.cfg: lg.lagom_cost_model(model, [p.cfg] * len(nbytes)).Z_us for p in lpts}
        pick = min(lpts, key=lambda p: z[p.cfg])
        best = min(lpts, key=lambda p: p.z_corun_us)
        res[label] = (cl, pick, best)
        print(f"\n[{label}] sigma {cl.sigma} penalty {cl.penalty}: Y error fitted {cl.fit_mean:.4f} held out {cl.held_mean:.4f} (max {cl.held_max:.4f}); "
              f"picks {pick.cfg} measured {pick.z_corun_us:.1f} us, best measured {best.cfg} {best.z_corun_us:.1f} us")
    plain, pen = res["sigma"][0], res["sigma_rho"][0]
    assert sorted(pen.penalty) == [128, 256] and pen.penalty[256] > pen.penalty[128] > 0.0
    assert pen.held_mean < 0.5 * plain.held_mean and pen.held_max < plain.held_max
    pick, best = res["sigma_rho"][1], res["sigma_rho"][2]
    assert pick.z_corun_us <= 1.02 * best.z_corun_us
    assert res["sigma"][1].z_corun_us > 1.05 * best.z_corun_us
