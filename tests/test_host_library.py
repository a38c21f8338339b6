"""Host-side checks that need no GPU: the C-ABI library loads and exports what the header
declares, and its cost model and tuner equal the oracle bit for bit."""
import json
import math
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import cost_model as ocm, model_fill as omf, search as osr
from paper_2602_20656_amd import binding as lg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lagom.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lagom_[a-z_]+)\s*\(", header)) - {"lagom_profile_fn"}
    assert {"lagom_comm_kernel", "lagom_gemm", "lagom_overlap_run", "lagom_cost_model", "lagom_tune"} <= declared
    L = lg.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert set(lg.EXPORTS) == declared
    assert L.lagom_strerror(lg.LAGOM_EALIGN).decode().startswith("device pointer")


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with no extensions and no C++."""
    src = tmp_path / "use_header.c"
    src.write_text('#include "lagom.h"\nint main(void) { lagom_cfg c = {1, 64, 16}; lagom_model m; (void)m; return c.nc - 1; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    "-c", str(src), "-o", str(tmp_path / "use_header.o")], check=True)


def test_host_only_helpers():
    assert lg.lagom_comm_bytes(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, 2, 1, 1 << 20) == 12 << 20
    assert lg.lagom_comm_bytes(lg.LAGOM_REDUCE_COPY, lg.LAGOM_BF16, 8, 1, 4194304) == 72 << 20
    assert lg.lagom_comm_bytes(lg.LAGOM_GATHER_COPY, lg.LAGOM_BF16, 8, 1, 2097152) == 64 << 20
    assert lg.lagom_comm_bytes(7, lg.LAGOM_BF16, 8, 1, 1) == -1
    g = lg.lagom_gemm_describe(8192, 8192, 8192)
    assert g.mu == (8192 // g.tile_m) * (8192 // g.tile_n) and g.tb >= 1
    assert g.d_bytes == (g.tile_m + g.tile_n) * 8192 * 2 + g.tile_m * g.tile_n * 2
    assert (g.tile_m, g.tile_n, g.tile_k) == (256, 256, 64)
    # at most 256 tiles of 128 x 128 (and K a multiple of 64): the small tiling
    few = lg.lagom_gemm_describe(100, 300, 64)
    assert (few.tile_m, few.tile_n, few.mu, few.tb) == (128, 128, 1 * 3, 1)
    assert few.d_bytes == (128 + 128) * 64 * 2 + 128 * 128 * 2
    assert lg.lagom_gemm_describe(2048, 2048, 4096).mu == 256
    mid = lg.lagom_gemm_describe(2048, 2176, 4096)             # 272 tiles of 128 x 128, 136 of 256 x 128
    assert (mid.tile_m, mid.tile_n, mid.mu) == (256, 128, 8 * 17)
    assert mid.d_bytes == (256 + 128) * 4096 * 2 + 256 * 128 * 2
    assert lg.lagom_gemm_describe(3072, 3072, 3072).tile_n == 256   # 288 tiles of 256 x 128: the large tiling
    assert lg.lagom_gemm_describe(512, 512, 72).tile_m == 128       # K need not be a multiple of 64 for that
    assert lg.lagom_gemm_describe(512, 512, 56).tile_m == 256       # K < 64: the general kernel's tiling
    # bytes past an XCD's L2: the 32 tiles an XCD holds at a time form an 8 x 4 block -> A panels shared by 4, B by 8
    for M, N, K in [(4096, 4096, 4096), (8192, 4096, 4096), (8192, 8192, 8192)]:
        assert lg.lagom_gemm_describe(M, N, K).d_bytes_past_l2 == (8 * 256 + 4 * 256) * K * 2 / 32 + 256 * 256 * 2
    small = lg.lagom_gemm_describe(512, 512, 512)          # 16 small tiles, two per XCD, in one tile-column: a B panel shared by 2
    assert small.d_bytes_past_l2 == (2 * 128 + 1 * 128) * 512 * 2 / 2 + 128 * 128 * 2
    lone = lg.lagom_gemm_describe(256, 256, 512)           # 4 tiles: nothing is shared
    assert lone.d_bytes_past_l2 == lone.d_bytes
    # 16 x 14 tiles: 28 per XCD at a time, 8 tile-rows x 4 tile-columns (the last one half full)
    assert lg.lagom_gemm_describe(4096, 3584, 8192).d_bytes_past_l2 == (8 * 256 + 4 * 256) * 8192 * 2 / 28 + 256 * 256 * 2


def test_argument_errors_are_reported_before_any_gpu_work():
    good = (4, 256, 65536)
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [4096, 8192], [16384], 100, (4, 100, 65536))
    assert e.value.code == lg.LAGOM_EINVAL
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [4096, 8200], [16384], 100, good)
    assert e.value.code == lg.LAGOM_EALIGN
    for bad in [(0, 256, 65536), (4, 2048, 65536), (4, 256, 24), (4, 256, 0)]:
        with pytest.raises(lg.LagomError):
            lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [4096], [16384], 100, bad)
    with pytest.raises(lg.LagomError):
        lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [4096] * 17, [16384], 100, good)
    with pytest.raises(lg.LagomError):
        lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [4096], [16384], -1, good)
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_gemm(4096, 8192, 16384, 64, 64, 12)          # K not a multiple of 8
    assert e.value.code == lg.LAGOM_EINVAL
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_gemm(4096, 8192 + 2, 16384, 64, 64, 64)
    assert e.value.code == lg.LAGOM_EALIGN
    # count == 0 is a no-op that touches no device
    lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [4096], [16384], 0, good)


# ------------------------------------------------------------------- cost model parity
def _random_model(rng, N, M):
    lam = int(rng.choice([8, 64, 256]))
    bw = float(rng.uniform(1e3, 8e6))
    comps_o, comps_l = [], []
    for _ in range(M):
        mu, tb = int(rng.integers(0, 3000)), int(rng.integers(1, 3))
        d, th = float(rng.uniform(0, 1e7)), float(rng.uniform(0, 50))
        comps_o.append(ocm.Comp(mu, tb, d, th)); comps_l.append(lg.CompModel(mu, tb, d, th))
    tables, cfgs = [], []
    for _ in range(N):
        t = {}
        for nc in (1, 2, 4):
            for c in (4096, 65536):
                t[(nc, 256, c)] = (float(rng.uniform(0, 400)), float(rng.uniform(0, 0.95 * bw)))
        tables.append(t)
        cfgs.append((int(rng.choice([1, 2, 4])), 256, int(rng.choice([4096, 65536]))))
    return ocm.Model(lam, bw, comps_o, tables), lg.Model(lam, bw, comps_l, tables), cfgs


def test_cost_model_equals_oracle_bit_for_bit():
    rng = np.random.default_rng(11)
    for _ in range(300):
        N, M = int(rng.integers(0, 5)), int(rng.integers(0, 5))
        mo, ml, cfgs = _random_model(rng, N, M)
        po, pl = ocm.predict(mo, cfgs), lg.lagom_cost_model(ml, cfgs)
        assert pl.x_us == po.x and pl.y_us == po.y and pl.g == po.g
        assert (pl.X_us, pl.Y_us, pl.Z_us) == (po.X, po.Y, po.Z)


def test_cost_model_with_a_corun_share_equals_oracle_bit_for_bit(golden_dir):
    rng = np.random.default_rng(12)
    for _ in range(300):
        N, M = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        mo, ml, cfgs = _random_model(rng, N, M)
        mo.corun_share = ml.corun_share = float(rng.choice([0.0, 0.125, 0.3, 0.5, 0.77, 1.0, rng.uniform(0, 1)]))
        po, pl = ocm.predict(mo, cfgs), lg.lagom_cost_model(ml, cfgs)
        assert pl.x_us == po.x and pl.y_us == po.y and pl.g == po.g
        assert (pl.X_us, pl.Y_us, pl.Z_us) == (po.X, po.Y, po.Z)
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["corun_share_cases"]:
        tables = [{(c["nc"], 256, 65536): (c["x"], c["v"])} for c in case["comms"]]
        model = lg.Model(fx["lambda"], fx["bw_peak"], [lg.CompModel(c["mu"], c["tb"], c["d_bytes"], c["theta"]) for c in case["comps"]],
                         tables, corun_share=case["corun_share"])
        p = lg.lagom_cost_model(model, [(c["nc"], 256, 65536) for c in case["comms"]])
        assert p.y_us == case["y"] and p.g == case["g"] and (p.X_us, p.Y_us, p.Z_us) == (case["X"], case["Y"], case["Z"])
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(lg.LagomError) as e:
            lg.lagom_cost_model(lg.Model(8, 100.0, [lg.CompModel(10, 1, 1.0, 1.0)], [{(2, 64, 64): (1.0, 1.0)}], corun_share=bad), [(2, 64, 64)])
        assert e.value.code == lg.LAGOM_EINVAL


def test_cost_model_with_a_resident_penalty_equals_oracle_bit_for_bit(golden_dir):
    rng = np.random.default_rng(13)
    for trial in range(300):
        N, M = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        mo, ml, cfgs = _random_model(rng, N, M)
        mo.corun_share = ml.corun_share = float(rng.choice([0.0, 0.25, rng.uniform(0, 1)]))
        pen = {int(nt): float(rng.choice([0.0, 0.05, rng.uniform(0, 0.5)])) for nt in rng.choice([128, 256, 512], size=int(rng.integers(0, 3)), replace=False)}
        mo.resident_penalty, ml.resident_penalty = dict(pen), dict(pen)
        if trial % 3 == 0:
            mo_dep = [int(rng.integers(-1, min(i + 1, N))) for i in range(M)]
            ml.comp_after_comm = mo_dep
            po = ocm.predict(mo, cfgs, mo_dep, None)
        else:
            po = ocm.predict(mo, cfgs)
        pl = lg.lagom_cost_model(ml, cfgs)
        assert pl.x_us == po.x and pl.y_us == po.y and pl.g == po.g
        assert (pl.X_us, pl.Y_us, pl.Z_us) == (po.X, po.Y, po.Z)
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["resident_penalty_cases"]:
        tables = [{(c["nc"], 256, 65536): (c["x"], c["v"])} for c in case["comms"]]
        model = lg.Model(fx["lambda"], fx["bw_peak"], [lg.CompModel(c["mu"], c["tb"], c["d_bytes"], c["theta"]) for c in case["comps"]],
                         tables, corun_share=case["corun_share"], resident_penalty={int(k): v for k, v in case["penalty"].items()})
        p = lg.lagom_cost_model(model, [(c["nc"], 256, 65536) for c in case["comms"]])
        assert p.y_us == case["y"] and p.g == case["g"] and (p.X_us, p.Y_us, p.Z_us) == (case["X"], case["Y"], case["Z"])
    for bad in (-0.1, float("nan")):
        with pytest.raises(lg.LagomError) as e:
            lg.lagom_cost_model(lg.Model(8, 100.0, [lg.CompModel(10, 1, 1.0, 1.0)], [{(2, 64, 64): (1.0, 1.0)}], resident_penalty={64: bad}), [(2, 64, 64)])
        assert e.value.code == lg.LAGOM_EINVAL


def test_cost_model_on_the_hand_worked_fixture(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["cases"]:
        tables = [{(c["nc"], 256, 65536): (c["x"], c["v"])} for c in case["comms"]]
        model = lg.Model(fx["lambda"], fx["bw_peak"], [lg.CompModel(c["mu"], c["tb"], c["d_bytes"], c["theta"]) for c in case["comps"]], tables)
        p = lg.lagom_cost_model(model, [(c["nc"], 256, 65536) for c in case["comms"]])
        assert p.y_us == case["y"] and p.g == case["g"] and (p.X_us, p.Y_us, p.Z_us) == (case["X"], case["Y"], case["Z"])


def test_cost_model_rejects_bad_input():
    comps = [lg.CompModel(10, 1, 1.0, 0.5)]
    for lam, table, cfg in [(8, {(8, 64, 64): (1.0, 1.0)}, (8, 64, 64)),        # NC >= lambda
                            (8, {(2, 64, 64): (1.0, 100.0)}, (2, 64, 64)),      # V >= B
                            (8, {(2, 64, 64): (1.0, 1.0)}, (4, 64, 64)),        # not in the table
                            (8, {(2, 64, 64): (-1.0, 1.0)}, (2, 64, 64))]:      # negative x
        with pytest.raises(lg.LagomError) as e:
            lg.lagom_cost_model(lg.Model(lam, 100.0, comps, [table]), [cfg])
        assert e.value.code == lg.LAGOM_EINVAL


# ------------------------------------------------------------------------ tuner parity
def _same_trace(lib_trace, oracle_trace):
    assert len(lib_trace) == len(oracle_trace)
    for a, b in zip(lib_trace, oracle_trace):
        assert (a.comm, a.level_from, a.level_to, a.accepted, a.done) == (b.comm, b.level_from, b.level_to, b.accepted, b.done)
        for u, v in [(a.xj_prev, b.xj_prev), (a.xj_new, b.xj_new), (a.X, b.X), (a.Y, b.Y), (a.Z, b.Z), (a.H, b.H), (a.lr, b.lr)]:
            assert (math.isnan(u) and math.isnan(v)) or u == v


def _random_chain(rng, N):
    spaces_o, spaces_l = [], []
    for _ in range(N):
        nc = sorted(set(int(v) for v in rng.choice([1, 2, 3, 4, 6, 8, 16, 32, 61], size=rng.integers(1, 6), replace=False)))
        nt = sorted(set(int(v) for v in rng.choice([64, 128, 256, 512, 1024], size=rng.integers(1, 4), replace=False)))
        ch = sorted(set(int(v) for v in rng.choice([16384, 32768, 65536, 700416, 1398784, 2097152], size=rng.integers(1, 5), replace=False)))
        spaces_o.append(osr.Space(nc, nt, ch)); spaces_l.append(lg.Space(nc, nt, ch))
    base = rng.uniform(5, 300, size=N)
    a = rng.uniform(0.2, 1.2, size=N)
    pen = rng.uniform(0, 3, size=N)
    y0 = float(rng.uniform(5, 400))
    bump = rng.uniform(0, 0.02, size=N)

    def profile(cfgs):
        x = [float(base[j] / (c[0] ** a[j]) * (1 + bump[j] * c[0]) + 1e-6 * c[2] / c[1]) for j, c in enumerate(cfgs)]
        Y = y0 + sum(float(pen[j]) * c[0] + 1e-6 * c[2] for j, c in enumerate(cfgs))
        return x, Y
    return spaces_o, spaces_l, profile


def test_priority_search_equals_oracle_result_and_trace():
    rng = np.random.default_rng(3)
    for _ in range(300):
        N = int(rng.integers(1, 9))
        so, sl, profile = _random_chain(rng, N)
        ro = osr.priority_search(so, profile)
        rl = lg.lagom_tune(sl, profile, lg.LAGOM_PRIORITY)
        assert rl.cfgs == ro.cfgs and rl.levels == ro.levels and rl.calls == ro.calls
        assert (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)
        _same_trace(rl.trace, ro.trace)
        assert rl.calls <= 1 + sum(sp.K for sp in so)


def test_exhaustive_equals_oracle_brute_force():
    rng = np.random.default_rng(4)
    for _ in range(60):
        N = int(rng.integers(1, 4))
        so, sl, profile = _random_chain(rng, N)
        ro = osr.brute_force(so, profile)
        rl = lg.lagom_tune(sl, profile, lg.LAGOM_EXHAUSTIVE)
        assert rl.cfgs == ro.cfgs and rl.levels == ro.levels and rl.calls == ro.calls and rl.Z == ro.Z
    # ties: constant profile -> all-zero levels
    sl = [lg.Space([1, 2, 4], [64], [16]), lg.Space([1, 2], [64], [16])]
    assert lg.lagom_tune(sl, lambda c: ([1.0, 1.0], 5.0), lg.LAGOM_EXHAUSTIVE).levels == [0, 0]


def test_tuner_on_the_hand_worked_fixture(golden_dir):
    fx = json.load(open(os.path.join(golden_dir, "search_worked.json")))
    for case in fx["cases"]:
        so = [osr.Space(**sp) for sp in case["spaces"]]
        sl = [lg.Space(**sp) for sp in case["spaces"]]
        xs, coef = case["x_by_level"], case["Y_coef"]

        def profile(cfgs):
            lv = [[so[j].cfg(l) for l in range(so[j].K)].index(tuple(c)) for j, c in enumerate(cfgs)]
            return [xs[j][l] for j, l in enumerate(lv)], coef[0] + sum(coef[1 + j] * l for j, l in enumerate(lv))
        r = lg.lagom_tune(sl, profile, lg.LAGOM_PRIORITY)
        assert r.levels == case["final_levels"] and r.Z == case["final_Z"] and r.calls == case["calls"]
        for got, want in zip(r.trace, case["trace"]):
            assert (got.comm, got.level_from, got.level_to, got.accepted, got.done) == \
                (want["comm"], want["from"], want["to"], want["accepted"], want["done"])
        b = lg.lagom_tune(sl, profile, lg.LAGOM_EXHAUSTIVE)
        assert b.levels == case["brute_levels"] and b.Z == case["brute_Z"]


def test_tuner_with_the_native_model_callback_matches_oracle_on_the_same_model():
    rng = np.random.default_rng(9)
    nc_grid, ch_grid = [1, 2, 4, 8, 16, 32], [32768 << i for i in range(8)]
    lam, bw = 256, 8.0e6
    for trial in range(20):
        N = int(rng.integers(1, 4))
        tables = []
        for j in range(N):
            t = {}
            work = float(rng.uniform(2e7, 2e8))
            for l in range(8):
                nc, ch = nc_grid[min(l, 5)], ch_grid[l]
                v = min(0.9 * bw, nc * 6.0e4 * (1 + 0.1 * l))
                t[(nc, 256, ch)] = (work / v, v)
            tables.append(t)
        comps_o = [ocm.Comp(1024, 1, 4.3e6, 20.0) for _ in range(N)]
        comps_l = [lg.CompModel(1024, 1, 4.3e6, 20.0) for _ in range(N)]
        mo, ml = ocm.Model(lam, bw, comps_o, tables), lg.Model(lam, bw, comps_l, tables)

        def profile(cfgs):
            p = ocm.predict(mo, cfgs)
            return p.x, p.Y
        so = [osr.Space(nc_grid, [256], ch_grid) for _ in range(N)]
        sl = [lg.Space(nc_grid, [256], ch_grid) for _ in range(N)]
        for mode, oracle_fn in [(lg.LAGOM_PRIORITY, osr.priority_search), (lg.LAGOM_EXHAUSTIVE, osr.brute_force)]:
            ro, rl = oracle_fn(so, profile), lg.lagom_tune(sl, ml, mode)
            assert rl.cfgs == ro.cfgs and rl.Z == ro.Z and rl.calls == ro.calls


def test_callback_failure_returns_best_so_far():
    calls = []

    def profile(cfgs):
        calls.append(cfgs)
        if len(calls) == 3:
            raise RuntimeError("boom")
        return [100.0 / c[0] for c in cfgs], 1.0
    sl = [lg.Space([1, 2, 4, 8], [256], [65536])]
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_tune(sl, profile)
    assert e.value.code == lg.LAGOM_ECALLBACK
    calls.clear()
    r = lg.lagom_tune(sl, profile, raise_on_callback_error=False)
    assert r.code == lg.LAGOM_ECALLBACK and r.cfgs == [(2, 256, 65536)] and r.calls == 2
    with pytest.raises(lg.LagomError):
        lg.lagom_tune([lg.Space([2, 1], [256], [65536])], profile)
    with pytest.raises(lg.LagomError):
        lg.lagom_tune([lg.Space([1], [256], [65536])], lambda c: ([float("nan")], 1.0))


def test_comm_optimal_mode_equals_oracle_coordinate_descent():
    rng = np.random.default_rng(21)
    for _ in range(200):
        N = int(rng.integers(1, 6))
        so, sl, profile = _random_chain(rng, N)
        ro = osr.coordinate_descent(so, profile)
        rl = lg.lagom_tune(sl, profile, lg.LAGOM_COMM_OPTIMAL)
        assert rl.cfgs == ro.cfgs and rl.calls == ro.calls and (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)


def test_dependent_cost_model_equals_oracle_bit_for_bit(golden_dir):
    rng = np.random.default_rng(31)
    for _ in range(300):
        N, M = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        mo, ml, cfgs = _random_model(rng, N, M)
        cac = [int(rng.integers(-1, min(i + 1, N))) for i in range(M)]
        cap = [int(rng.integers(-1, min(j, M))) if j > 0 else -1 for j in range(N)]
        ml.comp_after_comm, ml.comm_after_comp = cac, cap
        po, pl = ocm.predict(mo, cfgs, cac, cap), lg.lagom_cost_model(ml, cfgs)
        assert pl.y_us == po.y and pl.g == po.g and (pl.X_us, pl.Y_us, pl.Z_us) == (po.X, po.Y, po.Z)
    fx = json.load(open(os.path.join(golden_dir, "cost_model_worked.json")))
    for case in fx["dependent_cases"]:
        tables = [{(c["nc"], 256, 65536): (c["x"], c["v"])} for c in case["comms"]]
        model = lg.Model(fx["lambda"], fx["bw_peak"], [lg.CompModel(c["mu"], c["tb"], c["d_bytes"], c["theta"]) for c in case["comps"]],
                         tables, case["comp_after_comm"], case["comm_after_comp"])
        p = lg.lagom_cost_model(model, [(c["nc"], 256, 65536) for c in case["comms"]])
        assert p.y_us == case["y"] and p.g == case["g"] and (p.X_us, p.Y_us, p.Z_us) == (case["X"], case["Y"], case["Z"])
    cyc = lg.Model(8, 100.0, [lg.CompModel(10, 1, 1.0, 0.5)], [{(2, 64, 64): (5.0, 1.0)}], [0], [0])
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_cost_model(cyc, [(2, 64, 64)])
    assert e.value.code == lg.LAGOM_EINVAL


# ------------------------------------------------- computation-bound objective, ladder helper
def test_hide_modes_equal_oracle_result_and_trace(golden_dir):
    rng = np.random.default_rng(41)
    hidden = 0
    for _ in range(300):
        N = int(rng.integers(1, 9))
        so, sl, profile = _random_chain(rng, N)
        ro = osr.hide_search(so, profile)
        rl = lg.lagom_tune(sl, profile, lg.LAGOM_HIDE_COMM)
        assert rl.cfgs == ro.cfgs and rl.levels == ro.levels and rl.calls == ro.calls
        assert (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)
        _same_trace(rl.trace, ro.trace)
        hidden += ro.X <= ro.Y
    assert 30 < hidden < 300
    for _ in range(60):
        N = int(rng.integers(1, 4))
        so, sl, profile = _random_chain(rng, N)
        ro = osr.brute_force_hide(so, profile)
        rl = lg.lagom_tune(sl, profile, lg.LAGOM_EXHAUSTIVE_HIDE)
        assert rl.cfgs == ro.cfgs and rl.levels == ro.levels and rl.calls == ro.calls and (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)
    fx = json.load(open(os.path.join(golden_dir, "hide_worked.json")))
    for case in fx["cases"]:
        so = [osr.Space(**sp) for sp in case["spaces"]]
        sl = [lg.Space(**sp) for sp in case["spaces"]]
        xs, coef = case["x_by_level"], case["Y_coef"]

        def profile(cfgs):
            lv = [[so[j].cfg(l) for l in range(so[j].K)].index(tuple(c)) for j, c in enumerate(cfgs)]
            return [xs[j][l] for j, l in enumerate(lv)], coef[0] + sum(coef[1 + j] * l for j, l in enumerate(lv))
        r = lg.lagom_tune(sl, profile, lg.LAGOM_HIDE_COMM)
        assert r.levels == case["final_levels"] and r.Y == case["final_Y"] and r.calls == case["calls"]
        for got, want in zip(r.trace, case["trace"]):
            assert (got.comm, got.level_from, got.level_to, got.accepted, got.done) == \
                (want["comm"], want["from"], want["to"], want["accepted"], want["done"])
        b = lg.lagom_tune(sl, profile, lg.LAGOM_EXHAUSTIVE_HIDE)
        assert b.levels == case["brute_levels"] and b.Y == case["brute_Y"]
    with pytest.raises(lg.LagomError):
        lg.lagom_tune([lg.Space([1], [64], [16])], lambda c: ([1.0], 1.0), 6)


def test_free_steps_mode_equals_oracle_result_and_trace(golden_dir):
    rng = np.random.default_rng(59)
    differs = 0
    for _ in range(300):
        N = int(rng.integers(1, 9))
        so, sl, profile = _random_chain(rng, N)
        falling = rng.uniform(0.0, 2.0, size=N)

        def prof(cfgs):                                   # a computation that gets faster as channels are added
            x, Y = profile(cfgs)
            return x, Y - sum(float(falling[j]) * c[0] for j, c in enumerate(cfgs)) + 200.0
        ro = osr.priority_search(so, prof, free_steps=True)
        rl = lg.lagom_tune(sl, prof, lg.LAGOM_PRIORITY_FREE)
        assert rl.cfgs == ro.cfgs and rl.levels == ro.levels and rl.calls == ro.calls and (rl.X, rl.Y, rl.Z) == (ro.X, ro.Y, ro.Z)
        _same_trace(rl.trace, ro.trace)
        differs += ro.levels != osr.priority_search(so, prof).levels
    assert differs > 20                                   # the variant was exercised where it departs from the printed algorithm
    case = json.load(open(os.path.join(golden_dir, "search_worked.json")))["free_steps_cases"][0]
    xs, Ys = case["x_by_level"], case["Y_by_level"]
    prof = lambda cfgs: ([xs[0][int(math.log2(cfgs[0][0]))]], Ys[int(math.log2(cfgs[0][0]))])
    sl = [lg.Space(**sp) for sp in case["spaces"]]
    r = lg.lagom_tune(sl, prof, lg.LAGOM_PRIORITY_FREE)
    assert r.levels == case["final_levels"] and r.Z == case["final_Z"] and r.calls == case["calls"]
    lit = lg.lagom_tune(sl, prof, lg.LAGOM_PRIORITY)
    assert lit.levels == case["literal"]["final_levels"] and lit.calls == case["literal"]["calls"]


def _sweep_points(rng, cfgs):
    return [lg.SweepPoint(c, float(rng.uniform(5, 500)), float(rng.uniform(5, 500)), float(rng.uniform(100, 900)),
                          float(rng.uniform(100, 1200)), float(rng.uniform(100, 1500)), float(rng.uniform(1e4, 9e6)),
                          float(rng.uniform(1e4, 9e6))) for c in cfgs]


def test_ladder_chunks_equals_oracle():
    rng = np.random.default_rng(43)
    for _ in range(200):
        grid = sorted(set(int(16 * v) for v in rng.integers(1, 300000, size=rng.integers(1, 9))))
        nc_max, nt_ref = int(rng.choice([1, 4, 32, 256])), int(rng.choice([128, 256]))
        per_src = int(rng.integers(0, 1 << 25))
        cfgs = [(nc, nt, c) for nc in (nc_max, 2 * nc_max) for nt in (128, 256) for c in grid]
        pts = _sweep_points(rng, cfgs)
        alone = {p.cfg: p.comm_alone_us for p in pts}
        for kind in (lg.LAGOM_LADDER_FULL, lg.LAGOM_LADDER_CUT, lg.LAGOM_LADDER_FIXED_CHUNK):
            assert lg.lagom_ladder_chunks(grid, nc_max, nt_ref, per_src, kind, pts) == osr.ladder_chunks(grid, nc_max, nt_ref, per_src, kind, alone)
    with pytest.raises(lg.LagomError):
        lg.lagom_ladder_chunks([32, 16], 4, 256, 100, lg.LAGOM_LADDER_CUT)
    with pytest.raises(lg.LagomError):
        lg.lagom_ladder_chunks([16, 32], 4, 256, 100, lg.LAGOM_LADDER_FIXED_CHUNK, None)
    with pytest.raises(lg.LagomError):
        lg.lagom_ladder_chunks([16, 32], 4, 256, 100, 9)


# ------------------------------------------------------------ model fill and calibration
def _fill_case(rng):
    lam = int(rng.choice([8, 64, 256]))
    bw = float(rng.uniform(1e5, 8e6))
    geo = omf.Geometry(int(rng.integers(1, 3000)), int(rng.integers(1, 3)), float(rng.uniform(1e3, 5e6)))
    ncomp, ncomm = int(rng.integers(1, 5)), int(rng.integers(1, 4))
    nbytes = [float(rng.integers(1, 1 << 28)) for _ in range(ncomm)]
    cfgs = [(nc, nt, c) for nc in (1, 4, 7) if nc < lam for nt in (128, 256) for c in (4096, 65536)]
    pts = _sweep_points(rng, cfgs)
    opts = [omf.SweepPoint(p.cfg, p.comm_corun_us, p.comp_alone_us, p.comp_corun_us, p.v_corun) for p in pts]
    return lam, bw, geo, ncomp, nbytes, pts, opts


def test_model_fill_equals_oracle_bit_for_bit():
    rng = np.random.default_rng(47)
    for _ in range(200):
        lam, bw, geo, ncomp, nbytes, pts, opts = _fill_case(rng)
        held = [bool(rng.integers(0, 2)) for _ in pts]
        held[int(rng.integers(0, len(pts)))] = False
        ml, t_alone = lg.lagom_model_fill(pts, lam, bw, geo.mu, geo.tb, geo.d_bytes, ncomp, nbytes, held)
        fit = [p for p, h in zip(opts, held) if not h]
        mo = omf.fill(opts, geo, ncomp, nbytes, lam, bw, theta_points=fit)
        assert t_alone == omf.t_alone(fit, ncomp)
        assert [c.theta_us for c in ml.comps] == [c.theta for c in mo.comps]
        assert [(c.mu, c.tb, c.d_bytes) for c in ml.comps] == [(c.mu, c.tb, c.d_bytes) for c in mo.comps]
        assert ml.tables == mo.tables
    # the pencil-worked numbers of tests/test_oracle_model_fill.py through the library
    pts = [lg.SweepPoint((2, 64, 16), 0.0, 40.0, a, 350.0, 0.0, 0.0, v) for a, v in ((330.0, 10.0), (300.0, 10.0), (360.0, 10.0))]
    pts[1].cfg, pts[2].cfg, pts[2].v_corun, pts[2].comm_corun_us = (4, 64, 32), (8, 64, 32), 120.0, 20.0
    m, t_alone = lg.lagom_model_fill(pts, 4, 100.0, 20, 2, 1000.0, 1, [300.0, 100.0])
    assert t_alone == 330.0 and m.comps[0].theta_us == 30.0
    assert m.tables[0][(2, 64, 16)] == (30.0, 10.0) and m.tables[1][(2, 64, 16)] == (10.0, 10.0)
    assert m.tables[0][(8, 64, 32)] == (15.0, 99.0)
    for bad in [dict(mu=0), dict(tb=0), dict(ncomp=0), dict(comm_bytes=[0.0, 0.0]), dict(lam=0), dict(v_cap_frac=1.0)]:
        kw = dict(lam=4, bw_peak=100.0, mu=20, tb=2, d_bytes=1000.0, ncomp=1, comm_bytes=[300.0, 100.0])
        kw.update(bad)
        with pytest.raises(lg.LagomError) as e:
            lg.lagom_model_fill(pts, **kw)
        assert e.value.code == lg.LAGOM_EINVAL
    with pytest.raises(lg.LagomError):
        lg.lagom_model_fill(pts, 4, 100.0, 20, 2, 1000.0, 1, [1.0], held_out=[True, True, True])


def test_model_calibrate_equals_oracle_bit_for_bit():
    rng = np.random.default_rng(53)
    sigmas = [i / 8 for i in range(9)]
    for trial in range(120):
        lam, bw, geo, ncomp, nbytes, pts, opts = _fill_case(rng)
        held = [i % 2 == 1 for i in range(len(pts))] if trial % 3 else None
        cac = cap = None
        if trial % 4 == 0:                                   # with cross-stream dependencies
            cac = [int(rng.integers(-1, min(i + 1, len(nbytes)))) for i in range(ncomp)]
            cap = [int(rng.integers(-1, min(j, ncomp))) if j > 0 else -1 for j in range(len(nbytes))]
        co = omf.calibrate(opts, held, geo, ncomp, nbytes, lam, bw, sigmas, cac, cap)
        cl = lg.lagom_model_calibrate(pts, lam, bw, geo.mu, geo.tb, geo.d_bytes, ncomp, nbytes, sigmas, held,
                                      comp_after_comm=cac, comm_after_comp=cap)
        assert (cl.sigma, cl.fit_mean, cl.fit_max, cl.held_mean, cl.held_max, cl.n_fit, cl.n_held) == \
            (co.sigma, co.fit_mean, co.fit_max, co.held_mean, co.held_max, co.n_fit, co.n_held)
    # with the resident penalty calibrated after sigma
    rhos = [0.0, 0.02, 0.05, 0.1, 0.2, 0.4]
    for trial in range(80):
        lam, bw, geo, ncomp, nbytes, pts, opts = _fill_case(rng)
        held = [i % 3 == 1 for i in range(len(pts))] if trial % 2 else None
        cac = cap = None
        if trial % 4 == 0:
            cac = [int(rng.integers(-1, min(i + 1, len(nbytes)))) for i in range(ncomp)]
            cap = [int(rng.integers(-1, min(j, ncomp))) if j > 0 else -1 for j in range(len(nbytes))]
        co = omf.calibrate(opts, held, geo, ncomp, nbytes, lam, bw, sigmas, cac, cap, rhos=rhos)
        cl = lg.lagom_model_calibrate(pts, lam, bw, geo.mu, geo.tb, geo.d_bytes, ncomp, nbytes, sigmas, held,
                                      comp_after_comm=cac, comm_after_comp=cap, rhos=rhos)
        assert (cl.sigma, cl.fit_mean, cl.fit_max, cl.held_mean, cl.held_max, cl.n_fit, cl.n_held) == \
            (co.sigma, co.fit_mean, co.fit_max, co.held_mean, co.held_max, co.n_fit, co.n_held)
        assert cl.penalty == co.penalty and list(cl.penalty) == sorted(cl.penalty)
    # the pencil-worked case
    fit = lg.SweepPoint((2, 64, 16), 0.0, 1000.0, 330.0, 400.0, 0.0, 0.0, 10.0)
    held = lg.SweepPoint((1, 64, 16), 0.0, 1000.0, 500.0, 350.0, 0.0, 0.0, 20.0)
    c = lg.lagom_model_calibrate([fit, held], 4, 100.0, 20, 2, 1000.0, 1, [4000.0], [0.0, 0.5, 1.0], [False, True])
    assert c.sigma == 0.5 and c.theta_us == 30.0 and c.fit_mean == pytest.approx(1 / 30, rel=1e-12)
    assert c.held_mean == pytest.approx(2.5 / 350, rel=1e-12)
    c = lg.lagom_model_calibrate([fit, held], 4, 100.0, 20, 2, 1000.0, 1, [4000.0], [0.0, 0.5, 1.0], [False, True], rhos=[0.0, 0.05, 0.1])
    assert c.sigma == 0.5 and c.penalty == {64: 0.05}
    assert c.fit_mean == pytest.approx(6 / 400, rel=1e-12) and c.held_mean == pytest.approx(20.125 / 350, rel=1e-12)
    with pytest.raises(lg.LagomError):
        lg.lagom_model_calibrate([fit], 4, 100.0, 20, 2, 1000.0, 1, [4000.0], [1.5])
    with pytest.raises(lg.LagomError):
        lg.lagom_model_calibrate([fit], 4, 100.0, 20, 2, 1000.0, 1, [4000.0], [0.5], rhos=[-0.5])
