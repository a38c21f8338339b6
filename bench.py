#!/usr/bin/env python3
"""Benchmark of the Lagom hot path on one MI355X.

One "step" is one pass of the whole overlapped group of a workload (every communication launch on one
stream, every GEMM on the other) with the parameters the priority search picked.  With no flags all five
workloads of the benchmark spec run -- tiny, dp_bucket, tp_layer, fsdp_chain, compute_bound -- and the
headline is the largest, fsdp_chain (eight all-gather / GEMM pairs).  Per workload: the contention
profiler sweeps the (NC, C[, NT]) grid, the cost model is filled and calibrated from the sweep (half of
the points held out), lagom_tune runs with measured profiles (Alg. 1/2, the communication-only descent,
the computation-bound objective) and with the model, and every chosen configuration is timed against the
default, interleaved round by round.

Prints ONE JSON line: value = makespan(default NC=8, C=2 MiB, NT=256) / makespan(tuned) of the headline
workload (median over the interleaved rounds); "configs" holds the same figures for every workload.
All method arithmetic (model fill, calibration, ladders, searches) runs inside liblagom.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0       # MI355X dense bf16 MFMA, published
LAMBDA = 256                    # compute units
DEFAULT_CFG = (8, 256, 2 << 20)  # the collective library default the paper quotes (Sec. 4.3), NT from the tiny config
EXTENDED_NC = (64, 128, 256)     # beyond the workloads' own grids: where the X = Y crossover lies on this part
EXTENDED_NT = (128,)             # channels of two wavefronts: the lightest the NT grids of the benchmark spec hold
FIVE = ["tiny", "dp_bucket", "tp_layer", "fsdp_chain", "compute_bound"]
HEADLINE = "fsdp_chain"
# Bytes past L2 per launch, from rocprofv3 FETCH_SIZE and WRITE_SIZE collected over `bench.py --standalone-only` and
# scaled by the same counters' reading of the 64 MiB calibration copy (x 1.9985 and x 0.9992); recorded figures per
# kernel and shape (commands and raw readings: profiles/hbm_traffic_by_kernel.md), not measured by this run.
MiB = 1 << 20
TRAFFIC_FROM_PROFILE = {
    "gemm 512x512x512": int(3.66 * MiB),              # algorithmic 1.5 MiB
    "gemm 4096x4096x4096": int(224.3 * MiB),          # algorithmic 96 MiB
    "gemm 4096x3584x8192": int(412.1 * MiB),          # algorithmic 148 MiB
    "gemm 8192x4096x4096": int(448.1 * MiB),          # algorithmic 160 MiB
    "gemm 8192x8192x8192": int(1689.7 * MiB),         # algorithmic 384 MiB
    "reduce_copy bf16 S=8 D=1 count=4194304": int(72.0 * MiB),
    "gather_copy bf16 S=8 D=1 count=2097152": int(64.0 * MiB),
}


def _up(x):
    import torch
    return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()


def build_workload(name: str, dependent: bool = False, fused: bool = True):
    """Device buffers + launch descriptors of one synthetic overlap group.  fused: the fourteen ring steps of the DP
    bucket's all-reduce share are issued as one kernel launch (lagom_comm_steps), the way a collective library runs a
    ring.  The back-to-back reduce-copies of the compute-bound workload are separate operators and stay separate
    launches (measured: persistent channels there cost the GEMM more than the launch boundaries cost the communication)."""
    import torch
    from paper_2602_20656_amd import binding as lg, inputs
    w = inputs.WORKLOADS[name]
    M, N, K = w.gemm
    keep = []
    launches = []
    dt = lg.LAGOM_F32 if w.comm.dtype == "f32" else lg.LAGOM_BF16
    gen = (lambda seed, n: inputs.uniform_f32(seed, n)) if w.comm.dtype == "f32" else \
          (lambda seed, n: inputs.normal_bf16(seed, n, w.scale))
    np_dt = np.float32 if w.comm.dtype == "f32" else np.uint16

    if name == "dp_bucket":
        P, m = 8, w.comm.count
        local = _up(gen(w.seeds[0], P * m))
        wire_in = [_up(gen(w.seeds[1 + i], m)) for i in range(2)]
        wire_out = [_up(np.zeros(m, np_dt)) for _ in range(2)]
        keep += [local, wire_in, wire_out]
        esz = 2
        chunk = lambda c: local.data_ptr() + c * m * esz
        r = 0
        for s in range(P - 1):                       # reduce-scatter phase: out = incoming + local
            c = (r - s - 1) % P
            dsts = [wire_out[s % 2]] + ([chunk(c)] if s == P - 2 else [])
            launches.append(lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, [wire_in[s % 2], chunk(c)], dsts, m, 0))
        for s in range(P - 1):                       # all-gather phase: store and forward
            c = (r - s) % P
            dsts = [chunk(c)] + ([wire_out[s % 2]] if s < P - 2 else [])
            launches.append(lg.CommLaunch(lg.LAGOM_GATHER_COPY, dt, [wire_in[s % 2]], dsts, m, 0))
        ncomm = 1
    elif name == "fsdp_chain":
        ncomm = w.ncomm
        weights = []
        for j in range(ncomm):
            shards = [_up(gen(w.seeds[j] * 100 + p, w.comm.count)) for p in range(w.comm.nsrc)]
            full = _up(np.zeros(w.comm.nsrc * w.comm.count, np_dt))
            keep += [shards, full]
            weights.append(full)
            launches.append(lg.CommLaunch(lg.LAGOM_GATHER_COPY, dt, shards, [full], w.comm.count, j))
    elif name == "ep_alltoall":
        ncomm, P, m, rank = 1, w.comm.nsrc, w.comm.count, 3
        send = [_up(gen(w.seeds[p], P * m)) for p in range(P)]          # every peer's send buffer: P blocks of m
        recv = _up(np.zeros(P * m, np_dt))
        keep += [send, recv]
        launches.append(lg.CommLaunch(lg.LAGOM_GATHER_COPY, dt, [b.data_ptr() + rank * m * 2 for b in send], [recv], m, 0))
    elif name == "tp_pipeline":
        ncomm = w.ncomm
        peers = [_up(gen(w.seeds[p], w.comm.count)) for p in range(1, 8)]     # the other ranks' partial outputs of this shard
        shard_out = [_up(np.zeros(w.comm.count, np_dt)) for _ in range(ncomm)]
        keep += [peers, shard_out]
    elif name == "rs_ag_pair":
        ncomm = 2
        grads = [_up(gen(w.seeds[p], w.comm.count)) for p in range(8)]
        shard = _up(np.zeros(w.comm.count, np_dt))
        shards = [_up(gen(w.seeds[8 + p], 2097152)) for p in range(8)]
        full = _up(np.zeros(8 * 2097152, np_dt))
        keep += [grads, shard, shards, full]
        launches.append(lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, grads, [shard], w.comm.count, 0))
        launches.append(lg.CommLaunch(lg.LAGOM_GATHER_COPY, dt, shards, [full], 2097152, 1))
    else:
        ncomm = 1
        reps = 1
        if name == "compute_bound":
            reps = 3      # back-to-back launches of the one operator: X at the default parameters is about Y/2
        for rep in range(reps):
            srcs = [_up(gen(w.seeds[s % len(w.seeds)] + 1000 * rep, w.comm.count)) for s in range(w.comm.nsrc)]
            dst = _up(np.zeros(w.comm.count, np_dt))
            keep += [srcs, dst]
            launches.append(lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, srcs, [dst], w.comm.count, 0))

    comps = []
    A = _up(inputs.normal_bf16(2, (M, K)))
    keep.append(A)
    for i in range(w.ncomp):
        if name == "fsdp_chain" and dependent and i > 0:
            B = weights[i - 1]          # prefetch: all-gather i-1 assembles the weight of GEMM i while GEMM i-1 runs
        elif name == "fsdp_chain":
            B = _up(inputs.normal_bf16(3 + i, (N, K), 0.02))   # literal Eq. 1: no cross-stream dependency
        else:
            B = _up(inputs.normal_bf16(3, (N, K), 0.02 if name != "tiny" else 1.0))
        Cm = torch.zeros((M, N), dtype=torch.int16, device="cuda")
        keep += [B, Cm]
        comps.append(lg.GemmDesc(A, B, Cm, M, N, K, True, lg.LAGOM_BF16,
                                 after_comm_id=i - 1 if (name == "fsdp_chain" and dependent and i > 0) else -1))
        if name == "tp_pipeline":      # communication i reduces this rank's first eighth of C_i with the peers' partials
            launches.append(lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, [Cm] + peers, [shard_out[i]], w.comm.count, i, after_comp=i))
    comp_after_comm = [c.after_comm_id for c in comps] if any(c.after_comm_id >= 0 for c in comps) else None
    comm_after_comp = None
    if any(l.after_comp >= 0 for l in launches):
        comm_after_comp = [-1] * ncomm
        for l in launches:
            comm_after_comp[l.comm_id] = max(comm_after_comp[l.comm_id], l.after_comp)
    if fused and name == "dp_bucket":
        for i in range(1, len(launches)):
            launches[i].fuse = True
    torch.cuda.synchronize()           # uploads ran on torch's stream; the library launches on its own streams
    return w, launches, comps, ncomm, keep, (comp_after_comm, comm_after_comp)


def comm_bytes(launches):
    from paper_2602_20656_amd import binding as lg
    return [lg.lagom_comm_bytes(l.op, l.dtype, len(l.srcs), len(l.dsts), l.count) for l in launches]


def gemm_kernel_name(geo, out_bf16=True):
    """The kernel lagom_gemm dispatches for a geometry (names as they appear in a kernel trace)."""
    if (geo.tile_m, geo.tile_n) == (128, 128):
        return "gemm_bf16_nk128_kernel"
    if (geo.tile_m, geo.tile_n) == (256, 128):
        return "gemm_bf16_nk256x128_kernel"
    return "gemm_bf16_nk_kernel"


def rotating_comm_roofline(st1, st2, op, dt_name, nsrc, count, cfgs, iters, final_iters=20):
    """Standalone bandwidth of one launch shape on buffer sets rotated through more than the 256 MB last-level cache,
    so that HBM has to serve every launch; the best of `cfgs` is measured once more, last, and reported."""
    import torch
    from paper_2602_20656_amd import binding as lg
    dt, tdt = (lg.LAGOM_F32, torch.float32) if dt_name == "f32" else (lg.LAGOM_BF16, torch.bfloat16)
    esz = 4 if dt_name == "f32" else 2
    per_launch = lg.lagom_comm_bytes(op, dt, nsrc, 1, count)
    nrot = max(2, -(-(576 << 20) // per_launch))
    out_count = count if op == lg.LAGOM_REDUCE_COPY else nsrc * count
    bufs = [([torch.empty(count, dtype=torch.float32, device="cuda").uniform_(-1, 1).to(tdt) for _ in range(nsrc)],
             torch.empty(out_count, dtype=tdt, device="cuda")) for _ in range(nrot)]
    torch.cuda.synchronize()
    launches = [lg.CommLaunch(op, dt, srcs, [dst], count, 0) for srcs, dst in bufs]
    best = None
    for cfg in cfgs:
        us = lg.lagom_overlap_run(launches, [cfg], [], st1, st2, 1, iters, lg.LAGOM_ALONE_COMM).X_us / nrot
        if best is None or us < best[0]:
            best = (us, cfg)
    t = lg.lagom_overlap_run(launches, [best[1]], [], st1, st2, 2, final_iters, lg.LAGOM_ALONE_COMM)
    us = t.X_us / nrot
    # the floor of a launch on this grid: the same kernel moving one 16-byte vector per source
    tiny = [lg.CommLaunch(op, dt, srcs, [dst], 16 // esz, 0) for srcs, dst in bufs]
    floor_us = lg.lagom_overlap_run(tiny, [best[1]], [], st1, st2, 2, final_iters, lg.LAGOM_ALONE_COMM).X_us / nrot
    # the same launches staged through LDS (lagom_comm_kernel_lds), best of the same configurations
    staged = [lg.CommLaunch(op, dt, srcs, [dst], count, 0, lds_staged=True) for srcs, dst in bufs]
    lds_best = min((lg.lagom_overlap_run(staged, [cfg], [], st1, st2, 1, iters, lg.LAGOM_ALONE_COMM).X_us / nrot, cfg) for cfg in cfgs)
    lds_us = lg.lagom_overlap_run(staged, [lds_best[1]], [], st1, st2, 2, final_iters, lg.LAGOM_ALONE_COMM).X_us / nrot
    name = f"{'reduce_copy' if op == lg.LAGOM_REDUCE_COPY else 'gather_copy'} {dt_name} S={nsrc} D=1 count={count}"
    gbps = per_launch / us / 1e3
    res = {"bound": "hbm", "kernel": "reduce_copy_kernel" if op == lg.LAGOM_REDUCE_COPY else "gather_copy_kernel",
           "workload": name, "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
           "traffic": None, "traffic_from_profile": TRAFFIC_FROM_PROFILE.get(name),
           "us_per_launch": us, "bytes_per_launch": per_launch, "cfg": list(best[1]), "rotation_mib": nrot * per_launch >> 20,
           "launches_timed": nrot * final_iters, "launch_floor_us": floor_us,
           "frac_outside_launch_floor": per_launch / max(us - floor_us, 1e-9) / 1e3 / HBM_PEAK_GBPS,
           "staged_through_lds": {"us_per_launch": lds_us, "achieved": per_launch / lds_us / 1e3,
                                  "frac": per_launch / lds_us / 1e3 / HBM_PEAK_GBPS, "cfg": list(lds_best[1])}}
    del bufs, launches, tiny, staged
    return res


def standalone_comm_rooflines(st1, st2, iters):
    """The two launch shapes of the workloads that move the most bytes: the eight-source bf16 reduce of the TP layer
    (72 MiB per launch) and the FSDP all-gather copy (64 MiB per launch)."""
    from paper_2602_20656_amd import binding as lg
    cands = [(nc, nt, c) for nc in (256, 512, 1024) for nt in (512, 1024) for c in (16 << 10, 32 << 10, 64 << 10)]
    red = rotating_comm_roofline(st1, st2, lg.LAGOM_REDUCE_COPY, "bf16", 8, 4194304, cands, iters)
    gat = rotating_comm_roofline(st1, st2, lg.LAGOM_GATHER_COPY, "bf16", 8, 2097152, cands, iters)
    red["gather_copy_64MiB"] = gat
    return red


def cpu_baseline(name, seconds_target=12.0):
    """The oracle's plain C loops, timed on the host cores on a bounded sample of the same workload."""
    from oracle import cloops
    from paper_2602_20656_amd import inputs
    w = inputs.WORKLOADS[name]
    threads = cloops.max_threads()
    # communication: the operator's launches, full size
    if w.comm.dtype == "f32":
        srcs = [inputs.uniform_f32(s, w.comm.count) for s in range(w.comm.nsrc)]
    else:
        srcs = [inputs.normal_bf16(s, w.comm.count, w.scale) for s in range(w.comm.nsrc)]
    t0 = time.perf_counter()
    if w.comm.op == "reduce_copy":
        cloops.reduce_copy(srcs, w.comm.dtype, w.comm.ndst, threads)
    else:
        cloops.gather_copy(srcs, w.comm.ndst, threads)
    comm_us = (time.perf_counter() - t0) * 1e6 * w.comm.launches * w.ncomm
    # GEMM: a slice of rows, all columns, all of K, scaled linearly to M rows
    M, N, K = w.gemm
    a = inputs.normal_bf16(2, (M, K)); b = inputs.normal_bf16(3, (N, K), 0.02)
    rows = min(M, 2 * threads)
    t0 = time.perf_counter(); cloops.gemm(a, b, True, 0, rows, threads); dt = time.perf_counter() - t0
    rows2 = int(min(M, max(rows, rows * seconds_target / max(dt, 1e-3)) // threads * threads))
    if rows2 > rows:
        t0 = time.perf_counter(); cloops.gemm(a, b, True, 0, rows2, threads); dt = time.perf_counter() - t0
        rows = rows2
    gemm_us = dt * 1e6 * (M / rows) * w.ncomp
    return {"value": comm_us + gemm_us, "unit": "us/step", "cores": threads, "kind": "oracle", "workload": name,
            "sample": f"communication launches at full size ({comm_us:.0f} us); GEMM rows 0..{rows} of {M}, all columns and K, "
                      f"scaled by {M / rows:.1f} ({gemm_us:.0f} us); no overlap on the CPU",
            "comm_us": comm_us, "gemm_us": gemm_us}


def ladder_cfgs(space):
    K = max(len(space.nc), len(space.nt), len(space.chunk))
    return [(space.nc[min(l, len(space.nc) - 1)], space.nt[min(l, len(space.nt) - 1)], space.chunk[min(l, len(space.chunk) - 1)])
            for l in range(K)]


def stop_test_audit(result, log):
    """How often Alg. 2's `x' - x > 0` stop fired on a difference smaller than the spread of the two measurements."""
    fired = within = 0
    for k, s in enumerate(result.trace):
        if s.comm < 0 or s.accepted or not s.done or k >= len(log):
            continue
        if s.xj_new - s.xj_prev > 0.0:
            fired += 1
            # spread of x' from this call; of x from the call that measured the configuration it is compared with
            prev = max((i for i in range(k) if i == 0 or result.trace[i].accepted), default=0)
            spread = log[k]["x_mad"][s.comm] + log[prev]["x_mad"][s.comm]
            within += (s.xj_new - s.xj_prev) < spread
    return {"stops_on_x_rise": fired, "of_which_within_spread": within}


def run_config(name, args, s_comm, s_comp, dependent=False):
    import torch
    from paper_2602_20656_amd import binding as lg
    t_start = time.perf_counter()
    w, launches, comps, ncomm, keep, (dep_arg, dep_comm) = build_workload(name, dependent)
    dependent = dep_arg is not None or dep_comm is not None
    nbytes = comm_bytes(launches)
    bytes_per_comm = [float(sum(b for b, l in zip(nbytes, launches) if l.comm_id == j)) for j in range(ncomm)]
    M, N, K = w.gemm
    flops = 2.0 * M * N * K
    geo = lg.lagom_gemm_describe(M, N, K)
    bw = HBM_PEAK_GBPS * 1e3                                     # bytes per microsecond
    nt_grid = list(w.nt_grid)
    nt_ref = 256 if 256 in nt_grid else nt_grid[0]
    esz = 4 if w.comm.dtype == "f32" else 2
    per_src = [min(l.count * esz * (len(l.srcs) if l.op == lg.LAGOM_GATHER_COPY else 1) for l in launches if l.comm_id == j)
               for j in range(ncomm)]

    # ---- contention profiler: the workload's own grid, then the extended channel counts
    points = [(nc, nt, c) for nt in nt_grid for nc in w.nc_grid for c in w.chunk_grid]
    nt_all = sorted(set(nt_grid) | set(EXTENDED_NT))
    ext_points = [(nc, nt, c) for nt in nt_all for nc in list(w.nc_grid) + list(EXTENDED_NC) for c in w.chunk_grid
                  if nc in EXTENDED_NC or nt not in nt_grid]
    t0 = time.perf_counter()
    sweep = lg.lagom_contention_sweep(launches, ncomm, comps, points, s_comm, s_comp, 1, args.sweep_iters)
    sweep_ext = lg.lagom_contention_sweep(launches, ncomm, comps, ext_points, s_comm, s_comp, 1, args.sweep_iters)
    sweep_s = time.perf_counter() - t0
    all_sweep = sweep + sweep_ext

    # ---- cost model: filled and calibrated by the library; every second point is held out of the fit
    usable = [p for p in all_sweep if p.cfg[0] < LAMBDA]          # Eq. 5 needs NC < lambda
    held = [i % 2 == 1 for i in range(len(usable))]
    sigmas = [i / 8 for i in range(9)]
    fill_args = dict(lam=LAMBDA, bw_peak=bw, mu=geo.mu, tb=geo.tb, ncomp=len(comps), comm_bytes=bytes_per_comm)
    cal = lg.lagom_model_calibrate(usable, d_bytes=geo.d_bytes_past_l2, sigmas=sigmas, held_out=held,
                                   comp_after_comm=dep_arg, comm_after_comp=dep_comm, **fill_args)
    cal_all = lg.lagom_model_calibrate(usable, d_bytes=geo.d_bytes_past_l2, sigmas=sigmas, comp_after_comm=dep_arg,
                                       comm_after_comp=dep_comm, **fill_args)
    cal_printed = lg.lagom_model_calibrate(usable, d_bytes=geo.d_bytes, sigmas=[0.0], held_out=held,
                                           comp_after_comm=dep_arg, comm_after_comp=dep_comm, **fill_args)
    # the resident penalty rho(NT), calibrated after sigma on the same halves
    rhos = [0.0, 0.01, 0.02, 0.03, 0.04, 0.05, 0.06, 0.08, 0.1, 0.125, 0.15, 0.2, 0.25, 0.3, 0.4, 0.5]
    cal_pen = lg.lagom_model_calibrate(usable, d_bytes=geo.d_bytes_past_l2, sigmas=sigmas, held_out=held, rhos=rhos,
                                       comp_after_comm=dep_arg, comm_after_comp=dep_comm, **fill_args)
    cal_pen_all = lg.lagom_model_calibrate(usable, d_bytes=geo.d_bytes_past_l2, sigmas=sigmas, rhos=rhos,
                                           comp_after_comm=dep_arg, comm_after_comp=dep_comm, **fill_args)
    model, _ = lg.lagom_model_fill(usable, d_bytes=geo.d_bytes_past_l2, comp_after_comm=dep_arg, comm_after_comp=dep_comm,
                                   corun_share=cal_all.sigma, **fill_args)
    model_pen, _ = lg.lagom_model_fill(usable, d_bytes=geo.d_bytes_past_l2, comp_after_comm=dep_arg, comm_after_comp=dep_comm,
                                       corun_share=cal_pen_all.sigma, resident_penalty=cal_pen_all.penalty, **fill_args)
    model_printed, _ = lg.lagom_model_fill(usable, d_bytes=geo.d_bytes, comp_after_comm=dep_arg, comm_after_comp=dep_comm,
                                           corun_share=0.0, **fill_args)

    # which uniform configuration each model would pick among the swept ones, and what that pick measured
    def uniform_pick(mdl):
        z_of = {tuple(p.cfg): lg.lagom_cost_model(mdl, [tuple(p.cfg)] * ncomm).Z_us for p in usable}
        pick = min(usable, key=lambda p: z_of[tuple(p.cfg)])
        best = min(usable, key=lambda p: p.z_corun_us)
        order_m = sorted(usable, key=lambda p: z_of[tuple(p.cfg)])
        order_z = sorted(usable, key=lambda p: p.z_corun_us)
        rank = {tuple(p.cfg): i for i, p in enumerate(order_z)}
        return {"cfg": list(pick.cfg), "z_model_us": z_of[tuple(pick.cfg)], "z_measured_us": pick.z_corun_us,
                "best_measured_cfg": list(best.cfg), "z_best_measured_us": best.z_corun_us,
                "pick_over_best": pick.z_corun_us / best.z_corun_us, "rank_of_pick": rank[tuple(pick.cfg)], "of": len(usable),
                "z_err_mean": float(np.mean([abs(z_of[tuple(p.cfg)] - p.z_corun_us) / p.z_corun_us for p in usable])),
                "top5_overlap": len(set(tuple(p.cfg) for p in order_m[:5]) & set(tuple(p.cfg) for p in order_z[:5]))}
    uniform_picks = {"as_printed": uniform_pick(model_printed), "sigma": uniform_pick(model), "sigma_and_rho": uniform_pick(model_pen)}

    # ---- ladders (lagom_ladder_chunks): the cut ladder is the graded one; the uncut and the fixed-chunk ones beside it
    def spaces_for(nc_grid, kind, pts, nt=None):
        return [lg.Space(list(nc_grid), nt if nt is not None else (nt_grid if len(nt_grid) > 1 else [256]),
                         lg.lagom_ladder_chunks(list(w.chunk_grid), max(nc_grid), nt_ref, per_src[j], kind, pts))
                for j in range(ncomm)]
    spaces = spaces_for(w.nc_grid, lg.LAGOM_LADDER_CUT, sweep)
    spaces_full = spaces_for(w.nc_grid, lg.LAGOM_LADDER_FULL, sweep)
    spaces_fixed = spaces_for(w.nc_grid, lg.LAGOM_LADDER_FIXED_CHUNK, sweep)
    ext_nc = list(w.nc_grid) + [n for n in EXTENDED_NC if n > max(w.nc_grid)]
    spaces_ext = spaces_for(ext_nc, lg.LAGOM_LADDER_FIXED_CHUNK, all_sweep)
    # a ladder that raises the channel count only, every channel as light as the extended grids allow (two wavefronts):
    # on this part a channel of four or more wavefronts delays the GEMM workgroups of a multi-round GEMM on its
    # compute unit, one of two wavefronts does not
    spaces_ext_ntmin = spaces_for(ext_nc, lg.LAGOM_LADDER_FIXED_CHUNK, all_sweep, [min(nt_all)])

    def prof(cap):
        return lg.OverlapProfile(launches, comps, s_comm, s_comp, 1, args.sweep_iters, min_total_us=args.profile_min_us,
                                 max_iters=args.profile_max_iters, log_capacity=cap)

    def search(sp, mode, label):
        cap = 4 + sum(3 * (len(s.nc) + len(s.nt) + len(s.chunk) + 3) for s in sp)
        p = prof(cap)
        t0 = time.perf_counter()
        r = lg.lagom_tune(sp, p, mode)
        d = {"cfgs": [list(c) for c in r.cfgs], "calls": r.calls, "seconds": time.perf_counter() - t0,
             "z_search_us": r.Z, "x_search_us": r.X, "y_search_us": r.Y}
        if mode in (lg.LAGOM_PRIORITY, lg.LAGOM_HIDE_COMM, lg.LAGOM_PRIORITY_FREE):
            d.update(stop_test_audit(r, p.log))
            d["median_rel_spread_x"] = float(np.median([m / max(x, 1e-9) for e in p.log for m, x in zip(e["x_mad"], e["x"])]))
            d["median_rel_spread_Y"] = float(np.median([e["Y_mad"] / max(e["Y"], 1e-9) for e in p.log]))
            d["profile_iters"] = int(np.median([e["iters"] for e in p.log]))
        return r, d, p.log

    searches, logs = {}, {}
    tuned, searches["priority"], logs["priority"] = search(spaces, lg.LAGOM_PRIORITY, "priority")
    tuned_full, searches["priority_uncut_ladder"], _ = search(spaces_full, lg.LAGOM_PRIORITY, "uncut")
    tuned_fixed, searches["priority_fixed_chunk"], logs["priority_fixed_chunk"] = search(spaces_fixed, lg.LAGOM_PRIORITY, "fixed")
    comm_cd, searches["comm_descent"], _ = search(spaces, lg.LAGOM_COMM_OPTIMAL, "descent")
    hide, searches["hide_comm"], logs["hide_comm"] = search(spaces_fixed, lg.LAGOM_HIDE_COMM, "hide")
    tuned_free, searches["priority_free_steps"], logs["priority_free_steps"] = search(spaces_fixed, lg.LAGOM_PRIORITY_FREE, "free")
    tuned_ext, searches["priority_extended"], logs["priority_extended"] = search(spaces_ext, lg.LAGOM_PRIORITY, "ext")
    tuned_free_ext, searches["priority_free_steps_extended"], logs["priority_free_steps_extended"] = search(spaces_ext, lg.LAGOM_PRIORITY_FREE, "free-ext")
    hide_ext, searches["hide_comm_extended"], _ = search(spaces_ext, lg.LAGOM_HIDE_COMM, "hide-ext")
    if spaces_ext_ntmin is not None:
        tuned_ntmin, searches["priority_free_steps_extended_nt_min"], logs["priority_free_steps_extended_nt_min"] = \
            search(spaces_ext_ntmin, lg.LAGOM_PRIORITY_FREE, "free-ext-ntmin")
        hide_ntmin, searches["hide_comm_extended_nt_min"], _ = search(spaces_ext_ntmin, lg.LAGOM_HIDE_COMM, "hide-ext-ntmin")
    # brute force over the extended ladder: every level vector for one communication, the uniform vectors otherwise
    ext_ladder = ladder_cfgs(spaces_ext[0])
    if ncomm == 1:
        brute_ext, searches["exhaustive_extended"], _ = search(spaces_ext, lg.LAGOM_EXHAUSTIVE, "brute-ext")
        brute_hide_ext, searches["exhaustive_hide_extended"], _ = search(spaces_ext, lg.LAGOM_EXHAUSTIVE_HIDE, "brute-hide-ext")
    else:
        brute_ext = brute_hide_ext = None
    # the model as ProfileTime (host only)
    in_tables = lambda sp: all(tuple(c) in model.tables[j] for j, s in enumerate(sp) for c in ladder_cfgs(s))
    t0 = time.perf_counter()
    tuned_model = lg.lagom_tune(spaces, model, lg.LAGOM_PRIORITY) if in_tables(spaces) else None
    model_tune_us = (time.perf_counter() - t0) * 1e6
    tuned_printed = lg.lagom_tune(spaces, model_printed, lg.LAGOM_PRIORITY) if in_tables(spaces) else None
    # the model with the resident penalty as ProfileTime over the extended ladders
    # (Eq. 5 needs NC < lambda, so these ladders end below it)
    model_pen_searches = {}
    nc_model = [n for n in ext_nc if n < LAMBDA]
    sp_model = spaces_for(nc_model, lg.LAGOM_LADDER_FIXED_CHUNK, all_sweep)
    sp_model_ntmin = spaces_for(nc_model, lg.LAGOM_LADDER_FIXED_CHUNK, all_sweep, [min(nt_all)])
    for label, sp, mode in (("model_rho_priority_extended", sp_model, lg.LAGOM_PRIORITY),
                            ("model_rho_free_steps_extended", sp_model, lg.LAGOM_PRIORITY_FREE),
                            ("model_rho_free_steps_extended_nt_min", sp_model_ntmin, lg.LAGOM_PRIORITY_FREE)):
        if in_tables(sp):
            model_pen_searches[label] = lg.lagom_tune(sp, model_pen, mode)

    # ---- the first three pairs of the chain: priority search against exhaustive search over the same ladder
    first3 = None
    if name == "fsdp_chain" and ncomm >= 3:
        l3 = [l for l in launches if l.comm_id < 3]
        c3 = comps[:3]
        sp3 = [lg.Space(sp.nc[:6], sp.nt, sp.chunk[:6]) for sp in spaces[:3]]
        prof3 = lg.OverlapProfile(l3, c3, s_comm, s_comp, 1, args.sweep_iters, min_total_us=args.profile_min_us, max_iters=args.profile_max_iters)
        model3 = lg.Model(model.lam, model.bw_peak, model.comps[:3], model.tables[:3],
                          comp_after_comm=dep_arg[:3] if dep_arg else None, corun_share=model.corun_share)
        t0 = time.perf_counter()
        pr_meas, ex_meas = lg.lagom_tune(sp3, prof3, lg.LAGOM_PRIORITY), lg.lagom_tune(sp3, prof3, lg.LAGOM_EXHAUSTIVE)
        first3_s = time.perf_counter() - t0
        pr_mod, ex_mod = lg.lagom_tune(sp3, model3, lg.LAGOM_PRIORITY), lg.lagom_tune(sp3, model3, lg.LAGOM_EXHAUSTIVE)
        zs = {k: [] for k in ("pm", "em", "pd", "ed")}
        for _ in range(args.rounds):
            for k, r in (("pm", pr_meas), ("em", ex_meas), ("pd", pr_mod), ("ed", ex_mod)):
                zs[k].append(lg.lagom_overlap_run(l3, r.cfgs, c3, s_comm, s_comp, 2, args.steps, lg.LAGOM_CORUN).Z_us)
        med = lambda v: float(np.median(v))
        first3 = {"ladder_levels": [max(len(sp.nc), len(sp.nt), len(sp.chunk)) for sp in sp3],
                  "measured": {"priority_cfgs": [list(c) for c in pr_meas.cfgs], "priority_calls": pr_meas.calls,
                               "exhaustive_cfgs": [list(c) for c in ex_meas.cfgs], "exhaustive_calls": ex_meas.calls,
                               "same_cfgs": pr_meas.cfgs == ex_meas.cfgs,
                               "same_cfgs_up_to_order": sorted(pr_meas.cfgs) == sorted(ex_meas.cfgs),
                               "z_priority_us": med(zs["pm"]), "z_exhaustive_us": med(zs["em"]),
                               "z_priority_over_exhaustive": [float(np.min(np.array(zs["pm"]) / np.array(zs["em"]))), med(np.array(zs["pm"]) / np.array(zs["em"])),
                                                              float(np.max(np.array(zs["pm"]) / np.array(zs["em"])))],
                               "seconds": first3_s},
                  "model": {"priority_cfgs": [list(c) for c in pr_mod.cfgs], "priority_calls": pr_mod.calls,
                            "exhaustive_cfgs": [list(c) for c in ex_mod.cfgs], "exhaustive_calls": ex_mod.calls,
                            "same_cfgs": pr_mod.cfgs == ex_mod.cfgs,
                            "same_cfgs_up_to_order": sorted(pr_mod.cfgs) == sorted(ex_mod.cfgs),
                            "z_priority_model_us": pr_mod.Z, "z_exhaustive_model_us": ex_mod.Z,
                            "z_priority_us": med(zs["pd"]), "z_exhaustive_us": med(zs["ed"])}}

    # ---- every candidate against the default, interleaved: one measurement of each per round, the order rotating
    best_sweep = min(sweep, key=lambda p: p.z_corun_us)
    best_sweep_ext = min(all_sweep, key=lambda p: p.z_corun_us)
    comm_opt = min(sweep, key=lambda p: p.comm_alone_us)
    # a second default: the library default's chunk clamped so that its eight channels all have a chunk of every launch
    clamped = [(DEFAULT_CFG[0], DEFAULT_CFG[1], min(DEFAULT_CFG[2], lg.lagom_ladder_chunks(list(w.chunk_grid) + ([DEFAULT_CFG[2]] if DEFAULT_CFG[2] > max(w.chunk_grid) else []),
                                                                                               DEFAULT_CFG[0], DEFAULT_CFG[1], per_src[j], lg.LAGOM_LADDER_CUT)[-1]))
               for j in range(ncomm)]
    cands = {"default": [DEFAULT_CFG] * ncomm, "default_chunk_clamped": clamped, "tuned": tuned.cfgs, "tuned_uncut_ladder": tuned_full.cfgs,
             "tuned_fixed_chunk": tuned_fixed.cfgs, "comm_descent": comm_cd.cfgs, "hide_comm": hide.cfgs,
             "best_swept": [best_sweep.cfg] * ncomm, "comm_optimal": [comm_opt.cfg] * ncomm,
             "tuned_free_steps": tuned_free.cfgs,
             "tuned_extended": tuned_ext.cfgs, "tuned_free_steps_extended": tuned_free_ext.cfgs,
             "hide_comm_extended": hide_ext.cfgs, "best_swept_extended": [best_sweep_ext.cfg] * ncomm}
    if spaces_ext_ntmin is not None:
        cands["tuned_free_steps_extended_nt_min"] = tuned_ntmin.cfgs
        cands["hide_comm_extended_nt_min"] = hide_ntmin.cfgs
    if brute_ext is not None:
        cands["exhaustive_extended"] = brute_ext.cfgs
        cands["exhaustive_hide_extended"] = brute_hide_ext.cfgs
    if tuned_model is not None:
        cands["model_tuned"] = tuned_model.cfgs
        cands["printed_model_tuned"] = tuned_printed.cfgs
    cands["model_rho_uniform_pick"] = [tuple(uniform_picks["sigma_and_rho"]["cfg"])] * ncomm
    for label, r in model_pen_searches.items():
        cands[label] = r.cfgs
    # the same parameters with every launch of a communication issued on its own (no lagom_comm_steps)
    separate = None
    if any(l.fuse for l in launches):
        separate = [lg.CommLaunch(l.op, l.dtype, l.srcs, l.dsts, l.count, l.comm_id, l.after_comp, False) for l in launches]
        cands["default_separate_launches"] = cands["default"]
        cands["tuned_separate_launches"] = tuned.cfgs
        cands["tuned_extended_separate_launches"] = tuned_ext.cfgs
    # the tuned parameters with every launch staged through LDS (such a workgroup cannot share a compute unit with a GEMM's)
    staged = [lg.CommLaunch(l.op, l.dtype, l.srcs, l.dsts, l.count, l.comm_id, l.after_comp, False, True) for l in launches]
    cands["default_lds_staged"] = cands["default"]
    cands["tuned_lds_staged"] = tuned.cfgs
    which_launches = lambda k: separate if k.endswith("_separate_launches") else (staged if k.endswith("_lds_staged") else launches)
    meas = {k: [] for k in cands}
    order = list(cands)
    y_alone_rounds = []
    for r in range(args.rounds):
        y_alone_rounds.append(lg.lagom_overlap_run(launches, cands["default"], comps, s_comm, s_comp, 2, args.steps, lg.LAGOM_ALONE_COMP))
        for k in order[r % len(order):] + order[:r % len(order)]:
            meas[k].append(lg.lagom_overlap_run(which_launches(k), cands[k], comps, s_comm, s_comp, 2, args.steps, lg.LAGOM_CORUN))
    y_alone_sum = float(np.median([sum(t.y_us) for t in y_alone_rounds]))
    gemm_us = y_alone_sum / len(comps)

    def summary(k):
        z = np.array([t.Z_us for t in meas[k]])
        zd = np.array([t.Z_us for t in meas["default"]])
        ratio = zd / z
        d = {"cfgs": [list(c) for c in cands[k]], "z_us": float(np.median(z)), "z_rounds_us": [float(v) for v in z],
             "x_us": float(np.median([sum(t.x_us) for t in meas[k]])), "y_us": float(np.median([sum(t.y_us) for t in meas[k]])),
             "gemm_slowdown": float(np.median([sum(t.y_us) for t in meas[k]])) / y_alone_sum,
             "speedup_vs_default": [float(ratio.min()), float(np.median(ratio)), float(ratio.max())]}
        d["verdict"] = "no gain" if ratio.min() <= 1.0 <= ratio.max() else ("faster" if ratio.min() > 1.0 else "slower")
        return d
    results = {k: summary(k) for k in cands}

    # ---- K steps as a training loop would run them: enqueued back to back, streams joined by events only
    lg.lagom_overlap_steps(launches, tuned.cfgs, comps, s_comm, s_comp, args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    chained_tuned_us = lg.lagom_overlap_steps(launches, tuned.cfgs, comps, s_comm, s_comp, args.steps)
    torch.cuda.synchronize()
    chained_wall_ms = (time.perf_counter() - t0) * 1e3
    chained_default_us = lg.lagom_overlap_steps(launches, cands["default"], comps, s_comm, s_comp, args.steps)
    # the same sustained rate for three parameter sets, interleaved like the gated candidates above (the two figures
    # above stay: the first is what the host clock around K steps sees)
    chained_keys = [k for k in ("default", "tuned", "tuned_free_steps", "tuned_free_steps_extended_nt_min") if k in cands]
    chained_rounds = {k: [] for k in chained_keys}
    for r in range(args.rounds):
        for k in chained_keys[r % len(chained_keys):] + chained_keys[:r % len(chained_keys)]:
            chained_rounds[k].append(lg.lagom_overlap_steps(launches, cands[k], comps, s_comm, s_comp, args.steps))
    chained_interleaved = {}
    for k in chained_keys:
        ratio = np.array(chained_rounds["default"]) / np.array(chained_rounds[k])
        chained_interleaved[k] = {"us_per_step": float(np.median(chained_rounds[k])),
                                  "speedup_vs_default": [float(ratio.min()), float(np.median(ratio)), float(ratio.max())]}
    graph_tuned_us = lg.lagom_overlap_steps_graph(launches, tuned.cfgs, comps, s_comm, s_comp, args.steps)

    tflops = flops / gemm_us / 1e6
    roofline = {"bound": "mfma", "kernel": gemm_kernel_name(geo), "shape": f"{M}x{N}x{K}", "achieved": tflops, "peak": BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": tflops / BF16_PEAK_TFLOPS, "traffic": None,
                "traffic_from_profile": TRAFFIC_FROM_PROFILE.get(f"gemm {M}x{N}x{K}"),
                "us_per_launch": gemm_us, "flop_per_launch": flops, "launches_timed": args.rounds * args.steps * len(comps)}
    # the workload's own communication, standalone, at its fastest point of the extended sweep (buffers may sit in the last-level cache)
    fastest = min(all_sweep, key=lambda p: p.comm_alone_us)
    out = {
        "comm": f"{w.comm.op} {w.comm.dtype} S={w.comm.nsrc} count={w.comm.count} launches={len(launches)} comms={ncomm}",
        "gemm": f"{M}x{N}x{K} bf16 x{len(comps)}", "dependent": dependent,
        "speedup_tuned_vs_default": results["tuned"]["speedup_vs_default"], "verdict": results["tuned"]["verdict"],
        "z_default_us": results["default"]["z_us"], "z_tuned_us": results["tuned"]["z_us"],
        "z_default_chunk_clamped_us": results["default_chunk_clamped"]["z_us"],
        "speedup_tuned_vs_default_chunk_clamped": results["default_chunk_clamped"]["z_us"] / results["tuned"]["z_us"],
        "z_comm_descent_us": results["comm_descent"]["z_us"], "z_best_swept_us": results["best_swept"]["z_us"],
        "z_tuned_free_steps_us": results["tuned_free_steps"]["z_us"],
        "z_tuned_extended_us": results["tuned_extended"]["z_us"], "z_tuned_free_steps_extended_us": results["tuned_free_steps_extended"]["z_us"],
        "z_best_swept_extended_us": results["best_swept_extended"]["z_us"],
        "launches_fused": any(l.fuse for l in launches),
        "gemm_alone_us": gemm_us, "gemm_mfma_util": tflops / BF16_PEAK_TFLOPS,
        "comm_alone_fastest_us": fastest.comm_alone_us, "comm_alone_fastest_cfg": list(fastest.cfg),
        "comm_alone_fastest_gbps": sum(nbytes) / fastest.comm_alone_us / 1e3,
        "candidates": results, "searches": searches,
        "ladders": {"cut": [list(sp.chunk) for sp in spaces], "fixed_chunk": [list(sp.chunk) for sp in spaces_fixed],
                    "extended_nc": ext_nc, "extended_chunk": [list(sp.chunk) for sp in spaces_ext]},
        "model": {"corun_share": cal_all.sigma, "theta_us": cal_all.theta_us, "d_bytes": geo.d_bytes_past_l2,
                  "y_err_all_points": [cal_all.fit_mean, cal_all.fit_max],
                  "held_out": {"sigma_fitted_on_half": cal.sigma, "fit_half": [cal.fit_mean, cal.fit_max],
                               "held_half": [cal.held_mean, cal.held_max], "n_fit": cal.n_fit, "n_held": cal.n_held},
                  "resident_penalty": {"rho_by_nt": {str(k): v for k, v in cal_pen_all.penalty.items()}, "sigma": cal_pen_all.sigma,
                                       "y_err_all_points": [cal_pen_all.fit_mean, cal_pen_all.fit_max],
                                       "rho_fitted_on_half": {str(k): v for k, v in cal_pen.penalty.items()},
                                       "fit_half": [cal_pen.fit_mean, cal_pen.fit_max],
                                       "held_half": [cal_pen.held_mean, cal_pen.held_max]},
                  "uniform_pick_among_swept": uniform_picks,
                  "searches_with_rho": {k: {"cfgs": [list(c) for c in r.cfgs], "calls": r.calls, "predicted_z_us": r.Z,
                                            "measured_z_us": results[k]["z_us"],
                                            "speedup_vs_default": results[k]["speedup_vs_default"]}
                                        for k, r in model_pen_searches.items()},
                  "as_printed": {"d_bytes": geo.d_bytes, "theta_us": cal_printed.theta_us,
                                 "fit_half": [cal_printed.fit_mean, cal_printed.fit_max],
                                 "held_half": [cal_printed.held_mean, cal_printed.held_max]},
                  "tune_us": model_tune_us if tuned_model else None, "tune_calls": tuned_model.calls if tuned_model else None,
                  "predicted_z_us": tuned_model.Z if tuned_model else None,
                  "measured_z_us": results["model_tuned"]["z_us"] if tuned_model else None,
                  "printed_predicted_z_us": tuned_printed.Z if tuned_printed else None,
                  "printed_measured_z_us": results["printed_model_tuned"]["z_us"] if tuned_printed else None},
        "chained_us_per_step_tuned": chained_tuned_us, "chained_us_per_step_default": chained_default_us,
        "chained_wall_ms_per_step": chained_wall_ms / args.steps, "graph_us_per_step_tuned": graph_tuned_us,
        "chained_interleaved": chained_interleaved,
        "sweep_points": len(all_sweep), "sweep_seconds": sweep_s, "roofline": roofline,
    }
    # the computation-bound objective over the swept points: least GEMM slow-down among those whose communication
    # finishes inside the GEMM window (X <= Y); what LAGOM_HIDE_COMM searches for
    hidden = [p for p in all_sweep if p.comm_corun_us <= p.comp_corun_us]
    if hidden:
        p_min = min(hidden, key=lambda p: p.comp_corun_us)
        out["swept_min_slowdown_with_comm_hidden"] = {"cfg": list(p_min.cfg), "y_us": p_min.comp_corun_us, "x_us": p_min.comm_corun_us,
                                                      "gemm_slowdown": p_min.comp_corun_us / p_min.comp_alone_us,
                                                      "points_with_comm_hidden": len(hidden)}
    if first3 is not None:
        out["first_three_pairs_priority_vs_exhaustive"] = first3
    out["seconds"] = time.perf_counter() - t_start
    if args.dump:
        os.makedirs(args.dump, exist_ok=True)
        with open(os.path.join(args.dump, f"{name}{'_dependent' if dependent else ''}.json"), "w") as f:
            json.dump({"workload": name, "geometry": {"mu": geo.mu, "tb": geo.tb, "d_bytes": geo.d_bytes, "d_bytes_past_l2": geo.d_bytes_past_l2},
                       "ncomp": len(comps), "bytes_per_comm": bytes_per_comm, "per_src_bytes": per_src,
                       "sweep": [p.__dict__ for p in sweep], "sweep_extended": [p.__dict__ for p in sweep_ext],
                       "traces": {"priority": [s.__dict__ for s in tuned.trace], "priority_extended": [s.__dict__ for s in tuned_ext.trace],
                                  "priority_free_steps": [s.__dict__ for s in tuned_free.trace],
                                  "priority_free_steps_extended": [s.__dict__ for s in tuned_free_ext.trace],
                                  "hide_comm": [s.__dict__ for s in hide.trace]},
                       "logs": logs}, f, indent=1, default=str)
    del keep
    torch.cuda.empty_cache()
    return out


def standalone_only(args):
    """Every kernel of the benchmark alone, nothing that needs two kernels at once: the form to run under
    rocprofv3 --pmc, which serialises dispatches."""
    import torch
    from paper_2602_20656_amd import binding as lg
    s_comm, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    names = FIVE if args.workload == "all" else [args.workload]
    res = {}
    for name in names:
        w, launches, comps, ncomm, keep, _ = build_workload(name)
        M, N, K = w.gemm
        points = [(nc, 256, c) for nc in (8, 32, 256) for c in (w.chunk_grid[0], w.chunk_grid[-1])]
        comm_alone = [lg.lagom_overlap_run(launches, [p] * ncomm, comps, s_comm, s_comp, 1, 3, lg.LAGOM_ALONE_COMM).X_us for p in points]
        t_gemm = lg.lagom_overlap_run(launches, [DEFAULT_CFG] * ncomm, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_ALONE_COMP)
        gemm_us = sum(t_gemm.y_us) / len(comps)
        res[name] = {"gemm_alone_us": gemm_us, "gemm_mfma_util": 2.0 * M * N * K / gemm_us / 1e6 / BF16_PEAK_TFLOPS,
                     "fastest_comm_alone_us": min(comm_alone)}
        del keep
        torch.cuda.empty_cache()
    roofline_comm = standalone_comm_rooflines(s_comm, s_comp, 3)
    cal_src = torch.empty(16 << 20, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    cal_dst = torch.empty_like(cal_src)
    torch.cuda.synchronize()
    lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, lg.LAGOM_F32, [cal_src], [cal_dst], 16 << 20, (1000, 512, 64 << 10), s_comm)
    torch.cuda.synchronize()
    print(json.dumps({"mode": "standalone-only", "configs": res, "roofline_comm": roofline_comm}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all", choices=["all"] + FIVE + ["ep_alltoall", "rs_ag_pair", "tp_pipeline"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-iters", type=int, default=7)
    ap.add_argument("--rounds", type=int, default=3, help="interleaved rounds of the tuned-versus-default comparison")
    ap.add_argument("--profile-min-us", type=float, default=20000.0, help="ProfileTime measures a group for at least this long")
    ap.add_argument("--profile-max-iters", type=int, default=100)
    ap.add_argument("--dependent", action="store_true",
                    help="fsdp_chain only: GEMM i (i > 0) consumes the weight gathered by communication i-1 and waits for it")
    ap.add_argument("--dump", default=None, help="directory for per-workload JSON files with the sweep tables, tuner traces and profile logs")
    ap.add_argument("--standalone-only", action="store_true",
                    help="run every kernel alone and nothing that needs two kernels at once: the form for rocprofv3 --pmc")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the overlapped step; run with --gpus 1 "
              "(peer buffers are emulated in this GPU's HBM, there is no multi-GPU path)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_20656_amd import binding as lg
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.standalone_only:
        standalone_only(args)
        return
    s_comm, s_comp = lg.overlapping_streams()
    names = FIVE if args.workload == "all" else [args.workload]
    headline = HEADLINE if args.workload == "all" else args.workload
    configs = {}
    for name in names:
        configs[name] = run_config(name, args, s_comm, s_comp, dependent=args.dependent and name == "fsdp_chain")
        print(f"bench: {name} done in {configs[name]['seconds']:.1f} s, tuned/default "
              f"{configs[name]['speedup_tuned_vs_default'][1]:.3f}x ({configs[name]['verdict']})", file=sys.stderr, flush=True)
    roofline_comm = standalone_comm_rooflines(s_comm, s_comp, 5)

    # one plain copy of known size (64 MiB read, 64 MiB written): the reference that rocprofv3's FETCH_SIZE /
    # WRITE_SIZE readings of the other kernels are scaled by
    cal_src = torch.empty(16 << 20, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    cal_dst = torch.empty_like(cal_src)
    torch.cuda.synchronize()
    lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, lg.LAGOM_F32, [cal_src], [cal_dst], 16 << 20, (1000, 512, 64 << 10), s_comm)
    torch.cuda.synchronize()

    h = configs[headline]
    out = {
        "metric": "overlap makespan speedup vs default params",
        "value": h["speedup_tuned_vs_default"][1],
        "unit": "x",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": h["chained_wall_ms_per_step"],      # K back-to-back steps of the headline workload with the tuned parameters
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": headline + ("+dependent" if h["dependent"] else ""), "comm": h["comm"], "gemm": h["gemm"],
                   "default_cfg": list(DEFAULT_CFG), "tuned_cfgs": h["candidates"]["tuned"]["cfgs"], "rounds": args.rounds},
        "value_min_median_max": h["speedup_tuned_vs_default"], "verdict": h["verdict"],
        # the same ratio for the other searches of the headline workload (min, median, max over the rounds): Alg. 1/2 with
        # free steps on the fixed-chunk ladder of the task's grids; the same on the extended space (NC up to 256, channels of
        # two wavefronts), driven by measurements and driven by the cost model with the resident penalty (no measurement
        # during the search); the communication-only descent; the best point of the profiler's sweeps
        "value_other_searches": {k: h["candidates"][k]["speedup_vs_default"] for k in
                                 ("tuned_free_steps", "tuned_free_steps_extended_nt_min", "model_rho_free_steps_extended_nt_min",
                                  "comm_descent", "best_swept", "best_swept_extended")
                                 if k in h["candidates"]},
        "value_sustained": h["chained_interleaved"]["tuned"]["speedup_vs_default"],   # the same ratio over back-to-back steps, no gate
        # what the paper reports on its own hardware (abstract, Sec. 5), end to end over whole training iterations: context
        # for the ratios above, which are one overlap group on one MI355X against default parameters of this kernel
        "paper_context": {"iteration_speedup_over_nccl": [1.07, 1.33], "iteration_speedup_over_autoccl": [1.03, 1.27],
                          "hardware": "2 nodes x 8 NVIDIA A40, NVLink or PCIe 4.0, InfiniBand; NCCL 2.18.3"},
        "z_tuned_us": h["z_tuned_us"], "z_default_us": h["z_default_us"],
        "comm_hbm_gbps": roofline_comm["achieved"], "gemm_mfma_util": h["gemm_mfma_util"],
        "gemm_mfma_util_by_shape": {c["roofline"]["shape"]: c["roofline"]["frac"] for c in configs.values()},
        "roofline": h["roofline"], "roofline_comm": roofline_comm,
        "configs": configs,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(headline)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
