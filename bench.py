#!/usr/bin/env python3
"""Benchmark of the Lagom hot path on one MI355X.

One "step" is one pass of the whole overlapped group of the chosen workload (every
communication launch on one stream, every GEMM on the other, through lagom_overlap_run)
with the parameters the priority search picked.  Before the timed region the contention
profiler sweeps the workload's (NC, C[, NT]) grid, the cost model is filled from it, and
lagom_tune runs once with measured profiles and once with the model.

Prints ONE JSON line:  value = makespan(default NC=8, C=2 MiB, NT=256) / makespan(tuned).
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
# Bytes past L2 per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the same counters' reading of a plain
# 64 MiB copy (factors 1.9986 and 0.9994); figures and commands: profiles/bench_dp_bucket_hbm_counters.md
MEASURED_TRAFFIC_BYTES = {
    "gemm 4096x4096x4096": int(224.3 * (1 << 20)),
    "reduce_copy bf16 S=8 D=1 count=4194304": int(72.0 * (1 << 20)),
    "reduce_copy f32 S=2 D=1 count=4194304": int(48.0 * (1 << 20)),
}
DEFAULT_CFG = (8, 256, 2 << 20)  # the collective library default the paper quotes (Sec. 4.3), NT from the tiny config


def _up(x):
    import torch
    return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()


def build_workload(name: str, dependent: bool = False):
    """Device buffers + launch descriptors of one of the five synthetic overlap groups."""
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
        pipeline_outputs = []                                                  # filled with the GEMM outputs below
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
    return w, launches, comps, ncomm, keep, (comp_after_comm, comm_after_comp)


def comm_bytes(launches):
    from paper_2602_20656_amd import binding as lg
    return [lg.lagom_comm_bytes(l.op, l.dtype, len(l.srcs), len(l.dsts), l.count) for l in launches]


def standalone_comm_roofline(st1, st2, iters, final_iters=20):
    """Best standalone reduce-copy bandwidth over an extended NC set, on buffers rotated through
    more than the 256 MB last-level cache so that HBM has to serve them.  Two shapes of the
    workloads are tried: the two-source fp32 reduce of 16 MiB buffers and the eight-source bf16
    reduce of 8 MiB shards."""
    import torch
    from paper_2602_20656_amd import binding as lg
    shapes = [("reduce_copy f32 S=2 D=1 count=4194304", lg.LAGOM_F32, torch.float32, 2, 4194304, 12),
              ("reduce_copy bf16 S=8 D=1 count=4194304", lg.LAGOM_BF16, torch.bfloat16, 8, 4194304, 8)]
    best, best_shape = None, None
    for shape in shapes:
        name, dt, tdt, nsrc, count, nrot = shape
        bufs = [[torch.empty(count, dtype=torch.float32, device="cuda").uniform_(-1, 1).to(tdt) for _ in range(nsrc + 1)]
                for _ in range(nrot)]
        launches = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, b[:nsrc], [b[nsrc]], count, 0) for b in bufs]
        per_launch = lg.lagom_comm_bytes(lg.LAGOM_REDUCE_COPY, dt, nsrc, 1, count)
        for nc in (256, 512, 1024):
            for nt in (512, 1024):
                for chunk in (16 << 10, 32 << 10, 64 << 10, 128 << 10):
                    t = lg.lagom_overlap_run(launches, [(nc, nt, chunk)], [], st1, st2, 1, iters, lg.LAGOM_ALONE_COMM)
                    us = t.X_us / nrot
                    gbps = per_launch / us / 1e3
                    if best is None or gbps > best["achieved"]:
                        best_shape = shape
                        best = {"bound": "hbm", "kernel": "reduce_copy_kernel", "workload": name, "achieved": gbps,
                                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                                "traffic": MEASURED_TRAFFIC_BYTES.get(name),
                                "us_per_launch": us, "bytes_per_launch": per_launch, "cfg": [nc, nt, chunk],
                                "rotation_mib": nrot * per_launch >> 20}
        del bufs, launches
    name, dt, tdt, nsrc, count, nrot = best_shape
    # context only: the same operator on an 8 times longer buffer (576 MiB per launch, two rotated sets), where the
    # fixed cost of a launch weighs less: what the kernel sustains once a launch is long enough
    try:
        big = count * 8
        bufs = [[torch.empty(big, dtype=torch.float32, device="cuda").uniform_(-1, 1).to(tdt) for _ in range(nsrc + 1)]
                for _ in range(2)]
        launches = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, b[:nsrc], [b[nsrc]], big, 0) for b in bufs]
        big_bytes = lg.lagom_comm_bytes(lg.LAGOM_REDUCE_COPY, dt, nsrc, 1, big)
        cands = [tuple(best["cfg"]), (1024, 1024, 16 << 10), (2048, 1024, 16 << 10), (4096, 512, 8 << 10), (4096, 1024, 16 << 10)]
        t_big = min((lg.lagom_overlap_run(launches, [c], [], st1, st2, 1, iters, lg.LAGOM_ALONE_COMM).X_us / 2, c) for c in cands)
        best["long_launch"] = {"count": big, "bytes_per_launch": big_bytes, "cfg": list(t_big[1]), "us_per_launch": t_big[0],
                               "achieved": big_bytes / t_big[0] / 1e3, "frac": big_bytes / t_big[0] / 1e3 / HBM_PEAK_GBPS}
        del bufs, launches
    except RuntimeError:
        best["long_launch"] = None
    # context only: the vendor's device-to-device copy (torch's copy_) moving the same number of bytes per launch,
    # half read and half written, on buffers rotated the same way, launches back to back
    try:
        half = best["bytes_per_launch"] // 2
        pairs = [(torch.empty(half, dtype=torch.uint8, device="cuda").random_(), torch.empty(half, dtype=torch.uint8, device="cuda"))
                 for _ in range(nrot)]
        for src, dst in pairs:
            dst.copy_(src)
        torch.cuda.synchronize()
        times = []
        for _ in range(final_iters):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for src, dst in pairs:
                dst.copy_(src)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3 / nrot)
        v_us = float(np.median(times))
        best.update({"vendor_copy_us_per_launch": v_us, "vendor_copy_gbps": 2 * half / v_us / 1e3})
        del pairs
    except RuntimeError:
        best.update({"vendor_copy_us_per_launch": None, "vendor_copy_gbps": None})
    # the figure that is reported, measured last: the winning configuration once more, final_iters passes of nrot launches each
    # (these are the last dispatches of that kernel in a trace of this run)
    bufs = [[torch.empty(count, dtype=torch.float32, device="cuda").uniform_(-1, 1).to(tdt) for _ in range(nsrc + 1)]
            for _ in range(nrot)]
    launches = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, dt, b[:nsrc], [b[nsrc]], count, 0) for b in bufs]
    t = lg.lagom_overlap_run(launches, [tuple(best["cfg"])], [], st1, st2, 2, final_iters, lg.LAGOM_ALONE_COMM)
    us = t.X_us / nrot
    best.update({"achieved": best["bytes_per_launch"] / us / 1e3, "frac": best["bytes_per_launch"] / us / 1e3 / HBM_PEAK_GBPS,
                 "us_per_launch": us, "launches_timed": nrot * final_iters})
    del bufs, launches
    return best


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
    return {"value": comm_us + gemm_us, "unit": "us/step", "cores": threads, "kind": "oracle",
            "sample": f"communication launches at full size ({comm_us:.0f} us); GEMM rows 0..{rows} of {M}, all columns and K, "
                      f"scaled by {M / rows:.1f} ({gemm_us:.0f} us); no overlap on the CPU",
            "comm_us": comm_us, "gemm_us": gemm_us}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="dp_bucket", choices=["tiny", "dp_bucket", "tp_layer", "fsdp_chain", "compute_bound", "ep_alltoall", "rs_ag_pair", "tp_pipeline"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-iters", type=int, default=5)
    ap.add_argument("--dependent", action="store_true",
                    help="fsdp_chain only: GEMM i (i > 0) consumes the weight gathered by communication i-1 and waits for it")
    ap.add_argument("--dump", default=None, help="write the sweep table and tuner traces to this JSON file")
    ap.add_argument("--standalone-only", action="store_true",
                    help="run every kernel of the benchmark alone (the sweep's communication launches, the GEMM, the standalone "
                         "roofline passes, the calibration copy) and nothing that needs two kernels at once: the form to run under "
                         "rocprofv3 --pmc, which serialises dispatches")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the overlapped step; run with --gpus 1 "
              "(peer buffers are emulated in this GPU's HBM, there is no multi-GPU path)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_20656_amd import binding as lg
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    s_comm, s_comp = (torch.cuda.Stream(), torch.cuda.Stream()) if args.standalone_only else lg.overlapping_streams()

    dependent = args.dependent and args.workload == "fsdp_chain"
    w, launches, comps, ncomm, keep, (dep_arg, dep_comm) = build_workload(args.workload, dependent)
    dependent = dep_arg is not None or dep_comm is not None
    nbytes = comm_bytes(launches)
    M, N, K = w.gemm
    flops = 2.0 * M * N * K

    # ---- contention profiler over the workload's grid (NT fixed at 256 unless the workload sweeps it)
    points = [(nc, nt, c) for nt in w.nt_grid for nc in w.nc_grid for c in w.chunk_grid]
    if args.standalone_only:
        comm_alone = [lg.lagom_overlap_run(launches, [p] * ncomm, comps, s_comm, s_comp, 1, args.sweep_iters, lg.LAGOM_ALONE_COMM).X_us
                      for p in points]
        t_gemm = lg.lagom_overlap_run(launches, [DEFAULT_CFG] * ncomm, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_ALONE_COMP)
        gemm_us = t_gemm.Y_us / len(comps)
        roofline_comm = standalone_comm_roofline(s_comm, s_comp, 5)
        cal_src = torch.empty(16 << 20, dtype=torch.float32, device="cuda").uniform_(-1, 1)
        cal_dst = torch.empty_like(cal_src)
        lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, lg.LAGOM_F32, [cal_src], [cal_dst], 16 << 20, (1000, 512, 64 << 10), s_comm)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "standalone-only", "config": {"workload": args.workload}, "gemm_alone_us": gemm_us,
                          "gemm_mfma_util": flops / gemm_us / 1e6 / BF16_PEAK_TFLOPS, "roofline_comm": roofline_comm,
                          "fastest_comm_alone_us": min(comm_alone), "sweep_points": len(points)}))
        return
    t0 = time.perf_counter()
    sweep = lg.lagom_contention_sweep(launches, ncomm, comps, points, s_comm, s_comp, 1, args.sweep_iters)
    sweep_s = time.perf_counter() - t0

    # ---- cost model filled from the sweep: x and V per configuration, theta fitted to the standalone GEMM
    geo = lg.lagom_gemm_describe(M, N, K)
    bw = HBM_PEAK_GBPS * 1e3                                     # bytes per microsecond
    y_alone = float(np.median([p.comp_alone_us for p in sweep])) / len(comps)
    g0 = -(-geo.mu // (LAMBDA * geo.tb))
    # the sweep times the communication stream as a whole; a communication's x is its share of the bytes
    share = [sum(b for b, l in zip(nbytes, launches) if l.comm_id == j) / sum(nbytes) for j in range(ncomm)]
    tables = [{p.cfg: (p.comm_corun_us * share[j], min(p.v_corun, 0.99 * bw)) for p in sweep} for j in range(ncomm)]

    def make_model(d_bytes, sigma):
        theta = max(0.0, y_alone / g0 - LAMBDA * geo.tb * d_bytes / bw)
        return lg.Model(LAMBDA, bw, [lg.CompModel(geo.mu, geo.tb, d_bytes, theta) for _ in comps], tables,
                        comp_after_comm=dep_arg, comm_after_comp=dep_comm, corun_share=sigma), theta

    def y_errors(mdl):   # predicted Y against the measured Y of every sweep point the model was filled from
        e = [abs(lg.lagom_cost_model(mdl, [pt.cfg] * ncomm).Y_us - pt.comp_corun_us) / pt.comp_corun_us for pt in sweep]
        return float(np.mean(e)), float(np.max(e))

    # (1) the model as printed: D = all bytes a workgroup reads and writes, a channel takes a compute unit (Eq. 5)
    model_printed, theta_printed = make_model(geo.d_bytes, 0.0)
    printed_mape, printed_max = y_errors(model_printed)
    # (2) calibrated to this part: D = the bytes that leave the XCD's L2, and the share sigma of a channel's
    #     compute unit that stays with the GEMM (its wavefronts run beside the GEMM's) fitted to the sweep
    fits = []
    for sigma in [i / 8 for i in range(9)]:
        mdl, th = make_model(geo.d_bytes_past_l2, sigma)
        fits.append((y_errors(mdl), sigma, mdl, th))
    (model_y_mape, model_y_max), sigma_fit, model, theta = min(fits, key=lambda f: f[0][0])

    # ---- the search: Alg. 1/2 with measured profiles, and with the model as ProfileTime
    nt_grid = list(w.nt_grid) if len(w.nt_grid) > 1 else [256]
    # The ladder's chunk grid is cut where a chunk would exceed (bytes one launch moves per source) / NC_max:
    # beyond that point part of the channels of every launch have no chunk to move (chunk g goes to channel
    # g mod NC), so a higher level could only be slower.  The profiler still sweeps the full grid.
    spaces = []
    for j in range(ncomm):
        esz = 4 if w.comm.dtype == "f32" else 2
        per_src = min(l.count * esz * (len(l.srcs) if l.op == lg.LAGOM_GATHER_COPY else 1) for l in launches if l.comm_id == j)
        cut = [c for c in w.chunk_grid if c * max(w.nc_grid) <= per_src] or [min(w.chunk_grid)]
        spaces.append(lg.Space(list(w.nc_grid), nt_grid, cut))
    ladder_ok = all(tuple(c) in tables[0] for c in
                    [(spaces[0].nc[min(l, len(spaces[0].nc) - 1)], spaces[0].nt[min(l, len(spaces[0].nt) - 1)],
                      spaces[0].chunk[min(l, len(spaces[0].chunk) - 1)]) for l in range(max(len(spaces[0].nc), len(spaces[0].nt), len(spaces[0].chunk)))])
    t0 = time.perf_counter()
    tuned = lg.lagom_tune(spaces, lg.OverlapProfile(launches, comps, s_comm, s_comp, 1, args.sweep_iters), lg.LAGOM_PRIORITY)
    tune_s = time.perf_counter() - t0
    t0 = time.perf_counter()
    tuned_model = lg.lagom_tune(spaces, model, lg.LAGOM_PRIORITY) if ladder_ok else None
    model_tune_us = (time.perf_counter() - t0) * 1e6      # host only: Alg. 1/2 with the native cost-model callback (binding marshalling included)
    tuned_printed = lg.lagom_tune(spaces, model_printed, lg.LAGOM_PRIORITY) if ladder_ok else None
    # the communication-bound reference (Eq. 2): per-communication coordinate descent on x_j alone
    comm_cd = lg.lagom_tune(spaces, lg.OverlapProfile(launches, comps, s_comm, s_comp, 1, args.sweep_iters), lg.LAGOM_COMM_OPTIMAL)

    # ---- the first three pairs of the chain: priority search against exhaustive search over the same ladder
    #      (216 level vectors), with measured profiles and with the calibrated model as ProfileTime
    first3 = None
    if args.workload == "fsdp_chain" and ncomm >= 3 and ladder_ok:
        l3 = [l for l in launches if l.comm_id < 3]
        c3 = comps[:3]
        sp3 = [lg.Space(sp.nc[:6], sp.nt, sp.chunk[:6]) for sp in spaces[:3]]
        prof3 = lg.OverlapProfile(l3, c3, s_comm, s_comp, 1, args.sweep_iters)
        model3 = lg.Model(model.lam, model.bw_peak, model.comps[:3], model.tables[:3],
                          comp_after_comm=dep_arg[:3] if dep_arg else None, corun_share=model.corun_share)
        t0 = time.perf_counter()
        pr_meas, ex_meas = lg.lagom_tune(sp3, prof3, lg.LAGOM_PRIORITY), lg.lagom_tune(sp3, prof3, lg.LAGOM_EXHAUSTIVE)
        first3_s = time.perf_counter() - t0
        pr_mod, ex_mod = lg.lagom_tune(sp3, model3, lg.LAGOM_PRIORITY), lg.lagom_tune(sp3, model3, lg.LAGOM_EXHAUSTIVE)
        run3 = lambda cfgs: lg.lagom_overlap_run(l3, cfgs, c3, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_CORUN).Z_us
        first3 = {"ladder_levels": [max(len(sp.nc), len(sp.nt), len(sp.chunk)) for sp in sp3],
                  "measured": {"priority_cfgs": [list(c) for c in pr_meas.cfgs], "priority_calls": pr_meas.calls,
                               "exhaustive_cfgs": [list(c) for c in ex_meas.cfgs], "exhaustive_calls": ex_meas.calls,
                               "z_priority_us": run3(pr_meas.cfgs), "z_exhaustive_us": run3(ex_meas.cfgs), "seconds": first3_s},
                  "model": {"priority_cfgs": [list(c) for c in pr_mod.cfgs], "priority_calls": pr_mod.calls,
                            "exhaustive_cfgs": [list(c) for c in ex_mod.cfgs], "exhaustive_calls": ex_mod.calls,
                            "z_priority_model_us": pr_mod.Z, "z_exhaustive_model_us": ex_mod.Z,
                            "z_priority_us": run3(pr_mod.cfgs), "z_exhaustive_us": run3(ex_mod.cfgs)}}

    # ---- timed region: W warm-up steps, then exactly K steps with the tuned parameters
    default_cfgs = [DEFAULT_CFG] * ncomm
    lg.lagom_overlap_run(launches, tuned.cfgs, comps, s_comm, s_comp, args.warmup, 1, lg.LAGOM_CORUN)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    t_tuned = lg.lagom_overlap_run(launches, tuned.cfgs, comps, s_comm, s_comp, 0, args.steps, lg.LAGOM_CORUN)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    t_default = lg.lagom_overlap_run(launches, default_cfgs, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_CORUN)
    # the same K steps once more as a training loop would run them: enqueued back to back, streams joined by events only
    lg.lagom_overlap_steps(launches, tuned.cfgs, comps, s_comm, s_comp, args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    chained_tuned_us = lg.lagom_overlap_steps(launches, tuned.cfgs, comps, s_comm, s_comp, args.steps)
    torch.cuda.synchronize()
    chained_wall_ms = (time.perf_counter() - t0) * 1e3
    chained_default_us = lg.lagom_overlap_steps(launches, default_cfgs, comps, s_comm, s_comp, args.steps)
    t0 = time.perf_counter()
    graph_tuned_us = lg.lagom_overlap_steps_graph(launches, tuned.cfgs, comps, s_comm, s_comp, args.steps)
    graph_wall_ms = (time.perf_counter() - t0) * 1e3      # includes capture, instantiation and one eager repetition
    best_sweep = min(sweep, key=lambda p: p.z_corun_us)
    comm_opt = min(sweep, key=lambda p: p.comm_alone_us)
    t_commopt = lg.lagom_overlap_run(launches, [comm_opt.cfg] * ncomm, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_CORUN)
    t_commcd = lg.lagom_overlap_run(launches, comm_cd.cfgs, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_CORUN)
    t_model = (lg.lagom_overlap_run(launches, tuned_model.cfgs, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_CORUN)
               if tuned_model else None)
    t_printed = (lg.lagom_overlap_run(launches, tuned_printed.cfgs, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_CORUN)
                 if tuned_printed else None)

    # ---- roofline of the dominant kernel (the GEMM), measured live with HIP events on its own stream
    t_gemm = lg.lagom_overlap_run(launches, default_cfgs, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_ALONE_COMP)
    gemm_us = t_gemm.Y_us / len(comps)
    tflops = flops / gemm_us / 1e6
    roofline = {"bound": "mfma", "kernel": "gemm_bf16_nk_kernel", "achieved": tflops, "peak": BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": tflops / BF16_PEAK_TFLOPS,
                "traffic": MEASURED_TRAFFIC_BYTES.get(f"gemm {M}x{N}x{K}"),
                "us_per_launch": gemm_us, "flop_per_launch": flops}
    # context only: the vendor BLAS for the same product (torch.matmul), timed the same way -- one event pair per launch
    vendor_us = None
    try:
        tA = torch.randn(M, K, device="cuda").bfloat16()
        tB = (torch.randn(N, K, device="cuda") * 0.02).bfloat16()
        with torch.cuda.stream(s_comp):
            for _ in range(args.warmup):
                torch.matmul(tA, tB.t())
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for e0, e1 in ev:
                e0.record(); torch.matmul(tA, tB.t()); e1.record()
        torch.cuda.synchronize()
        vendor_us = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3
        del tA, tB
    except Exception:        # the reference is optional; the bench line does not depend on it
        vendor_us = None
    roofline_comm = standalone_comm_roofline(s_comm, s_comp, 5)
    # the workload's own communication, standalone, at its fastest swept point
    t_comm = lg.lagom_overlap_run(launches, [comm_opt.cfg] * ncomm, comps, s_comm, s_comp, args.warmup, args.steps, lg.LAGOM_ALONE_COMM)

    # one plain copy of known size (64 MiB read, 64 MiB written): the reference that rocprofv3's FETCH_SIZE /
    # WRITE_SIZE readings of the other kernels are scaled by
    cal_src = torch.empty(16 << 20, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    cal_dst = torch.empty_like(cal_src)
    lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, lg.LAGOM_F32, [cal_src], [cal_dst], 16 << 20, (1000, 512, 64 << 10), s_comm)
    torch.cuda.synchronize()

    out = {
        "metric": "overlap makespan speedup vs default params",
        "value": t_default.Z_us / t_tuned.Z_us,
        "unit": "x",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": chained_wall_ms / args.steps,       # K back-to-back steps with the tuned parameters, host clock between synchronisations
        "gated_wall_ms_per_step": wall_ms / args.steps,    # the same K steps run one by one behind a start gate (what z_tuned_us is the median of)
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload + ("+dependent" if dependent else ""), "comm": f"{w.comm.op} {w.comm.dtype} S={w.comm.nsrc} count={w.comm.count} "
                   f"launches={len(launches)} comms={ncomm}", "gemm": f"{M}x{N}x{K} bf16 x{len(comps)}",
                   "default_cfg": list(DEFAULT_CFG), "tuned_cfgs": [list(c) for c in tuned.cfgs],
                   "ladder_chunk_grids": [list(sp.chunk) for sp in spaces]},
        "z_tuned_us": t_tuned.Z_us, "z_default_us": t_default.Z_us,
        "chained_us_per_step_tuned": chained_tuned_us, "chained_us_per_step_default": chained_default_us,
        "chained_speedup": chained_default_us / chained_tuned_us,
        "graph_us_per_step_tuned": graph_tuned_us, "graph_call_wall_ms": graph_wall_ms,
        "x_tuned_us": t_tuned.X_us, "y_tuned_us": t_tuned.Y_us, "x_default_us": t_default.X_us, "y_default_us": t_default.Y_us,
        "z_comm_optimal_us": t_commopt.Z_us, "comm_optimal_cfg": list(comm_opt.cfg),
        "z_comm_descent_us": t_commcd.Z_us, "comm_descent_cfgs": [list(c) for c in comm_cd.cfgs], "comm_descent_calls": comm_cd.calls,
        "z_best_swept_us": best_sweep.z_corun_us, "best_swept_cfg": list(best_sweep.cfg),
        "z_model_tuned_us": t_model.Z_us if t_model else None,
        "model_tuned_cfgs": [list(c) for c in tuned_model.cfgs] if tuned_model else None,
        "model_predicted_z_us": lg.lagom_cost_model(model, tuned_model.cfgs).Z_us if tuned_model else None,
        "model_y_mean_abs_rel_err": model_y_mape, "model_y_max_abs_rel_err": model_y_max,
        "model_corun_share": sigma_fit, "model_d_bytes": geo.d_bytes_past_l2, "model_theta_us": theta,
        "printed_model_y_mean_abs_rel_err": printed_mape, "printed_model_y_max_abs_rel_err": printed_max,
        "printed_model_d_bytes": geo.d_bytes, "printed_model_theta_us": theta_printed,
        "z_printed_model_tuned_us": t_printed.Z_us if t_printed else None,
        "printed_model_predicted_z_us": lg.lagom_cost_model(model_printed, tuned_printed.cfgs).Z_us if tuned_printed else None,
        "model_tune_us": model_tune_us if tuned_model else None, "model_tune_profile_calls": tuned_model.calls if tuned_model else None,
        "tune_profile_calls": tuned.calls, "tune_seconds": tune_s, "sweep_points": len(points), "sweep_seconds": sweep_s,
        "gemm_alone_us": gemm_us, "gemm_mfma_util": tflops / BF16_PEAK_TFLOPS,
        "vendor_blas_gemm_us": vendor_us, "vendor_blas_mfma_util": (flops / vendor_us / 1e6 / BF16_PEAK_TFLOPS) if vendor_us else None,
        "gemm_slowdown_default": t_default.Y_us / t_gemm.Y_us, "gemm_slowdown_tuned": t_tuned.Y_us / t_gemm.Y_us,
        "comm_alone_us": t_comm.X_us, "comm_alone_gbps": sum(nbytes) / t_comm.X_us / 1e3,
        "comm_hbm_gbps": roofline_comm["achieved"],
        "roofline": roofline, "roofline_comm": roofline_comm,
    }
    # the compute-bound objective: the swept point with the least GEMM slow-down among those whose communication
    # still finishes inside the GEMM window (X <= Y)
    hidden = [p for p in sweep if p.comm_corun_us <= p.comp_corun_us]
    if hidden:
        p_min = min(hidden, key=lambda p: p.comp_corun_us)
        out["min_slowdown_with_comm_hidden"] = {"cfg": list(p_min.cfg), "y_us": p_min.comp_corun_us, "x_us": p_min.comm_corun_us,
                                                "gemm_slowdown": p_min.comp_corun_us / p_min.comp_alone_us,
                                                "points_with_comm_hidden": len(hidden)}
    if first3 is not None:
        out["first_three_pairs_priority_vs_exhaustive"] = first3
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    if args.dump:
        with open(args.dump, "w") as f:
            json.dump({"sweep": [p.__dict__ for p in sweep],
                       "trace": [s.__dict__ for s in tuned.trace],
                       "model_trace": [s.__dict__ for s in tuned_model.trace] if tuned_model else None,
                       "theta_us": theta, "geometry": {"mu": geo.mu, "tb": geo.tb, "d_bytes": geo.d_bytes}}, f, indent=1, default=str)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
