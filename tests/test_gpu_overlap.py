"""GPU checks of the overlap runner, the contention profiler and the measured tuner."""
import numpy as np
import pytest
import torch

from oracle import collective as oc, gemm as og
from paper_2602_20656_amd import binding as lg, inputs
from gpu_util import dev, host, same_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tiny():
    a, b = inputs.uniform_f32(0, 1 << 20), inputs.uniform_f32(1, 1 << 20)
    A, B = inputs.normal_bf16(2, (512, 512)), inputs.normal_bf16(3, (512, 512))
    d = dict(a=a, b=b, A=A, B=B, da=dev(a), db=dev(b), dout=dev(np.zeros(1 << 20, np.float32)),
             dA=dev(A), dB=dev(B), dC=dev(np.zeros((512, 512), np.uint16)),
             s1=None, s2=None)
    d["s1"], d["s2"] = lg.overlapping_streams()
    d["launches"] = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [d["da"], d["db"]], [d["dout"]], 1 << 20, 0)]
    d["comps"] = [lg.GemmDesc(d["dA"], d["dB"], d["dC"], 512, 512, 512)]
    return d


def test_corun_keeps_both_results_correct_and_times_are_consistent(tiny):
    t = lg.lagom_overlap_run(tiny["launches"], [(4, 256, 128 << 10)], tiny["comps"], tiny["s1"], tiny["s2"], 2, 10, lg.LAGOM_CORUN)
    torch.cuda.synchronize()
    assert same_bits(host(tiny["dout"], np.float32), oc.reduce_copy([tiny["a"], tiny["b"]], oc.F32)[0])
    got = oc.bf16_to_f32(host(tiny["dC"], np.uint16))
    e_max, e_fro = og.rel_errors(got, og.gemm_f64(tiny["A"], tiny["B"], True))
    assert e_max <= 2e-2 and e_fro <= 2e-2
    assert t.X_us > 0 and t.Y_us > 0 and t.Z_us >= max(t.X_us, t.Y_us) * 0.999
    assert t.x_us[0] == pytest.approx(t.X_us, rel=0.5) and t.y_us[0] == pytest.approx(t.Y_us, rel=0.5)
    for mode, which in [(lg.LAGOM_ALONE_COMM, "X_us"), (lg.LAGOM_ALONE_COMP, "Y_us")]:
        r = lg.lagom_overlap_run(tiny["launches"], [(4, 256, 128 << 10)], tiny["comps"], tiny["s1"], tiny["s2"], 1, 5, mode)
        assert getattr(r, which) > 0


def test_both_streams_are_released_at_the_same_instant(tiny):
    """The start gate: the first kernels of the two streams start within a few microseconds of each other (an event wait
    across streams would release the computation stream 6 - 7 us late), Z is the later of the two ends, and a stream that
    does not run reports no release."""
    for cfg in [(4, 256, 128 << 10), (64, 256, 64 << 10)]:
        t = lg.lagom_overlap_run(tiny["launches"], [cfg], tiny["comps"], tiny["s1"], tiny["s2"], 3, 15, lg.LAGOM_CORUN)
        print(f"\nrelease after the gate: communication {t.comm_start_us:.2f} us, computation {t.comp_start_us:.2f} us; "
              f"X {t.X_us:.1f} Y {t.Y_us:.1f} Z {t.Z_us:.1f}")
        assert t.comm_start_us >= 0.0 and t.comp_start_us >= 0.0
        assert abs(t.comm_start_us - t.comp_start_us) <= 4.0
        later_end = max(t.comm_start_us + t.X_us, t.comp_start_us + t.Y_us)
        assert t.Z_us == pytest.approx(later_end, abs=3.0)          # medians of different repetitions: not an identity
    r = lg.lagom_overlap_run(tiny["launches"], [(4, 256, 128 << 10)], tiny["comps"], tiny["s1"], tiny["s2"], 1, 5, lg.LAGOM_ALONE_COMM)
    assert r.comp_start_us == 0.0 and r.comm_start_us >= 0.0


def test_streams_that_share_a_hardware_queue_are_detected_and_refused(tiny):
    assert lg.lagom_streams_overlap(tiny["s1"], tiny["s2"]) and not lg.lagom_streams_overlap(tiny["s1"], tiny["s1"])
    pool = [torch.cuda.Stream() for _ in range(8)]        # HIP has 4 hardware queues per process by default
    shared = [(a, b) for i, a in enumerate(pool) for b in pool[i + 1:] if not lg.lagom_streams_overlap(a, b)]
    if not shared:
        pytest.skip("every pair of eight streams overlapped")
    a, b = shared[0]
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_overlap_run(tiny["launches"], [(4, 256, 65536)], tiny["comps"], a, b, 0, 1, lg.LAGOM_CORUN)
    assert e.value.code == lg.LAGOM_EINVAL and "hardware queue" in str(e.value)
    # the alone modes use one stream only and take any pair
    assert lg.lagom_overlap_run(tiny["launches"], [(4, 256, 65536)], tiny["comps"], a, b, 0, 1, lg.LAGOM_ALONE_COMM).X_us > 0


def test_runner_rejects_bad_groups(tiny):
    with pytest.raises(lg.LagomError):   # same stream for both
        lg.lagom_overlap_run(tiny["launches"], [(4, 256, 65536)], tiny["comps"], tiny["s1"], tiny["s1"], 1, 1, lg.LAGOM_CORUN)
    with pytest.raises(lg.LagomError):   # comm_id out of range
        bad = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [tiny["da"]], [tiny["dout"]], 16, 3)]
        lg.lagom_overlap_run(bad, [(4, 256, 65536)], tiny["comps"], tiny["s1"], tiny["s2"], 1, 1, lg.LAGOM_CORUN)
    with pytest.raises(lg.LagomError):   # non-contiguous ids
        l0 = lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [tiny["da"]], [tiny["dout"]], 16, 0)
        l1 = lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [tiny["da"]], [tiny["dout"]], 16, 1)
        lg.lagom_overlap_run([l0, l1, l0], [(4, 256, 65536)] * 2, tiny["comps"], tiny["s1"], tiny["s2"], 1, 1, lg.LAGOM_CORUN)
    with pytest.raises(lg.LagomError):
        lg.lagom_overlap_run(tiny["launches"], [(4, 256, 65536)], tiny["comps"], tiny["s1"], tiny["s2"], 1, 0, lg.LAGOM_CORUN)


def test_contention_sweep_on_the_tiny_grid(tiny):
    points = [(nc, 256, c) for nc in (2, 4) for c in (64 << 10, 128 << 10)]
    pts = lg.lagom_contention_sweep(tiny["launches"], 1, tiny["comps"], points, tiny["s1"], tiny["s2"], 1, 5)
    assert [p.cfg for p in pts] == points
    nbytes = lg.lagom_comm_bytes(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, 2, 1, 1 << 20)
    for p in pts:
        assert p.comm_alone_us > 0 and p.comm_corun_us > 0 and p.comp_alone_us > 0 and p.comp_corun_us > 0
        assert p.v_alone == pytest.approx(nbytes / p.comm_alone_us) and p.v_corun == pytest.approx(nbytes / p.comm_corun_us)
        assert p.z_corun_us >= max(p.comm_corun_us, p.comp_corun_us) * 0.999
    # four channels move the same bytes faster than two
    assert pts[2].comm_alone_us < pts[0].comm_alone_us


def test_measured_priority_search_stays_on_the_ladder_and_is_linear(tiny):
    space = lg.Space([1, 2, 4, 8, 16, 32], [256], [32768 << i for i in range(8)])
    prof = lg.OverlapProfile(tiny["launches"], tiny["comps"], tiny["s1"], tiny["s2"], 1, 3)
    r = lg.lagom_tune([space], prof, lg.LAGOM_PRIORITY)
    ladder = [(space.nc[min(l, 5)], 256, space.chunk[l]) for l in range(8)]
    assert r.cfgs[0] == ladder[r.levels[0]] and 1 <= r.calls <= 9 and len(r.trace) == r.calls
    assert r.Z > 0
    torch.cuda.synchronize()
    assert same_bits(host(tiny["dout"], np.float32), oc.reduce_copy([tiny["a"], tiny["b"]], oc.F32)[0])


def test_cross_stream_dependencies_are_honoured():
    """FSDP-like: the GEMM multiplies by the weight an all-gather is still writing, so it must wait for it;
    TP-like: a reduce-copy consumes the GEMM's output, so it must wait for the GEMM."""
    M = N = K = 512
    shards = [inputs.normal_bf16(300 + p, N * K // 8, scale=0.05) for p in range(8)]
    A = inputs.normal_bf16(2, (M, K))
    other = inputs.normal_bf16(7, M * N)
    d_sh = [dev(s) for s in shards]
    dW = dev(np.zeros(N * K, np.uint16))                       # zeros until the gather has run
    dA, dC = dev(A), dev(np.zeros(M * N, np.uint16))
    d_other, d_sum = dev(other), dev(np.zeros(M * N, np.uint16))
    s1, s2 = lg.overlapping_streams()
    launches = [lg.CommLaunch(lg.LAGOM_GATHER_COPY, lg.LAGOM_BF16, d_sh, [dW], N * K // 8, 0),
                lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_BF16, [dC, d_other], [d_sum], M * N, 1, after_comp=0)]
    comps = [lg.GemmDesc(dA, dW, dC, M, N, K, True, lg.LAGOM_BF16, after_comm_id=0)]
    cfgs = [(1, 64, 16384), (2, 256, 65536)]                   # one slow channel: the gather outlasts an unsynchronised GEMM
    t = lg.lagom_overlap_run(launches, cfgs, comps, s1, s2, 1, 3, lg.LAGOM_CORUN)
    torch.cuda.synchronize()
    W = oc.gather_copy(shards)[0].reshape(N, K)
    assert same_bits(host(dW, np.uint16), W.reshape(-1))
    ref = og.gemm_f64(A, W, True)
    got_bits = host(dC, np.uint16)
    e_max, e_fro = og.rel_errors(oc.bf16_to_f32(got_bits).reshape(M, N), ref)
    assert e_max <= 2e-2 and e_fro <= 2e-2, "the GEMM did not wait for its weights"
    want_sum = oc.reduce_copy([got_bits, other], oc.BF16)[0]   # exact on the bits the GEMM produced
    assert same_bits(host(d_sum, np.uint16), want_sum), "the reduce-copy did not wait for the GEMM"
    # the chain is serial: gather -> GEMM -> reduce, so the makespan holds all three
    assert t.Z_us >= 0.98 * (t.x_us[0] + t.y_us[0] + t.x_us[1])
    # the profiler and the measured ProfileTime report sums of the operators' own times (Eq. 1): the GEMM's wait for
    # the gather is in the computation stream's span (Y_us of the run) but not in Y of a sweep point or of a profile
    pt = lg.lagom_contention_sweep(launches, 2, comps, [cfgs[0]], s1, s2, 1, 3)[0]
    assert pt.comp_corun_us == pytest.approx(t.y_us[0], rel=0.5)
    big = [dev(inputs.normal_bf16(400 + p, 1 << 19)) for p in range(8)]          # 8 MiB through one 64-thread channel: ~1 ms
    d_big = dev(np.zeros(8 << 19, np.uint16))
    slow = [lg.CommLaunch(lg.LAGOM_GATHER_COPY, lg.LAGOM_BF16, big, [d_big], 1 << 19, 0)]
    two = [lg.GemmDesc(dA, dW, dC, M, N, K, True, lg.LAGOM_BF16), lg.GemmDesc(dA, dW, dC, M, N, K, True, lg.LAGOM_BF16, after_comm_id=0)]
    t2 = lg.lagom_overlap_run(slow, cfgs[:1], two, s1, s2, 1, 3, lg.LAGOM_CORUN)
    assert t2.Y_us > 5 * (t2.y_us[0] + t2.y_us[1])              # the span holds the second GEMM's wait for the slow gather
    pt2 = lg.lagom_contention_sweep(slow, 1, two, [cfgs[0]], s1, s2, 1, 3)[0]
    assert pt2.comp_corun_us < 0.5 * t2.Y_us and pt2.comp_corun_us == pytest.approx(t2.y_us[0] + t2.y_us[1], rel=0.5)
    # a cycle is refused and leaves nothing queued
    cyc_l = [lg.CommLaunch(lg.LAGOM_GATHER_COPY, lg.LAGOM_BF16, d_sh, [dW], N * K // 8, 0, after_comp=0)]
    with pytest.raises(lg.LagomError) as e:
        lg.lagom_overlap_run(cyc_l, cfgs[:1], comps, s1, s2, 0, 1, lg.LAGOM_CORUN)
    assert e.value.code == lg.LAGOM_EINVAL
    torch.cuda.synchronize()
    # alone modes ignore dependencies
    assert lg.lagom_overlap_run(cyc_l, cfgs[:1], comps, s1, s2, 0, 2, lg.LAGOM_ALONE_COMP).Y_us > 0


def test_full_size_corun_under_heavy_communication_keeps_both_results():
    """The benchmark's GEMM (4096^3) next to a 32-channel, 1024-thread eight-source reduce-copy that shares its
    compute units and its memory system: the GEMM's partial waits on its LDS-direct loads must still hold.
    GEMM: 64 seeded rows x all columns against the oracle; reduce-copy: bit-exact on sampled ranges."""
    M = N = K = 4096
    A, B = inputs.normal_bf16(2, (M, K)), inputs.normal_bf16(3, (N, K), 0.02)
    count = 4194304
    shards = [inputs.normal_bf16(20 + p, count) for p in range(8)]
    dA, dB, dC = dev(A), dev(B), dev(np.zeros(M * N, np.uint16))
    d_sh, d_out = [dev(x) for x in shards], dev(np.zeros(count, np.uint16))
    s1, s2 = lg.overlapping_streams()
    launches = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_BF16, d_sh, [d_out], count, 0)] * 6    # ~6 x 60 us beside ~100 us of GEMM
    comps = [lg.GemmDesc(dA, dB, dC, M, N, K)] * 2
    t = lg.lagom_overlap_run(launches, [(32, 1024, 64 << 10)], comps, s1, s2, 1, 3, lg.LAGOM_CORUN)
    torch.cuda.synchronize()
    assert t.X_us > 0.5 * t.Y_us, "the communication was too short to overlap the GEMMs"
    got = oc.bf16_to_f32(host(dC, np.uint16)).reshape(M, N)
    rows = np.unique(np.random.default_rng(7).integers(0, M, size=64))
    e_max, e_fro = og.rel_errors(got[rows], og.gemm_f64(A, B, True, rows=rows))
    assert e_max <= 2e-2 and e_fro <= 2e-2, (e_max, e_fro)
    out = host(d_out, np.uint16)
    for lo in (0, 1 << 20, count - 65536):
        want = oc.reduce_copy([x[lo:lo + 65536] for x in shards], oc.BF16)[0]
        assert same_bits(out[lo:lo + 65536], want)


def test_back_to_back_steps_keep_results_and_cost_about_one_makespan_each(tiny):
    cfg = [(4, 256, 128 << 10)]
    t = lg.lagom_overlap_run(tiny["launches"], cfg, tiny["comps"], tiny["s1"], tiny["s2"], 2, 10, lg.LAGOM_CORUN)
    per_step = lg.lagom_overlap_steps(tiny["launches"], cfg, tiny["comps"], tiny["s1"], tiny["s2"], 50)
    torch.cuda.synchronize()
    assert same_bits(host(tiny["dout"], np.float32), oc.reduce_copy([tiny["a"], tiny["b"]], oc.F32)[0])
    got = oc.bf16_to_f32(host(tiny["dC"], np.uint16))
    e_max, e_fro = og.rel_errors(got, og.gemm_f64(tiny["A"], tiny["B"], True))
    assert e_max <= 2e-2 and e_fro <= 2e-2
    # a repetition starts when the previous one has ended on both streams: no faster than the longer stream alone,
    # and not much slower than a gated makespan (joins and launch gaps only)
    assert per_step >= 0.9 * max(t.x_us[0], t.y_us[0]) and per_step <= 3.0 * t.Z_us
    with pytest.raises(lg.LagomError):
        lg.lagom_overlap_steps(tiny["launches"], cfg, tiny["comps"], tiny["s1"], tiny["s1"], 5)
    with pytest.raises(lg.LagomError):
        lg.lagom_overlap_steps(tiny["launches"], cfg, tiny["comps"], tiny["s1"], tiny["s2"], 0)


def test_graph_replay_runs_every_repetition_exactly_once(tiny):
    """An accumulating reduce-copy (destination = first source) counts the repetitions: after the call's one eager
    repetition and K replays of the captured graph the buffer holds (K + 1) * b exactly.  Several calls, with eager
    work and synchronisations between them, as a caller would mix them."""
    n = 1 << 18
    b = np.random.default_rng(3).integers(-8, 9, size=n).astype(np.float32)
    d_acc, d_b = dev(np.zeros(n, np.float32)), dev(b)
    launches = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [d_acc, d_b], [d_acc], n, 0)]
    cfg = [(4, 256, 64 << 10)]
    total = 0
    for K in (1, 3, 7):
        per_step = lg.lagom_overlap_steps_graph(launches, cfg, tiny["comps"], tiny["s1"], tiny["s2"], K)
        total += K + 1
        torch.cuda.synchronize()
        assert per_step > 0
        assert np.array_equal(host(d_acc, np.float32), total * b), (K, total)
        got = oc.bf16_to_f32(host(tiny["dC"], np.uint16))
        e_max, e_fro = og.rel_errors(got, og.gemm_f64(tiny["A"], tiny["B"], True))
        assert e_max <= 2e-2 and e_fro <= 2e-2
        # eager work between the graph calls
        lg.lagom_overlap_run(launches, cfg, tiny["comps"], tiny["s1"], tiny["s2"], 0, 2, lg.LAGOM_CORUN)
        total += 2
        torch.cuda.synchronize()
        assert np.array_equal(host(d_acc, np.float32), total * b)
    # the eager back-to-back path counts the same way
    lg.lagom_overlap_steps(launches, cfg, tiny["comps"], tiny["s1"], tiny["s2"], 5)
    torch.cuda.synchronize()
    assert np.array_equal(host(d_acc, np.float32), (total + 5) * b)
