"""GPU parity: lagom_comm_kernel through the C ABI against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import collective as oc
from paper_2602_20656_amd import binding as lg, inputs
from gpu_util import dev, host, same_bits

pytestmark = pytest.mark.gpu

GUARD = 64  # elements of padding on both sides of every destination


def _sources(dtype, nsrc, count, seed0):
    if dtype == "f32":
        return [inputs.uniform_f32(seed0 + s, count) for s in range(nsrc)]
    return [inputs.normal_bf16(seed0 + s, count) for s in range(nsrc)]


def _run(op, dtype, srcs, ndst, cfg, out_len):
    np_dt = np.float32 if dtype == "f32" else np.uint16
    d_srcs = [dev(s) for s in srcs]
    fill = np.full(out_len + 2 * GUARD, 0x7B if np_dt == np.uint16 else 123.0, dtype=np_dt)
    d_dsts = [dev(fill) for _ in range(ndst)]
    esz = np.dtype(np_dt).itemsize
    ptrs = [d.data_ptr() + GUARD * esz for d in d_dsts]
    lg.lagom_comm_kernel(op, lg.LAGOM_F32 if dtype == "f32" else lg.LAGOM_BF16, d_srcs, ptrs,
                         len(srcs[0]), cfg, torch.cuda.current_stream())
    torch.cuda.synchronize()
    outs = []
    for d in d_dsts:
        h = host(d, np_dt)
        assert same_bits(h[:GUARD], fill[:GUARD]) and same_bits(h[GUARD + out_len:], fill[GUARD + out_len:]), "guard region clobbered"
        outs.append(h[GUARD:GUARD + out_len])
    return outs


def test_tiny_config_and_its_grid():
    a, b = inputs.uniform_f32(0, 1 << 20), inputs.uniform_f32(1, 1 << 20)
    want = oc.reduce_copy([a, b], oc.F32)[0]
    for nc in (2, 4):
        for chunk in (64 << 10, 128 << 10):
            got = _run(lg.LAGOM_REDUCE_COPY, "f32", [a, b], 1, (nc, 256, chunk), 1 << 20)[0]
            assert same_bits(got, want), (nc, chunk)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nsrc,ndst", [(1, 1), (2, 1), (2, 2), (3, 1), (4, 4), (5, 1), (8, 1), (16, 2)])
def test_reduce_copy_ragged_lengths(dtype, nsrc, ndst):
    for count, cfg in [(1, (1, 64, 16)), (3, (4, 128, 4096)), (1000003, (7, 256, 65536)), (262144 + 5, (32, 1024, 32768)),
                       (70001, (3, 512, 1 << 20))]:
        srcs = _sources(dtype, nsrc, count, 100 + nsrc)
        want = oc.reduce_copy(srcs, dtype, ndst)
        got = _run(lg.LAGOM_REDUCE_COPY, dtype, srcs, ndst, cfg, count)
        for g, w in zip(got, want):
            assert same_bits(g, w), (dtype, nsrc, ndst, count, cfg)


def test_result_is_identical_for_every_swept_configuration():
    count = 1638400 // 4 + 24          # several chunks, ragged tail
    srcs = _sources("bf16", 2, count, 10)
    want = oc.reduce_copy(srcs, oc.BF16)[0]
    for nc in (1, 2, 4, 8, 16, 32, 256, 1000):
        for chunk in (32 << 10, 256 << 10, 4 << 20, 16, 4080):
            for nt in (64, 256, 1024):
                got = _run(lg.LAGOM_REDUCE_COPY, "bf16", srcs, 1, (nc, nt, chunk), count)[0]
                assert same_bits(got, want), (nc, nt, chunk)


def test_special_values_and_rounding_cases():
    one, eps = 0x3F80, 0x3B80
    patt = np.array([one, 0x7F80, 0xFF80, 0x7FC0, 0x0001, 0x8000, 0x7F7F, 0x3F81], dtype=np.uint16)
    a = np.tile(patt, 9)
    b = np.tile(np.array([eps, 0x7F80, 0x7F80, one, 0x0001, 0x0000, 0x7F7F, eps], dtype=np.uint16), 9)
    c = np.tile(np.array([eps, one, one, one, 0x8001, 0x8000, 0x0000, 0x0000], dtype=np.uint16), 9)
    want = oc.reduce_copy([a, b, c], oc.BF16)[0]
    got = _run(lg.LAGOM_REDUCE_COPY, "bf16", [a, b, c], 1, (2, 64, 64), len(a))[0]
    assert same_bits(got, want)
    assert got[0] == 0x3F81                                   # 1 + 2^-8 + 2^-8 rounds once
    big, o = np.float32(1e8), np.float32(1.0)
    f = [np.array([big, o, np.inf, np.nan], np.float32), np.array([-big, big, -np.inf, o], np.float32),
         np.array([o, -big, o, o], np.float32)]
    gotf = _run(lg.LAGOM_REDUCE_COPY, "f32", f, 1, (1, 64, 16), 4)[0]
    assert gotf[:2].tolist() == [1.0, 0.0] and np.isnan(gotf[2]) and np.isnan(gotf[3])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_copy(dtype):
    for P, count, cfg in [(8, 2097152 // 8, (8, 256, 2 << 20)), (8, 1237, (4, 256, 1024)), (3, 70001, (5, 128, 65536)),
                          (1, 1000003, (6, 256, 32768)), (2, 8, (1, 64, 16)), (16, 4099, (32, 512, 4096))]:
        shards = _sources(dtype, P, count, 30)
        want = np.concatenate(shards)
        for ndst in (1, 2):
            for g in _run(lg.LAGOM_GATHER_COPY, dtype, shards, ndst, cfg, P * count):
                assert same_bits(g, want), (dtype, P, count, cfg)


def test_empty_input_is_a_no_op():
    a = dev(np.zeros(16, np.float32)); d = dev(np.ones(16, np.float32))
    lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [a], [d], 0, (4, 256, 65536), torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert d.cpu().numpy().tolist() == [1.0] * 16


@pytest.mark.parametrize("dtype,P,m", [("bf16", 8, 1638400 // 64), ("f32", 4, 1000)])
def test_ring_all_reduce_emulated_on_one_gpu(dtype, P, m):
    """Every rank's 2(P-1) local steps run through the kernel; peers are separate allocations."""
    if dtype == "bf16":
        buckets = [inputs.normal_bf16(10 + r, P * m, scale=0.125) for r in range(P)]
    else:
        buckets = [inputs.uniform_f32(40 + r, P * m) for r in range(P)]
    want = oc.ring_all_reduce(buckets, dtype)
    dt = lg.LAGOM_BF16 if dtype == "bf16" else lg.LAGOM_F32
    esz = 2 if dtype == "bf16" else 4
    local = [dev(b) for b in buckets]
    # wire[r] = what rank r sends next (the receive buffer of rank r+1), double-buffered
    wire = [[torch.empty_like(local[0][:m]) for _ in range(P)] for _ in range(2)]
    st = torch.cuda.current_stream()
    cfg = (4, 256, 32768)
    chunk_ptr = lambda r, c: local[r].data_ptr() + c * m * esz
    for r in range(P):  # step 0 sends the rank's own chunk r
        lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, dt, [chunk_ptr(r, r)], [wire[0][r]], m, cfg, st)
    cur = 0
    for s in range(P - 1):
        for r in range(P):
            c = (r - s - 1) % P
            dsts = [wire[1 - cur][r]] + ([chunk_ptr(r, c)] if s == P - 2 else [])
            lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, dt, [wire[cur][(r - 1) % P], chunk_ptr(r, c)], dsts, m, cfg, st)
        cur = 1 - cur
    for s in range(P - 1):
        for r in range(P):
            c = (r - s) % P
            dsts = [chunk_ptr(r, c)] + ([wire[1 - cur][r]] if s < P - 2 else [])
            lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, dt, [wire[cur][(r - 1) % P]], dsts, m, cfg, st)
        cur = 1 - cur
    torch.cuda.synchronize()
    for r in range(P):
        assert same_bits(host(local[r], buckets[0].dtype), want[r]), r


def test_tp_reduce_scatter_share_full_size_sampled():
    """Full-size TP share (8 x 4,194,304 bf16) in the benchmark's launch shape; the oracle checks slices."""
    count = 4194304
    srcs = [inputs.normal_bf16(20 + s, count) for s in range(8)]
    got = _run(lg.LAGOM_REDUCE_COPY, "bf16", srcs, 1, (32, 256, 2 << 20), count)[0]
    rng = np.random.default_rng(0)
    for lo in [0, count - 4096] + [int(v) for v in rng.integers(0, count - 4096, size=14)]:
        want = oc.reduce_copy([s[lo:lo + 4096] for s in srcs], oc.BF16)[0]
        assert same_bits(got[lo:lo + 4096], want), lo


def test_full_size_workload_launches_sampled():
    """The other benchmark launches at full size and in their benchmark launch shapes; the oracle checks slices."""
    rng = np.random.default_rng(1)
    # DP bucket ring step: 1,638,400 bf16, two sources, two destinations (last reduce step)
    m = 1638400
    srcs = [inputs.normal_bf16(10 + s, m, scale=0.125) for s in range(2)]
    outs = _run(lg.LAGOM_REDUCE_COPY, "bf16", srcs, 2, (32, 256, 128 << 10), m)
    want = oc.reduce_copy(srcs, oc.BF16)[0]            # 1.6M elements: the oracle does all of them
    assert same_bits(outs[0], want) and same_bits(outs[1], want)
    # compute-bound: 4,194,304 fp32, two sources
    n = 4194304
    f = [inputs.uniform_f32(40 + s, n) for s in range(2)]
    got = _run(lg.LAGOM_REDUCE_COPY, "f32", f, 1, (8, 256, 2 << 20), n)[0]
    assert same_bits(got, oc.reduce_copy(f, oc.F32)[0])
    # FSDP all-gather: 8 shards of 2,097,152 bf16 into one 32 MiB weight buffer
    shards = [inputs.normal_bf16(3000 + p, 2097152, scale=0.02) for p in range(8)]
    full = _run(lg.LAGOM_GATHER_COPY, "bf16", shards, 1, (8, 256, 2 << 20), 8 * 2097152)[0]
    assert same_bits(full, oc.gather_copy(shards)[0])
    # extended channel counts used for the standalone bandwidth figure
    for cfg in [(512, 512, 16 << 10), (256, 1024, 32 << 10), (1024, 512, 64 << 10)]:
        got = _run(lg.LAGOM_REDUCE_COPY, "f32", f, 1, cfg, n)[0]
        assert same_bits(got, oc.reduce_copy(f, oc.F32)[0]), cfg


@pytest.mark.parametrize("dtype,P,m", [("bf16", 8, 4096 * 24), ("f32", 4, 1004)])
def test_all_to_all_emulated_on_one_gpu(dtype, P, m):
    """Expert-parallel exchange: rank r's local step is a gather-copy whose source s starts at block r of peer s."""
    send = _sources(dtype, P, P * m, 500)
    want = oc.all_to_all(send)
    dt = lg.LAGOM_BF16 if dtype == "bf16" else lg.LAGOM_F32
    esz = 2 if dtype == "bf16" else 4
    d_send = [dev(b) for b in send]
    d_recv = [torch.zeros_like(d_send[0]) for _ in range(P)]
    st = torch.cuda.current_stream()
    for r in range(P):
        srcs = [d_send[s].data_ptr() + r * m * esz for s in range(P)]
        lg.lagom_comm_kernel(lg.LAGOM_GATHER_COPY, dt, srcs, [d_recv[r]], m, (4, 256, 32768), st)
    torch.cuda.synchronize()
    for r in range(P):
        assert same_bits(host(d_recv[r], send[0].dtype), want[r]), r


def test_limits_of_the_argument_ranges():
    """Most sources and destinations the ABI allows, the largest channel count, the smallest chunk and block."""
    count = 40000 + 3
    for dtype in ("f32", "bf16"):
        srcs = _sources(dtype, 16, count, 700)
        want = oc.reduce_copy(srcs, dtype, 4)
        for cfg in [(65535, 64, 16), (1, 1024, 4 << 20), (300, 192, 48)]:
            got = _run(lg.LAGOM_REDUCE_COPY, dtype, srcs, 4, cfg, count)
            for g, w in zip(got, want):
                assert same_bits(g, w), (dtype, cfg)
        shards = _sources(dtype, 16, 1001, 800)
        for g in _run(lg.LAGOM_GATHER_COPY, dtype, shards, 4, (65535, 64, 16), 16 * 1001):
            assert same_bits(g, np.concatenate(shards))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("which", [0, 2])
def test_reduce_copy_onto_one_of_its_sources(dtype, which):
    """In-place accumulation: the destination is exactly source `which`; a second destination gets the same values.
    Ragged length (a tail shorter than 16 bytes) and a configuration with several chunks per channel."""
    count = 3 * 65536 + 5
    srcs = _sources(dtype, 3, count, 900)
    want = oc.reduce_copy(srcs, oc.F32 if dtype == "f32" else oc.BF16)[0]
    d = [dev(s) for s in srcs]
    np_dt = np.float32 if dtype == "f32" else np.uint16
    other = dev(np.zeros(count, np_dt))
    lg.lagom_comm_kernel(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32 if dtype == "f32" else lg.LAGOM_BF16, d, [d[which], other],
                         count, (3, 128, 16384), torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert same_bits(host(d[which], np_dt), want) and same_bits(host(other, np_dt), want)
    for s in range(3):
        if s != which:
            assert same_bits(host(d[s], np_dt), srcs[s]), "a source that is not the destination changed"


# ------------------------------------------------------------- several steps in one launch
def _steps_case(dtype, count, cfg, names_steps, bufs):
    """Runs `names_steps` over named buffers through lagom_comm_steps and returns the final contents."""
    np_dt = np.float32 if dtype == "f32" else np.uint16
    d = {k: dev(np.concatenate([np.full(GUARD, 7, np_dt), v, np.full(GUARD, 7, np_dt)])) for k, v in bufs.items()}
    esz = np.dtype(np_dt).itemsize
    ptr = {k: t.data_ptr() + GUARD * esz for k, t in d.items()}
    steps = [(lg.LAGOM_REDUCE_COPY if op == "reduce_copy" else lg.LAGOM_GATHER_COPY, [ptr[s] for s in srcs], [ptr[x] for x in dsts])
             for op, srcs, dsts in names_steps]
    lg.lagom_comm_steps(lg.LAGOM_F32 if dtype == "f32" else lg.LAGOM_BF16, steps, count, cfg, torch.cuda.current_stream())
    torch.cuda.synchronize()
    out = {}
    for k, t in d.items():
        h = host(t, np_dt)
        assert (h[:GUARD] == 7).all() and (h[GUARD + count:] == 7).all(), f"guard region of {k} clobbered"
        out[k] = h[GUARD:GUARD + count]
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_steps_in_one_launch_equal_the_oracle_sequence(dtype):
    gen = (lambda s, n: inputs.uniform_f32(s, n)) if dtype == "f32" else (lambda s, n: inputs.normal_bf16(s, n))
    for count, cfg in [(5, (1, 64, 16)), (1000003, (7, 256, 65536)), (262144 + 5, (32, 1024, 32768)), (70001, (300, 512, 4096)),
                       (1 << 20, (128, 256, 32768))]:
        bufs = {k: gen(300 + i, count) for i, k in enumerate("abcdefg")}
        # an accumulation chain through one buffer (every step reads what the previous one wrote), a fan-out copy,
        # a three-source and a five-source reduce (the general path), an overwrite of an earlier result
        steps = [("reduce_copy", ["a", "b"], ["b"]), ("reduce_copy", ["b", "c"], ["b", "d"]), ("gather_copy", ["b"], ["e", "f"]),
                 ("reduce_copy", ["e", "a", "c"], ["g"]), ("reduce_copy", ["g", "b"], ["b"]), ("reduce_copy", ["a", "b", "c", "d", "e"], ["f"]),
                 ("reduce_copy", ["a"], ["c"]), ("gather_copy", ["f"], ["a"])]
        want = oc.comm_steps(bufs, steps, dtype)
        got = _steps_case(dtype, count, cfg, steps, bufs)
        for k in bufs:
            assert same_bits(got[k], want[k]), (dtype, count, cfg, k)


def test_ring_share_as_one_launch_equals_the_separate_launches_and_the_oracle():
    """The DP bucket's share of the ring (7 reduce steps, 7 store-and-forward steps over two wire buffers each way) as
    one lagom_comm_steps launch: the same bits as fourteen lagom_comm_kernel launches and as the oracle's sequence."""
    P, m = 8, 1638400
    local = inputs.normal_bf16(10, P * m, 0.125)
    bufs = {f"c{c}": local[c * m:(c + 1) * m] for c in range(P)}
    bufs.update({"in0": inputs.normal_bf16(11, m, 0.125), "in1": inputs.normal_bf16(12, m, 0.125),
                 "out0": np.zeros(m, np.uint16), "out1": np.zeros(m, np.uint16)})
    steps = []
    for s in range(P - 1):
        c = (0 - s - 1) % P
        steps.append(("reduce_copy", [f"in{s % 2}", f"c{c}"], [f"out{s % 2}"] + ([f"c{c}"] if s == P - 2 else [])))
    for s in range(P - 1):
        c = (0 - s) % P
        steps.append(("gather_copy", [f"in{s % 2}"], [f"c{c}"] + ([f"out{s % 2}"] if s < P - 2 else [])))
    want = oc.comm_steps(bufs, steps, "bf16")
    for cfg in [(32, 256, 65536), (256, 512, 32768), (3, 1024, 1 << 20)]:
        got = _steps_case("bf16", m, cfg, steps, bufs)
        for k in bufs:
            assert same_bits(got[k], want[k]), (cfg, k)


def test_steps_launch_rejects_what_it_cannot_order():
    t = dev(np.zeros(4096, np.float32))
    p = t.data_ptr()
    good = (4, 256, 4096)
    with pytest.raises(lg.LagomError) as e:       # a two-source gather-copy is not a step
        lg.lagom_comm_steps(lg.LAGOM_F32, [(lg.LAGOM_GATHER_COPY, [p, p + 4096], [p + 8192])], 1024, good)
    assert e.value.code == lg.LAGOM_EINVAL
    with pytest.raises(lg.LagomError) as e:       # step 1 writes memory that step 0 reads, shifted by 64 bytes
        lg.lagom_comm_steps(lg.LAGOM_F32, [(lg.LAGOM_REDUCE_COPY, [p], [p + 8192]), (lg.LAGOM_REDUCE_COPY, [p + 8192], [p + 64])], 1024, good)
    assert e.value.code == lg.LAGOM_EINVAL and "overlap in part" in str(e.value)
    with pytest.raises(lg.LagomError):
        lg.lagom_comm_steps(lg.LAGOM_F32, [], 1024, good)
    with pytest.raises(lg.LagomError):
        lg.lagom_comm_steps(lg.LAGOM_F32, [(lg.LAGOM_REDUCE_COPY, [p], [p + 8192])] * 33, 1024, good)
    lg.lagom_comm_steps(lg.LAGOM_F32, [(lg.LAGOM_REDUCE_COPY, [p], [p + 8192])], 0, good)      # count 0: nothing is launched


# ------------------------------------------------------------------ staged through LDS
def _run_lds(op, dtype, srcs, ndst, cfg, out_len):
    np_dt = np.float32 if dtype == "f32" else np.uint16
    d_srcs = [dev(s) for s in srcs]
    fill = np.full(out_len + 2 * GUARD, 0x7B if np_dt == np.uint16 else 123.0, dtype=np_dt)
    d_dsts = [dev(fill) for _ in range(ndst)]
    esz = np.dtype(np_dt).itemsize
    lg.lagom_comm_kernel_lds(op, lg.LAGOM_F32 if dtype == "f32" else lg.LAGOM_BF16, d_srcs, [d.data_ptr() + GUARD * esz for d in d_dsts],
                             len(srcs[0]), cfg, torch.cuda.current_stream())
    torch.cuda.synchronize()
    outs = []
    for d in d_dsts:
        h = host(d, np_dt)
        assert same_bits(h[:GUARD], fill[:GUARD]) and same_bits(h[GUARD + out_len:], fill[GUARD + out_len:]), "guard region clobbered"
        outs.append(h[GUARD:GUARD + out_len])
    return outs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nsrc,ndst", [(1, 1), (2, 1), (2, 2), (3, 1), (5, 4), (8, 1), (16, 2)])
def test_lds_staged_reduce_copy_equals_oracle(dtype, nsrc, ndst):
    """Whole batches through LDS, the rest of every chunk through the register path, a short tail at the end; one to
    sixteen wavefronts; chunks smaller than, equal to and larger than a workgroup's batch round."""
    for count, cfg in [(1, (1, 64, 16)), (3, (4, 128, 4096)), (1000003, (7, 256, 65536)), (262144 + 5, (32, 1024, 32768)),
                       (70001, (3, 512, 1 << 20)), (1 << 20, (256, 512, 16384)), (123457, (5, 64, 2048)), (40000, (2, 192, 6000 * 16))]:
        srcs = _sources(dtype, nsrc, count, 400 + nsrc)
        want = oc.reduce_copy(srcs, dtype, ndst)
        got = _run_lds(lg.LAGOM_REDUCE_COPY, dtype, srcs, ndst, cfg, count)
        for g, w in zip(got, want):
            assert same_bits(g, w), (dtype, nsrc, ndst, count, cfg)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lds_staged_gather_copy_equals_oracle(dtype):
    for nsrc, ndst, count, cfg in [(8, 1, 2097152, (32, 256, 1 << 20)), (8, 2, 100000, (5, 512, 32768)), (3, 1, 70008, (256, 1024, 16384)),
                                   (1, 3, 1000003, (9, 128, 65536)), (4, 1, 1001, (2, 64, 4096))]:     # the last: shards not 16-byte multiples
        srcs = _sources(dtype, nsrc, count, 500 + nsrc)
        want = oc.gather_copy(srcs, ndst)
        got = _run_lds(lg.LAGOM_GATHER_COPY, dtype, srcs, ndst, cfg, nsrc * count)
        for g, w in zip(got, want):
            assert same_bits(g, w), (dtype, nsrc, ndst, count, cfg)


def test_lds_staged_in_place_and_through_the_runner():
    n = 1 << 20
    a, b = inputs.uniform_f32(0, n), inputs.uniform_f32(1, n)
    da, db = dev(a), dev(b)
    lg.lagom_comm_kernel_lds(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [da, db], [db], n, (16, 512, 65536), torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert same_bits(host(db, np.float32), oc.reduce_copy([a, b], oc.F32)[0])          # b <- a + b, in place
    s1, s2 = lg.overlapping_streams()
    out = dev(np.zeros(n, np.float32))
    db2 = dev(b)
    A, B = inputs.normal_bf16(2, (512, 512)), inputs.normal_bf16(3, (512, 512))
    comps = [lg.GemmDesc(dev(A), dev(B), dev(np.zeros((512, 512), np.uint16)), 512, 512, 512)]
    launches = [lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [da, db2], [out], n, 0, lds_staged=True)]
    t = lg.lagom_overlap_run(launches, [(4, 256, 128 << 10)], comps, s1, s2, 1, 3, lg.LAGOM_CORUN)
    torch.cuda.synchronize()
    assert t.X_us > 0 and same_bits(host(out, np.float32), oc.reduce_copy([a, b], oc.F32)[0])
    bad = [launches[0], lg.CommLaunch(lg.LAGOM_REDUCE_COPY, lg.LAGOM_F32, [da, db2], [out], n, 0, fuse=True, lds_staged=True)]
    with pytest.raises(lg.LagomError):
        lg.lagom_overlap_run(bad, [(4, 256, 128 << 10)], comps, s1, s2, 0, 1, lg.LAGOM_ALONE_COMM)


def test_full_size_launches_in_the_light_channel_and_roofline_shapes():
    """The launch shapes the extended searches, the penalised model and the standalone bandwidth figure end at, at full
    size, register path and LDS path: the 72 MiB eight-source reduce and the 64 MiB all-gather copy.  The oracle
    computes sampled slices of the reduce and the whole gather."""
    count = 4194304
    srcs = [inputs.normal_bf16(20 + s, count) for s in range(8)]
    rng = np.random.default_rng(7)
    lows = [0, count - 4096] + [int(v) for v in rng.integers(0, count - 4096, size=10)]
    wants = {lo: oc.reduce_copy([s[lo:lo + 4096] for s in srcs], oc.BF16)[0] for lo in lows}
    for run, cfgs in ((_run, [(128, 128, 64 << 10), (256, 128, 32 << 10), (64, 128, 128 << 10), (512, 512, 16 << 10)]),
                      (_run_lds, [(512, 512, 16 << 10), (128, 128, 64 << 10)])):
        for cfg in cfgs:
            got = run(lg.LAGOM_REDUCE_COPY, "bf16", srcs, 1, cfg, count)[0]
            for lo, want in wants.items():
                assert same_bits(got[lo:lo + 4096], want), (run.__name__, cfg, lo)
    shards = [inputs.normal_bf16(3000 + p, 2097152, scale=0.02) for p in range(8)]
    whole = oc.gather_copy(shards)[0]
    for run, cfgs in ((_run, [(128, 128, 64 << 10), (256, 128, 32 << 10), (512, 512, 16 << 10)]), (_run_lds, [(512, 512, 16 << 10)])):
        for cfg in cfgs:
            assert same_bits(run(lg.LAGOM_GATHER_COPY, "bf16", shards, 1, cfg, 8 * 2097152)[0], whole), (run.__name__, cfg)
