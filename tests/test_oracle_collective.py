"""Pins for oracle/collective.py and oracle/loops.c: every check here compares the oracle
with something other than itself (a library routine, exact integer arithmetic, a
hand-built case whose answer is known, or an invariant of the collective)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import cloops, collective as oc
from paper_2602_20656_amd import inputs


# ------------------------------------------------------------------------ bf16
def _all_f32_patterns():
    upper = np.arange(1 << 16, dtype=np.uint32)
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    return ((upper[:, None] << 16) | lows[None, :]).reshape(-1)


def test_bf16_widen_matches_torch():
    bits = np.arange(1 << 16, dtype=np.uint16)
    ours = oc.bf16_to_f32(bits)
    ref = inputs.bits_to_torch_bf16(bits).to(torch.float32).numpy()
    assert np.array_equal(ours.view(np.uint32), ref.view(np.uint32))


def test_bf16_round_matches_torch_on_every_upper_half():
    u = _all_f32_patterns()
    f = u.view(np.float32)
    finite_or_inf = ~np.isnan(f)
    ours = oc.f32_to_bf16(f)
    ref = inputs.to_bf16_bits(f)
    assert np.array_equal(ours[finite_or_inf], ref[finite_or_inf])
    # NaN stays NaN
    assert np.all(np.isnan(oc.bf16_to_f32(ours[~finite_or_inf])))


def test_bf16_round_is_nearest_even_by_exact_rationals():
    rng = np.random.default_rng(7)
    u = rng.integers(0, 1 << 32, size=400, dtype=np.uint64).astype(np.uint32)
    u = np.concatenate([u, np.array([0x3F808000, 0x3F818000, 0x3F800001, 0x3F80FFFF, 0x00008000, 0x80018000],
                                    dtype=np.uint32)])
    f = u.view(np.float32)
    keep = np.isfinite(f)
    for val, got in zip(f[keep], oc.f32_to_bf16(f[keep])):
        lo_bits = int(np.float32(val).view(np.uint32)) & 0xFFFF0000  # truncation toward zero
        lo = np.uint32(lo_bits).view(np.float32)
        hi = np.uint32(lo_bits + 0x10000).view(np.float32)           # next bf16 away from zero
        exact = Fraction(float(val))
        cands = [(abs(exact - Fraction(float(lo))), (lo_bits >> 16) & 1, lo_bits >> 16)]
        if np.isfinite(hi):
            cands.append((abs(exact - Fraction(float(hi))), ((lo_bits >> 16) + 1) & 1, (lo_bits >> 16) + 1))
        else:  # rounding up from the largest finite bf16 overflows to infinity when at/above the midpoint
            mid = Fraction(float(lo)) + (Fraction(float(lo)) - Fraction(float(np.uint32(lo_bits - 0x10000).view(np.float32)))) / 2
            cands.append((abs(exact - mid) if abs(exact) < abs(mid) else Fraction(0), ((lo_bits >> 16) + 1) & 1, (lo_bits >> 16) + 1))
        best = min(cands, key=lambda c: (c[0], c[1]))  # nearest, then even
        assert int(got) == best[2], hex(int(np.float32(val).view(np.uint32)))


# ------------------------------------------------------------------ reduce-copy
def test_two_source_f32_equals_numpy_add_and_commutes():
    a = inputs.uniform_f32(0, 100003)
    b = inputs.uniform_f32(1, 100003)
    out = oc.reduce_copy([a, b], oc.F32)[0]
    assert np.array_equal(out.view(np.uint32), (a + b).view(np.uint32))
    assert np.array_equal(out.view(np.uint32), oc.reduce_copy([b, a], oc.F32)[0].view(np.uint32))


def test_source_order_is_left_to_right():
    big = np.float32(1e8)
    one = np.float32(1.0)
    a = np.array([big, one], dtype=np.float32)
    b = np.array([-big, big], dtype=np.float32)
    c = np.array([one, -big], dtype=np.float32)
    out = oc.reduce_copy([a, b, c], oc.F32)[0]
    # (1e8 - 1e8) + 1 = 1 ; (1 + 1e8) - 1e8 = 0 in fp32 (1 is below half an ulp of 1e8)
    assert out.tolist() == [1.0, 0.0]


def test_bf16_rounds_once_at_the_end():
    one, eps = 0x3F80, 0x3B80  # 1.0 and 2^-8 = half a bf16 ulp at 1.0
    srcs = [np.array([v], dtype=np.uint16) for v in (one, eps, eps)]
    # exact sum 1 + 2^-7 is a bf16 value; rounding after each add would give 1.0 twice (ties to even)
    assert oc.reduce_copy(srcs, oc.BF16)[0].tolist() == [0x3F81]
    # and a tie after a single fp32 add goes to even
    assert oc.reduce_copy(srcs[:2], oc.BF16)[0].tolist() == [0x3F80]
    assert oc.reduce_copy([np.array([0x3F81], np.uint16), srcs[1]], oc.BF16)[0].tolist() == [0x3F82]


@pytest.mark.parametrize("dtype", [oc.F32, oc.BF16])
@pytest.mark.parametrize("nsrc", [1, 2, 3, 8])
def test_integer_valued_sources_sum_exactly(dtype, nsrc):
    rng = np.random.default_rng(nsrc)
    ints = [rng.integers(-15, 16, size=5000) for _ in range(nsrc)]  # |sum| <= 120: exact in bf16 and fp32
    if dtype == oc.F32:
        srcs = [v.astype(np.float32) for v in ints]
        outs = oc.reduce_copy(srcs, dtype, ndst=2)
        got = outs[0]
    else:
        srcs = [inputs.to_bf16_bits(v.astype(np.float32)) for v in ints]
        outs = oc.reduce_copy(srcs, dtype, ndst=2)
        got = oc.bf16_to_f32(outs[0])
    assert np.array_equal(got.astype(np.int64), sum(ints))
    assert np.array_equal(outs[0], outs[1]) and outs[0] is not outs[1]


def test_result_does_not_depend_on_channels_or_chunk():
    n = 70001
    srcs = [inputs.normal_bf16(s, n) for s in (20, 21, 22)]
    ref = oc.reduce_copy(srcs, oc.BF16)[0]
    for nc, chunk in [(1, 64), (3, 4096), (4, 1 << 20), (32, 32), (7, 1000)]:
        assert np.array_equal(oc.reduce_copy_chunked(srcs, oc.BF16, nc, chunk), ref)


def test_chunk_schedule_partitions_every_shard():
    nbytes, nshards, nc, chunk = 10_000, 3, 4, 4096
    plan = oc.chunk_schedule(nbytes, nshards, nc, chunk)
    assert len(plan) == nc
    seen = np.zeros((nshards, nbytes), dtype=np.int32)
    order = []
    for k, channel in enumerate(plan):
        for (r, off, length) in channel:
            assert 0 < length <= chunk and off % chunk == 0 and off + length <= nbytes  # never straddles a shard
            seen[r, off:off + length] += 1
            order.append((r * 3 + off // chunk, k))
    assert np.all(seen == 1)
    assert all(k == g % nc for g, k in order)               # chunk g -> channel g mod NC
    assert sorted(g for g, _ in order) == list(range(9))    # 3 chunks per shard (4096, 4096, 1808)


# ------------------------------------------------------------------ gather-copy
def test_gather_copy_is_concatenation():
    shards = [inputs.normal_bf16(30 + r, 1237) for r in range(8)]
    outs = oc.gather_copy(shards, ndst=2)
    assert np.array_equal(outs[0], np.concatenate(shards)) and np.array_equal(outs[1], outs[0])
    for full in oc.all_gather(shards):
        assert np.array_equal(full, np.concatenate(shards))


# ------------------------------------------------------------------ collectives
@pytest.mark.parametrize("dtype", [oc.F32, oc.BF16])
def test_reduce_scatter_shards_concatenate_to_the_full_reduce(dtype):
    P, n = 8, 8 * 515
    if dtype == oc.F32:
        contribs = [inputs.uniform_f32(40 + p, n) for p in range(P)]
    else:
        contribs = [inputs.normal_bf16(20 + p, n) for p in range(P)]
    shards = oc.reduce_scatter_direct(contribs, dtype)
    assert np.array_equal(np.concatenate(shards), oc.reduce_copy(contribs, dtype)[0])


@pytest.mark.parametrize("P", [2, 3, 8])
def test_ring_all_reduce_exact_on_integers_and_identical_on_every_rank(P):
    rng = np.random.default_rng(P)
    ints = [rng.integers(-7, 8, size=P * 33) for _ in range(P)]
    for dtype in (oc.F32, oc.BF16):
        if dtype == oc.F32:
            buckets = [v.astype(np.float32) for v in ints]
        else:
            buckets = [inputs.to_bf16_bits(v.astype(np.float32)) for v in ints]
        outs = oc.ring_all_reduce(buckets, dtype)
        vals = [o if dtype == oc.F32 else oc.bf16_to_f32(o) for o in outs]
        for v in vals:
            assert np.array_equal(v.astype(np.int64), sum(ints))
        for o in outs[1:]:
            assert np.array_equal(o, outs[0])


def test_ring_all_reduce_summation_order_and_per_step_rounding():
    """Chunk c is accumulated around the ring starting at rank c, re-rounded to bf16 at each hop."""
    P, m = 4, 257
    buckets = [inputs.normal_bf16(10 + p, P * m, scale=0.125) for p in range(P)]
    outs = oc.ring_all_reduce(buckets, oc.BF16)
    for c in range(P):
        acc = torch.from_numpy(oc.bf16_to_f32(buckets[c][c * m:(c + 1) * m]).copy())
        for hop in range(1, P):
            nxt = torch.from_numpy(oc.bf16_to_f32(buckets[(c + hop) % P][c * m:(c + 1) * m]).copy())
            acc = (acc + nxt).to(torch.bfloat16).to(torch.float32)   # torch's own rounding
        want = inputs.to_bf16_bits(acc.numpy())
        for r in range(P):
            assert np.array_equal(outs[r][c * m:(c + 1) * m], want)


def test_all_reduce_equals_reduce_scatter_then_all_gather_in_f32_for_two_ranks():
    # with two ranks every chunk is one commutative fp32 add, so the ring and the direct form agree bit for bit
    a, b = inputs.uniform_f32(0, 2000), inputs.uniform_f32(1, 2000)
    ring = oc.ring_all_reduce([a, b], oc.F32)
    direct = np.concatenate(oc.reduce_scatter_direct([a, b], oc.F32))
    assert np.array_equal(ring[0], direct) and np.array_equal(ring[1], direct)


# ------------------------------------------------------------------ the C loops
@pytest.mark.parametrize("threads", [1, 4])
def test_c_loops_match_numpy_oracle(threads):
    n = 40013
    f = [inputs.uniform_f32(s, n) for s in (0, 1, 2)]
    h = [inputs.normal_bf16(s, n) for s in (20, 21, 22, 23)]
    for a, b in zip(cloops.reduce_copy(f, "f32", 2, threads), oc.reduce_copy(f, oc.F32, 2)):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    for a, b in zip(cloops.reduce_copy(h, "bf16", 1, threads), oc.reduce_copy(h, oc.BF16, 1)):
        assert np.array_equal(a, b)
    assert np.array_equal(cloops.gather_copy(h, 1, threads)[0], np.concatenate(h))
    # the order-sensitive and single-rounding cases again, through the C code
    big, one = np.float32(1e8), np.float32(1.0)
    out = cloops.reduce_copy([np.array([big, one], np.float32), np.array([-big, big], np.float32),
                              np.array([one, -big], np.float32)], "f32")[0]
    assert out.tolist() == [1.0, 0.0]
    srcs = [np.array([v], dtype=np.uint16) for v in (0x3F80, 0x3B80, 0x3B80)]
    assert cloops.reduce_copy(srcs, "bf16")[0].tolist() == [0x3F81]


def test_all_to_all_is_a_block_transpose_and_an_involution():
    P, m = 4, 37
    send = [np.arange(r * 1000, r * 1000 + P * m, dtype=np.float32) for r in range(P)]
    recv = oc.all_to_all(send)
    grid = np.stack([b.reshape(P, m) for b in send])              # [sender, block, i]
    want = grid.transpose(1, 0, 2)                                # [receiver, sender, i]
    for r in range(P):
        assert np.array_equal(recv[r], want[r].reshape(-1))
        assert recv[r][2 * m + 5] == send[2][r * m + 5]           # element 5 of what rank 2 sent to rank r
    back = oc.all_to_all(recv)                                    # exchanging twice returns every buffer
    for r in range(P):
        assert np.array_equal(back[r], send[r])
    # per rank it is a gather-copy whose sources start at that rank's block of every peer
    for r in range(P):
        assert np.array_equal(oc.gather_copy([b[r * m:(r + 1) * m] for b in send])[0], recv[r])


def test_comm_steps_is_the_sequence_of_its_steps():
    """Pins: a chain b <- a + b applied k times to integer data is b + k*a exactly; the emulated ring share written as a
    list of steps gives the all-reduce of oracle.ring_all_reduce on the owning rank's buffers; inputs are not modified."""
    rng = np.random.default_rng(1)
    a = rng.integers(-50, 50, size=1000).astype(np.float32)
    b = rng.integers(-50, 50, size=1000).astype(np.float32)
    out = oc.comm_steps({"a": a, "b": b}, [("reduce_copy", ["a", "b"], ["b"])] * 5, oc.F32)
    assert np.array_equal(out["b"], b + 5 * a) and np.array_equal(out["a"], a) and np.array_equal(b, rng.integers(0, 1, 1000) * 0 + b)
    # store-and-forward is a copy of bits, NaN payloads included
    weird = np.array([0x7FC1, 0x7F81, 0xFFFF, 0x0001, 0x8000], dtype=np.uint16)
    out = oc.comm_steps({"w": weird, "x": np.zeros(5, np.uint16), "y": np.zeros(5, np.uint16)}, [("gather_copy", ["w"], ["x", "y"])], oc.BF16)
    assert np.array_equal(out["x"], weird) and np.array_equal(out["y"], weird)
    # fp32 summation order is the steps' order: ((1e8 + -1e8) + 1) = 1, but a different order would give 0
    big = {"p": np.array([1e8], np.float32), "q": np.array([-1e8], np.float32), "r": np.array([1.0], np.float32), "acc": np.zeros(1, np.float32)}
    out = oc.comm_steps(big, [("reduce_copy", ["acc", "p"], ["acc"]), ("reduce_copy", ["acc", "q"], ["acc"]), ("reduce_copy", ["acc", "r"], ["acc"])], oc.F32)
    assert out["acc"][0] == 1.0
    out = oc.comm_steps(big, [("reduce_copy", ["acc", "q"], ["acc"]), ("reduce_copy", ["acc", "r"], ["acc"]), ("reduce_copy", ["acc", "p"], ["acc"])], oc.F32)
    assert out["acc"][0] == 0.0
    with pytest.raises(ValueError):
        oc.comm_steps({"a": a, "b": b}, [("gather_copy", ["a", "b"], ["b"])], oc.F32)
