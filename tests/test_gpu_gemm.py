"""GPU parity: lagom_gemm through the C ABI against the fp64 oracle, rel-err <= 2e-2
(bf16 inputs, fp32 accumulation), both error measures."""
import numpy as np
import pytest
import torch

from oracle import collective as oc, gemm as og
from paper_2602_20656_amd import binding as lg, inputs
from gpu_util import dev, host

pytestmark = pytest.mark.gpu
GATE = 2e-2


def _gemm(a_bits, b_bits, b_is_nk, out):
    M, K = a_bits.shape
    N = b_bits.shape[0] if b_is_nk else b_bits.shape[1]
    dA, dB = dev(a_bits), dev(b_bits)
    pad = 256
    if out == "bf16":
        dC = dev(np.full(M * N + 2 * pad, 0x7B7B, np.uint16)); esz = 2
    else:
        dC = dev(np.full(M * N + 2 * pad, 123.0, np.float32)); esz = 4
    lg.lagom_gemm(dA, dB, dC.data_ptr() + pad * esz, M, N, K, b_is_nk,
                  lg.LAGOM_BF16 if out == "bf16" else lg.LAGOM_F32, torch.cuda.current_stream())
    torch.cuda.synchronize()
    h = host(dC, np.uint16 if out == "bf16" else np.float32)
    guard = h[:pad].tolist() + h[pad + M * N:].tolist()
    assert all(v == (0x7B7B if out == "bf16" else 123.0) for v in guard), "guard region clobbered"
    c = h[pad:pad + M * N].reshape(M, N)
    return oc.bf16_to_f32(c) if out == "bf16" else c


@pytest.mark.parametrize("M,N,K", [(512, 512, 512), (1, 1, 8), (300, 200, 136), (700, 520, 264), (256, 256, 64),
                                   (257, 255, 72), (33, 1000, 4096), (130, 77, 128), (513, 260, 192), (700, 300, 320), (1000, 520, 256), (300, 300, 64),
                                   # more than 256 tiles of 128 x 128 but not of 256 x 128: the 256 x 128 kernels, ragged, 1 to 4 K-steps
                                   (2100, 2200, 192), (2100, 2200, 64), (1800, 2440, 128), (2312, 1800, 256),
                                   # more than 256 tiles of 256 x 128, or a K tail: the 256 x 256 kernels, ragged in M and N
                                   (2100, 3720, 192), (2100, 3720, 64), (2100, 3720, 136),
                                   # K tails on the two smaller tilings
                                   (2312, 1800, 136), (1000, 520, 328)])
@pytest.mark.parametrize("b_is_nk", [True, False])
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_gemm_small_shapes(M, N, K, b_is_nk, out):
    if not b_is_nk and N % 8:
        pytest.skip("[K,N] layout needs N % 8 == 0")
    a = inputs.normal_bf16(2, (M, K))
    b = inputs.normal_bf16(3, (N, K) if b_is_nk else (K, N))
    ref = og.gemm_f64(a, b, b_is_nk)
    got = _gemm(a, b, b_is_nk, out)
    e_max, e_fro = og.rel_errors(got, ref)
    assert e_max <= GATE and e_fro <= GATE, (e_max, e_fro)
    if out == "f32":   # fp32 accumulation alone is orders of magnitude inside the gate
        assert e_fro < 1e-5, e_fro


@pytest.mark.parametrize("K", [1 << 22, (1 << 22) + 64])
def test_gemm_longest_k_of_the_fast_kernel_and_the_first_beyond_it(K):
    """K = 2^22 is the last K the LDS-direct kernel takes (32-bit lane offsets); the next multiple of 64 goes to the general one."""
    a = inputs.normal_bf16(2, (2, K)); b = inputs.normal_bf16(3, (3, K), 0.02)
    ref = og.gemm_f64(a, b, True)
    for out in ("bf16", "f32"):
        e_max, e_fro = og.rel_errors(_gemm(a, b, True, out), ref)
        assert e_max <= GATE and e_fro <= GATE, (K, out, e_max, e_fro)


def test_gemm_b_kn_widest_n_of_the_fast_kernel_and_the_first_beyond_it():
    """B stored [K,N]: N = 2^23 is the widest row the LDS-direct kernel takes (its lane offsets reach two
    K-steps = 128 rows of B ahead in 32 bits); N + 8 goes to the general one.  Three K-steps, so that the
    look-ahead offsets are used.  Checked on the first, some middle and the last columns."""
    M, K, wide = 2, 192, (1 << 23) + 8
    a = inputs.normal_bf16(2, (M, K))
    b_wide = inputs.random_bits_bf16(3, (K, wide))
    for N in (wide, 1 << 23):
        b = b_wide if N == wide else np.ascontiguousarray(b_wide[:, :N])
        got = _gemm(a, b, False, "f32")
        rng = np.random.default_rng(N)
        cols = np.unique(np.concatenate([np.arange(0, 64), rng.integers(0, N, size=256), np.arange(N - 300, N)]))
        ref = og.gemm_f64(a, np.ascontiguousarray(b[:, cols]), False)
        e_max, e_fro = og.rel_errors(got[:, cols], ref)
        assert e_max <= GATE and e_fro <= GATE and e_fro < 1e-5, (N, e_max, e_fro)
        del b, got


def test_gemm_integer_inputs_are_exact():
    rng = np.random.default_rng(5)
    ai = rng.integers(-4, 5, size=(260, 320)); bi = rng.integers(-4, 5, size=(270, 320))
    a, b = inputs.to_bf16_bits(ai.astype(np.float32)), inputs.to_bf16_bits(bi.astype(np.float32))
    got = _gemm(a, b, True, "f32")
    assert np.array_equal(got.astype(np.int64), ai @ bi.T)


@pytest.mark.parametrize("M,N,K", [(260, 272, 320), (100, 8, 64), (256, 776, 128), (513, 264, 192), (64, 1032, 576),
                                   (2100, 2056, 128), (2304, 2312, 320), (2100, 3720, 128)])
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_gemm_b_kn_integer_inputs_are_exact(M, N, K, out):
    """B stored [K,N] with K a multiple of 64 takes the kernel whose LDS reads transpose B: any mix-up of
    rows, columns or k order shows as a wrong integer.  One to nine K-steps, ragged M and N tiles, N = 8; the
    last three shapes run on 256 x 128 (two) and 256 x 256 tiles, the others on 128 x 128."""
    rng = np.random.default_rng(M + N + K)
    ai = rng.integers(-3, 4, size=(M, K)); bi = rng.integers(-3, 4, size=(K, N))
    a, b = inputs.to_bf16_bits(ai.astype(np.float32)), inputs.to_bf16_bits(bi.astype(np.float32))
    got = _gemm(a, b, False, out)
    want = ai @ bi
    if out == "bf16":   # |sums| < 9 * 576: not all representable in bf16; compare after the same rounding
        want = oc.bf16_to_f32(inputs.to_bf16_bits(want.astype(np.float32)))
    assert np.array_equal(got.astype(np.float64), want.astype(np.float64))


@pytest.mark.parametrize("K", [72, 96, 104, 120, 184, 4104])
@pytest.mark.parametrize("b_is_nk", [True, False])
@pytest.mark.parametrize("M,N", [(260, 272), (2100, 2056), (2100, 3720)])
def test_gemm_ragged_k_integer_inputs_are_exact(K, b_is_nk, M, N):
    """K >= 64 that is no multiple of 64: the LDS-direct kernels multiply the last K % 64 columns (8 to 56
    of them, one or two 32-wide slices) in a step of their own, zero filled from K on.  The three shapes
    run on 128 x 128, 256 x 128 and 256 x 256 tiles."""
    if K == 4104 and M > 1000:
        pytest.skip("one long K is enough")
    rng = np.random.default_rng(K)
    ai = rng.integers(-3, 4, size=(M, K)); bi = rng.integers(-3, 4, size=(K, N))
    a = inputs.to_bf16_bits(ai.astype(np.float32))
    b = inputs.to_bf16_bits((bi.T if b_is_nk else bi).astype(np.float32))
    got = _gemm(a, b, b_is_nk, "f32")
    assert np.array_equal(got.astype(np.int64), ai @ bi)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for i in range(n):
        M = int(rng.integers(1, 700)); N = 8 * int(rng.integers(1, 90))
        K = 64 * int(rng.integers(1, 7)) if i % 3 else 8 * int(rng.integers(1, 40))   # two in three on the LDS-direct kernels
        shapes.append((M, N, K))
    return shapes


@pytest.mark.parametrize("b_is_nk", [True, False])
def test_gemm_seeded_random_shapes(b_is_nk):
    """24 seeded shapes with ragged tiles in M and N and one to six K-steps, both kernels of each layout."""
    for n, (M, N, K) in enumerate(_random_shapes(24, 77)):
        a = inputs.normal_bf16(100 + n, (M, K))
        b = inputs.normal_bf16(200 + n, (N, K) if b_is_nk else (K, N))
        ref = og.gemm_f64(a, b, b_is_nk)
        got = _gemm(a, b, b_is_nk, "f32" if n % 2 else "bf16")
        e_max, e_fro = og.rel_errors(got, ref)
        assert e_max <= GATE and e_fro <= GATE, (M, N, K, e_max, e_fro)


def test_gemm_b_kn_full_size_sampled_rows():
    M = N = K = 4096
    a = inputs.normal_bf16(2, (M, K))
    b = inputs.normal_bf16(3, (K, N), scale=0.02)
    got = _gemm(a, b, False, "bf16")
    rng = np.random.default_rng(11)
    rows = np.unique(np.concatenate([rng.integers(0, M, size=64), np.arange(0, 4), np.arange(M - 4, M)]))
    ref = og.gemm_f64(a, b, False, rows=rows)
    e_max, e_fro = og.rel_errors(got[rows], ref)
    assert e_max <= GATE and e_fro <= GATE, (e_max, e_fro)
    corners = ref[:, np.r_[0:32, N - 32:N]]
    e_max, e_fro = og.rel_errors(got[rows][:, np.r_[0:32, N - 32:N]], corners)
    assert e_max <= GATE and e_fro <= GATE


def test_b_kn_layout_rejects_unaligned_n():
    with pytest.raises(lg.LagomError):
        lg.lagom_gemm(4096, 8192, 16384, 64, 60, 64, False)


@pytest.mark.parametrize("M,N,K", [(4096, 4096, 4096), (4096, 3584, 8192), (8192, 4096, 4096), (8192, 8192, 8192)])
def test_gemm_full_size_sampled_rows(M, N, K):
    """Benchmark shapes: 64 seeded rows x all columns, plus the four corner tiles, against the oracle."""
    a = inputs.normal_bf16(2, (M, K))
    b = inputs.normal_bf16(3, (N, K), scale=0.02)
    got = _gemm(a, b, True, "bf16")
    rng = np.random.default_rng(M + N + K)
    rows = np.unique(np.concatenate([rng.integers(0, M, size=64), np.arange(0, 4), np.arange(M - 4, M)]))
    ref = og.gemm_f64(a, b, True, rows=rows)
    e_max, e_fro = og.rel_errors(got[rows], ref)
    assert e_max <= GATE and e_fro <= GATE, (e_max, e_fro)
    corners = ref[:, np.r_[0:32, N - 32:N]]
    e_max, e_fro = og.rel_errors(got[rows][:, np.r_[0:32, N - 32:N]], corners)
    assert e_max <= GATE and e_fro <= GATE


# More 256 x 256 tiles than compute units: several rounds of workgroups, ragged in M and N.
@pytest.mark.parametrize("M,N,K", [(4100, 4200, 128),      # 17 x 17 = 289 tiles, ragged in M and N: 33 tiles in a second round
                                   (4352, 7704, 64),       # 17 x 31 = 527 tiles: two to three rounds, one K-step
                                   (8192, 8200, 192)])     # 32 x 33 = 1056 tiles: four to five rounds
@pytest.mark.parametrize("b_is_nk", [True, False])
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_gemm_more_tiles_than_compute_units_integer_inputs_are_exact(M, N, K, b_is_nk, out):
    """Small integers in bf16: every product and every partial sum is exact in fp32, so any tile that is skipped, done
    twice, mixed with its neighbour's operands or written to the wrong place shows as a wrong integer."""
    rng = np.random.default_rng(M + N + K)
    a = rng.integers(-4, 5, size=(M, K)).astype(np.float32)
    b = rng.integers(-4, 5, size=(N, K) if b_is_nk else (K, N)).astype(np.float32)
    got = _gemm(oc.f32_to_bf16(a), oc.f32_to_bf16(b), b_is_nk, out)
    want = (a @ (b.T if b_is_nk else b)).astype(np.float32)       # exact: every partial sum is a small integer
    if out == "bf16":                                                # one rounding at the store, the oracle's
        want = oc.bf16_to_f32(oc.f32_to_bf16(want))
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{len(bad)} wrong elements, first at {bad[0]} (tile {bad[0][0] // 256}, {bad[0][1] // 256})"
