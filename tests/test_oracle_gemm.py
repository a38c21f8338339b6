"""Pins for oracle/gemm.py and the C GEMM loop: exact special cases, brute force on tiny
inputs with exact rationals, and the library matmul on integer-valued data."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import cloops, collective as oc, gemm as og
from paper_2602_20656_amd import inputs


def _bits(x):
    return inputs.to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_k1_is_an_outer_product():
    a = inputs.normal_bf16(2, (37, 1))
    b_nk = inputs.normal_bf16(3, (29, 1))
    c = og.gemm_f64(a, b_nk, b_is_nk=True)
    want = np.outer(oc.bf16_to_f32(a[:, 0]).astype(np.float64), oc.bf16_to_f32(b_nk[:, 0]).astype(np.float64))
    assert np.array_equal(c, want)


def test_identity_b_returns_a_in_both_layouts():
    a = inputs.normal_bf16(2, (19, 16))
    eye = _bits(np.eye(16))
    for nk in (True, False):
        c = og.gemm_f64(a, eye, b_is_nk=nk)
        assert np.array_equal(c, oc.bf16_to_f32(a).astype(np.float64))
        assert np.array_equal(og.round_output(c, "bf16"), a)


def test_b_layout_flag_selects_the_right_operand_index():
    # A = e_1 e_2^T (M=3, K=4); B[k=2, n=5] = 7 only -> C[1, 5] = 7 and nothing else
    a = np.zeros((3, 4), np.float32); a[1, 2] = 1.0
    b_kn = np.zeros((4, 6), np.float32); b_kn[2, 5] = 7.0
    want = np.zeros((3, 6)); want[1, 5] = 7.0
    assert np.array_equal(og.gemm_f64(_bits(a), _bits(b_kn), b_is_nk=False), want)
    assert np.array_equal(og.gemm_f64(_bits(a), _bits(b_kn.T.copy()), b_is_nk=True), want)
    assert np.array_equal(cloops.gemm(_bits(a), _bits(b_kn), b_is_nk=False), want)
    assert np.array_equal(cloops.gemm(_bits(a), _bits(b_kn.T.copy()), b_is_nk=True), want)


def test_tiny_case_against_exact_rational_brute_force():
    a_bits = inputs.normal_bf16(2, (4, 5))
    b_bits = inputs.normal_bf16(3, (3, 5))   # [N, K]
    a = oc.bf16_to_f32(a_bits); b = oc.bf16_to_f32(b_bits)
    c = og.gemm_f64(a_bits, b_bits, True)
    c32 = og.gemm_f32_kascending(a_bits, b_bits, True)
    for m in range(4):
        for n in range(3):
            exact = sum(Fraction(float(a[m, k])) * Fraction(float(b[n, k])) for k in range(5))
            assert abs(Fraction(float(c[m, n])) - exact) <= abs(exact) * Fraction(1, 2**48) + Fraction(1, 2**80)
            assert abs(Fraction(float(c32[m, n])) - exact) <= Fraction(1, 2**18)


def test_integer_valued_inputs_are_exact_in_every_routine():
    rng = np.random.default_rng(5)
    ai = rng.integers(-8, 9, size=(33, 70)); bi = rng.integers(-8, 9, size=(21, 70))
    want = ai @ bi.T
    a, b = _bits(ai), _bits(bi)
    assert np.array_equal(og.gemm_f64(a, b, True).astype(np.int64), want)
    assert np.array_equal(og.gemm_f32_kascending(a, b, True).astype(np.int64), want)
    assert np.array_equal(cloops.gemm(a, b, True, threads=3).astype(np.int64), want)
    rows = [0, 5, 32]
    assert np.array_equal(og.gemm_f64(a, b, True, rows=rows).astype(np.int64), want[rows])
    assert np.array_equal(cloops.gemm(a, b, True, row_lo=5, row_hi=9).astype(np.int64), want[5:9])


def test_fp32_accumulation_error_and_bf16_output_error_are_far_below_the_gate():
    a = inputs.normal_bf16(2, (64, 512)); b = inputs.normal_bf16(3, (48, 512))
    ref = og.gemm_f64(a, b, True)
    e_max, e_fro = og.rel_errors(og.gemm_f32_kascending(a, b, True), ref)
    assert e_max < 1e-5 and e_fro < 1e-5
    stored = oc.bf16_to_f32(og.round_output(ref, "bf16"))
    e_max, e_fro = og.rel_errors(stored, ref)
    assert e_max < 2 ** -8 and e_fro < 2 ** -8          # one bf16 rounding: half an ulp = 2^-9 relative
    assert og.rel_errors(ref, ref) == (0.0, 0.0)
    assert og.rel_errors(ref * 1.5, ref)[0] == pytest.approx(0.5)


def test_c_loop_matches_numpy_reference_on_random_data():
    a = inputs.normal_bf16(2, (17, 96)); b = inputs.normal_bf16(3, (23, 96))
    ref = og.gemm_f64(a, b, True)
    got = cloops.gemm(a, b, True, threads=2)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
