"""Oracle: C = A . B from bf16 inputs -- TEST INFRASTRUCTURE ONLY.

The computation whose slow-down the paper studies is a matrix multiply (the FFN of
Fig. 3, the MatMuls of Sec. 3.3).  Its definition is the plain contraction
C[m, n] = sum_k A[m, k] * B[k, n].  Inputs are bf16 bit patterns (``uint16``); the
reference accumulates in fp64 (no rounding of consequence), and a second routine
accumulates in fp32 with k ascending, to size the error a fp32-accumulating kernel
may show.  B is stored either [N, K] (weight layout, ``b_is_nk=True``) or [K, N].
"""
from __future__ import annotations

import numpy as np

from .collective import bf16_to_f32, f32_to_bf16


def _operands(a_bits, b_bits, b_is_nk):
    a = bf16_to_f32(a_bits).astype(np.float64)
    b = bf16_to_f32(b_bits).astype(np.float64)
    if a.ndim != 2 or b.ndim != 2:
        raise ValueError("A and B must be matrices")
    if b_is_nk:
        b = b.T  # now [K, N]
    if a.shape[1] != b.shape[0]:
        raise ValueError("inner dimensions differ")
    return a, b


def gemm_f64(a_bits, b_bits, b_is_nk: bool = True, rows=None) -> np.ndarray:
    """fp64 reference.  ``rows`` (optional index array) restricts to those rows of C."""
    a, b = _operands(a_bits, b_bits, b_is_nk)
    if rows is not None:
        a = a[np.asarray(rows)]
    return a @ b


def gemm_f32_kascending(a_bits, b_bits, b_is_nk: bool = True) -> np.ndarray:
    """fp32 accumulation, k ascending, one multiply and one add per term (small sizes)."""
    a, b = _operands(a_bits, b_bits, b_is_nk)
    a32, b32 = a.astype(np.float32), b.astype(np.float32)
    acc = np.zeros((a32.shape[0], b32.shape[1]), dtype=np.float32)
    for k in range(a32.shape[1]):
        prod = (a32[:, k:k + 1] * b32[k:k + 1, :]).astype(np.float32)
        acc = (acc + prod).astype(np.float32)
    return acc


def round_output(c: np.ndarray, out_dtype: str) -> np.ndarray:
    """What the stored output would be: fp32, or bf16 bit patterns (RNE)."""
    c32 = c.astype(np.float32)
    return c32 if out_dtype == "f32" else f32_to_bf16(c32)


def rel_errors(c: np.ndarray, ref: np.ndarray):
    """(max-abs error / max-abs reference, Frobenius error / Frobenius reference)."""
    c = np.asarray(c, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = c - ref
    max_ref = float(np.max(np.abs(ref))) if ref.size else 0.0
    fro_ref = float(np.sqrt(np.sum(ref * ref)))
    e_max = float(np.max(np.abs(diff))) / max_ref if max_ref > 0 else float(np.max(np.abs(diff), initial=0.0))
    e_fro = float(np.sqrt(np.sum(diff * diff))) / fro_ref if fro_ref > 0 else float(np.sqrt(np.sum(diff * diff)))
    return e_max, e_fro
