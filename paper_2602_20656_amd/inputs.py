"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

This module holds no arithmetic of the method: it only draws numbers from a
counter-based generator (Philox keyed by the seed) and, for bf16 data, hands them to
PyTorch's own float32 -> bfloat16 conversion.  bf16 arrays are returned as
``numpy.uint16`` bit patterns so that the same bytes can be fed to the CPU oracle and
uploaded to the GPU.

The workloads mirror the shapes of the overlap patterns the paper studies
(Sec. 2.1: DP/TP AllReduce, FSDP AllGather/ReduceScatter; Fig. 3: one collective
against one FFN GEMM); the paper prints no tensor shapes, so the sizes below are this
build's stand-ins for its model workloads.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np
import torch

KiB = 1024
MiB = 1024 * 1024


def _gen(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def uniform_f32(seed: int, n: int) -> np.ndarray:
    """U[-1, 1) as float32."""
    u = _gen(seed).random(int(n), dtype=np.float32)
    return (u * np.float32(2.0) - np.float32(1.0)).astype(np.float32)


def normal_f32(seed: int, shape, scale: float = 1.0) -> np.ndarray:
    z = _gen(seed).standard_normal(shape, dtype=np.float32)
    return (z * np.float32(scale)).astype(np.float32)


def to_bf16_bits(values: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns through torch's conversion (a library routine)."""
    t = torch.from_numpy(np.ascontiguousarray(values, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def normal_bf16(seed: int, shape, scale: float = 1.0) -> np.ndarray:
    return to_bf16_bits(normal_f32(seed, shape, scale))


def random_bits_bf16(seed: int, shape) -> np.ndarray:
    """bf16 bit patterns drawn directly (cheap for very large arrays): random sign, exponent field in
    120..127 (magnitudes in [2^-7, 2)), random 7-bit mantissa; no zeros, infinities or NaNs."""
    n = int(np.prod(shape))
    words = _gen(seed).integers(0, np.iinfo(np.uint64).max, size=(n + 3) // 4, dtype=np.uint64, endpoint=True)
    r = words.view(np.uint16)[:n]
    r &= np.uint16(0x83FF)      # keep sign, the low 3 exponent bits and the mantissa
    r |= np.uint16(0x3C00)      # exponent bits 7..3 = 01111
    return r.reshape(shape)


def uniform_bf16(seed: int, n: int) -> np.ndarray:
    return to_bf16_bits(uniform_f32(seed, n))


def bits_to_torch_bf16(bits: np.ndarray, device="cpu") -> torch.Tensor:
    """View uint16 bit patterns as a torch.bfloat16 tensor (no value change)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t.to(device)


def torch_bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


# ------------------------------------------------------------------ workload shapes
@dataclass(frozen=True)
class CommShape:
    op: str            # "reduce_copy" | "gather_copy"
    dtype: str         # "f32" | "bf16"
    nsrc: int
    ndst: int
    count: int         # elements per source
    launches: int = 1  # kernel launches that make up one communication operator


@dataclass(frozen=True)
class Workload:
    name: str
    comm: CommShape
    ncomm: int                         # communication operators in the chain
    gemm: Tuple[int, int, int]         # (M, N, K)
    ncomp: int
    nc_grid: Tuple[int, ...]
    chunk_grid: Tuple[int, ...]
    nt_grid: Tuple[int, ...]
    seeds: Tuple[int, ...]
    scale: float = 1.0


_NC = (1, 2, 4, 8, 16, 32)
_C = tuple(32 * KiB << i for i in range(8))          # 32 KiB .. 4 MiB

WORKLOADS = {
    # two emulated peer buffers of 2^20 fp32, out = a + b, against a 512^3 GEMM
    "tiny": Workload("tiny", CommShape("reduce_copy", "f32", 2, 1, 1 << 20), 1, (512, 512, 512), 1,
                     (2, 4), (64 * KiB, 128 * KiB), (256,), (0, 1, 2, 3)),
    # one rank's share of a ring all-reduce of a 25 MiB bf16 bucket in 8 rank-chunks:
    # 7 reduce steps then 7 copy steps, all one communication operator
    "dp_bucket": Workload("dp_bucket", CommShape("reduce_copy", "bf16", 2, 1, 1638400, launches=14), 1,
                          (4096, 4096, 4096), 1, _NC, _C, (256,), tuple(range(10, 18)), scale=0.125),
    # one-shot reduce-scatter share: 8 shards of 1/8 of a 4096 x 8192 bf16 activation
    "tp_layer": Workload("tp_layer", CommShape("reduce_copy", "bf16", 8, 1, 4194304), 1,
                         (4096, 3584, 8192), 1, _NC, _C, (128, 256, 512, 1024), tuple(range(20, 28))),
    # 8 all-gather copies (8 bf16 shards -> one 32 MiB weight) against 8 GEMMs
    "fsdp_chain": Workload("fsdp_chain", CommShape("gather_copy", "bf16", 8, 1, 2097152), 8,
                           (8192, 4096, 4096), 8, _NC, _C, (256,), tuple(range(30, 38)), scale=0.02),
    # back-to-back 16 MiB fp32 two-buffer reduce-copies against one 8192^3 GEMM
    "compute_bound": Workload("compute_bound", CommShape("reduce_copy", "f32", 2, 1, 4194304, launches=3), 1,
                              (8192, 8192, 8192), 1, _NC, _C, (128, 256, 512, 1024), (40, 41)),
    # expert parallelism: one rank's share of an all-to-all of 8 x 4096 tokens x 2048 bf16 (a gather-copy whose
    # sources start at this rank's block of every peer's send buffer) against one expert GEMM
    "ep_alltoall": Workload("ep_alltoall", CommShape("gather_copy", "bf16", 8, 1, 1048576), 1,
                            (4096, 8192, 2048), 1, _NC, _C, (256,), tuple(range(50, 58))),
    # two communications of different kinds in one overlap (reduce-scatter share, then all-gather) against
    # three GEMMs: which one the search raises first is decided by the metric H
    # tensor parallelism with batch pipelining: four micro-batches, the reduce-scatter share of micro-batch b
    # (this rank's partial output + seven peers' partials) waits for GEMM b and overlaps GEMM b+1
    "tp_pipeline": Workload("tp_pipeline", CommShape("reduce_copy", "bf16", 8, 1, 1835008), 4,
                            (4096, 3584, 8192), 4, _NC, _C, (256,), tuple(range(80, 88))),
    "rs_ag_pair": Workload("rs_ag_pair", CommShape("reduce_copy", "bf16", 8, 1, 4194304), 2,
                           (8192, 4096, 4096), 3, _NC, _C, (256,), tuple(range(60, 76)), scale=0.02),
}
