"""Oracle: the local data-movement steps of chunked collectives, on the CPU.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

The paper (Sec. 3.2, "Global Resource Competition") describes a communication
operator as NC thread blocks that read and write data at a granularity of C, and
Sec. 2.1 names the collectives whose local steps are meant (AllReduce for TP/DP,
AllGather and ReduceScatter for FSDP).  The *result* of such a step has a plain
definition that does not depend on (NC, NT, C); that definition is what is written
out here:

* reduce-copy:  dst_d[i] = round_dt(((src_0[i] + src_1[i]) + src_2[i]) + ...),
  fp32 additions in source order, one final rounding to the element type, the same
  value stored to every destination;
* gather-copy:  dst[r*n + i] = src_r[i]  (concatenation in rank order).

bf16 values travel as ``numpy.uint16`` bit patterns; fp32 as ``numpy.float32``.
"""
from __future__ import annotations

import numpy as np

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------- bf16
def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly (bf16 is the upper half of fp32)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(values: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 bit patterns, round-to-nearest, ties to even.

    Textbook rule on the 32-bit pattern u: keep the upper 16 bits and add one to
    them when the discarded half is above 0x8000, or equal to 0x8000 with the kept
    half odd.  NaN stays NaN (quiet bit forced so the payload cannot round to Inf).
    """
    u = np.ascontiguousarray(values, dtype=np.float32).view(np.uint32)
    upper = u >> np.uint32(16)
    lower = u & np.uint32(0xFFFF)
    round_up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    out = upper + round_up.astype(np.uint32)
    is_nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    out = np.where(is_nan, upper | np.uint32(0x0040), out)
    return out.astype(np.uint16)


def _widen(buf: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == F32:
        a = np.asarray(buf)
        assert a.dtype == np.float32
        return a
    if dtype == BF16:
        return bf16_to_f32(buf)
    raise ValueError(f"unknown dtype {dtype!r}")


def _narrow(acc: np.ndarray, dtype: str) -> np.ndarray:
    return acc.astype(np.float32) if dtype == F32 else f32_to_bf16(acc)


# ------------------------------------------------------------- local steps (a1, a2)
def reduce_copy(srcs, dtype: str, ndst: int = 1):
    """Left fold of the sources in fp32, one rounding, copied to ``ndst`` outputs.

    Sec. 3.2: the local step of a ring all-reduce / reduce-scatter.  Returns a list
    of ``ndst`` identical arrays (separate objects, as separate peer buffers).
    """
    if len(srcs) < 1 or ndst < 1:
        raise ValueError("need at least one source and one destination")
    n = len(srcs[0])
    acc = _widen(srcs[0], dtype).astype(np.float32, copy=True)
    with np.errstate(over="ignore", invalid="ignore"):   # Inf and NaN inputs are legal data
        for s in srcs[1:]:
            if len(s) != n:
                raise ValueError("sources differ in length")
            acc = (acc + _widen(s, dtype)).astype(np.float32)  # one fp32 add per source, in order
    out = _narrow(acc, dtype)
    return [out.copy() for _ in range(ndst)]


def gather_copy(srcs, ndst: int = 1):
    """Concatenate the shards in rank order (the local step of an all-gather)."""
    if len(srcs) < 1 or ndst < 1:
        raise ValueError("need at least one source and one destination")
    n = len(srcs[0])
    for s in srcs:
        if len(s) != n:
            raise ValueError("shards differ in length")
    out = np.empty(n * len(srcs), dtype=np.asarray(srcs[0]).dtype)
    for r, s in enumerate(srcs):
        for_slice = slice(r * n, (r + 1) * n)
        out[for_slice] = s
    return [out.copy() for _ in range(ndst)]


# ------------------------------------------------ chunk -> channel schedule (Sec. 3.2)
def chunk_schedule(nbytes_per_shard: int, nshards: int, nc: int, chunk_bytes: int):
    """Which channel moves which byte range: NC channels, granularity C.

    Chunks are numbered shard by shard (chunking restarts at every shard so that no
    chunk straddles a shard boundary); chunk g belongs to channel g mod NC; the last
    chunk of a shard may be short.  Returns a list of NC lists of
    (shard, byte_offset_in_shard, byte_length).
    """
    if nc < 1 or chunk_bytes < 1 or nshards < 1 or nbytes_per_shard < 0:
        raise ValueError("bad schedule arguments")
    per_shard = -(-nbytes_per_shard // chunk_bytes)
    plan = [[] for _ in range(nc)]
    g = 0
    for r in range(nshards):
        for c in range(per_shard):
            off = c * chunk_bytes
            plan[g % nc].append((r, off, min(chunk_bytes, nbytes_per_shard - off)))
            g += 1
    return plan


def reduce_copy_chunked(srcs, dtype: str, nc: int, chunk_bytes: int):
    """reduce_copy carried out chunk by chunk in channel order.

    Exists to show that the result does not depend on (NC, C): tests compare it with
    ``reduce_copy`` bit for bit.
    """
    esize = 4 if dtype == F32 else 2
    if chunk_bytes % esize:
        raise ValueError("chunk must hold whole elements")
    n = len(srcs[0])
    out = np.zeros(n, dtype=np.float32 if dtype == F32 else np.uint16)
    for channel in chunk_schedule(n * esize, 1, nc, chunk_bytes):
        for _, off, length in channel:
            lo, hi = off // esize, (off + length) // esize
            out[lo:hi] = reduce_copy([s[lo:hi] for s in srcs], dtype)[0]
    return out


# ------------------------------------------------- collectives composed of local steps
def reduce_scatter_direct(contribs, dtype: str):
    """One-shot reduce-scatter on P emulated ranks.

    ``contribs[p]`` is rank p's full-length contribution (length divisible by P).
    Rank r's output is the fixed-order fold over p = 0..P-1 of slice r, rounded once.
    Returns the list of P per-rank outputs.
    """
    P = len(contribs)
    n = len(contribs[0])
    if n % P:
        raise ValueError("length must divide by the number of ranks")
    m = n // P
    return [reduce_copy([c[r * m:(r + 1) * m] for c in contribs], dtype)[0] for r in range(P)]


def all_gather(shards):
    """Every rank ends with the concatenation of all shards."""
    full = gather_copy(shards)[0]
    return [full.copy() for _ in shards]


def all_to_all(send_buffers):
    """Every rank sends block s of its buffer to rank s (Sec. 2.1, expert parallelism).

    ``send_buffers[r]`` holds P equal blocks; rank r's receive buffer is the concatenation over
    senders s of block r of ``send_buffers[s]``.  On rank r this is a gather-copy whose source s
    starts at block r of peer s's buffer, which is how the kernel is driven.
    """
    P = len(send_buffers)
    n = len(send_buffers[0])
    if n % P:
        raise ValueError("buffer length must divide by the number of ranks")
    m = n // P
    out = []
    for r in range(P):
        recv = np.empty(n, dtype=np.asarray(send_buffers[0]).dtype)
        for s_ in range(P):
            recv[s_ * m:(s_ + 1) * m] = send_buffers[s_][r * m:(r + 1) * m]
        out.append(recv)
    return out


def ring_all_reduce(buckets, dtype: str):
    """Textbook ring all-reduce on P emulated ranks, built from local steps only.

    Each bucket is split into P rank-chunks.  Reduce-scatter phase, step s = 0..P-2:
    rank r receives chunk (r - s - 1) mod P from rank r-1, folds its own copy of that
    chunk onto it (incoming first, then local: out = incoming + local) and the result,
    rounded to the wire dtype, is what it forwards at the next step.  After P-1 steps
    rank r holds the finished chunk (r + 1) mod P.  All-gather phase, step s = 0..P-2:
    rank r receives the finished chunk (r - s) mod P from rank r-1, stores it locally
    and forwards it.  Because the wire carries ``dtype``, partial sums are re-rounded
    at every reduce step.  Returns the P final buckets (identical bits on every rank).
    """
    P = len(buckets)
    n = len(buckets[0])
    if n % P:
        raise ValueError("bucket length must divide by the number of ranks")
    m = n // P
    data = [np.array(b, copy=True) for b in buckets]

    def chunk(r, c):
        return data[r][c * m:(c + 1) * m]

    # what rank r sends at step 0 of the reduce phase: its own chunk r
    outgoing = [chunk(r, r).copy() for r in range(P)]
    for s in range(P - 1):
        incoming = [outgoing[(r - 1) % P] for r in range(P)]
        new_out = []
        for r in range(P):
            c = (r - s - 1) % P
            red = reduce_copy([incoming[r], chunk(r, c)], dtype)[0]
            if s == P - 2:
                chunk(r, c)[:] = red  # last reduce step also lands in the local bucket
            new_out.append(red)
        outgoing = new_out
    # now rank r owns finished chunk (r + 1) mod P, held in outgoing[r]
    for s in range(P - 1):
        incoming = [outgoing[(r - 1) % P] for r in range(P)]
        new_out = []
        for r in range(P):
            c = (r - s) % P
            chunk(r, c)[:] = incoming[r]
            new_out.append(incoming[r])
        outgoing = new_out
    return data


def comm_steps(buffers: dict, steps, dtype: str) -> dict:
    """Several local steps of one collective, one after the other (Sec. 2.1: a ring all-reduce share is P-1 reduce
    steps followed by P-1 copy steps).  `buffers` maps a name to an array; `steps` is a list of
    (op, source names, destination names) with op "reduce_copy" or "gather_copy" (one source: store and forward).
    Every step is the plain definition above applied to the current contents; a step sees what earlier steps wrote.
    Returns the final contents (the input dict is not modified)."""
    state = {k: np.array(v, copy=True) for k, v in buffers.items()}
    for op, srcs, dsts in steps:
        if op == "reduce_copy":
            out = reduce_copy([state[s] for s in srcs], dtype, 1)[0]
        elif op == "gather_copy":
            if len(srcs) != 1:
                raise ValueError("a copy step forwards one source")
            out = state[srcs[0]].copy()
        else:
            raise ValueError("unknown step")
        for d in dsts:
            state[d] = out.copy()
    return state
