"""ctypes binding of liblagom.so: argument marshalling only.

Every function here has the name and the meaning of the C entry point it wraps
(see include/lagom.h); all work is done by the native library.  Device buffers may be
passed as torch tensors (their ``data_ptr()`` is taken) or as integer addresses; streams
as ``torch.cuda.Stream`` objects or integer ``hipStream_t`` handles.

There is no fallback: if the shared library has not been built, importing a symbol
raises, and every call that returns an error code raises ``LagomError``.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple, Union

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblagom.so")

LAGOM_OK, LAGOM_EINVAL, LAGOM_EALIGN, LAGOM_EHIP, LAGOM_ECALLBACK = 0, -1, -2, -3, -4
LAGOM_F32, LAGOM_BF16 = 0, 1
LAGOM_REDUCE_COPY, LAGOM_GATHER_COPY = 0, 1
LAGOM_ALONE_COMM, LAGOM_ALONE_COMP, LAGOM_CORUN = 0, 1, 2
LAGOM_PRIORITY, LAGOM_EXHAUSTIVE, LAGOM_COMM_OPTIMAL, LAGOM_HIDE_COMM, LAGOM_EXHAUSTIVE_HIDE, LAGOM_PRIORITY_FREE = 0, 1, 2, 3, 4, 5
LAGOM_LADDER_FULL, LAGOM_LADDER_CUT, LAGOM_LADDER_FIXED_CHUNK = 0, 1, 2
LAGOM_MAX_SRCS, LAGOM_MAX_DSTS, LAGOM_MAX_LAUNCHES, LAGOM_MAX_COMMS = 16, 4, 256, 64
LAGOM_MAX_STEPS, LAGOM_MAX_STEP_PTRS = 32, 96

EXPORTS = ["lagom_strerror", "lagom_last_error", "lagom_comm_kernel", "lagom_gemm", "lagom_gemm_describe",
           "lagom_overlap_run", "lagom_contention_sweep", "lagom_comm_bytes", "lagom_cost_model", "lagom_tune",
           "lagom_model_profile", "lagom_overlap_profile", "lagom_streams_overlap", "lagom_overlap_steps", "lagom_overlap_steps_graph",
           "lagom_model_fill", "lagom_model_calibrate", "lagom_ladder_chunks", "lagom_comm_steps", "lagom_comm_kernel_lds"]


class LagomError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"lagom error {code}: {text}")
        self.code = code


# ------------------------------------------------------------------------ C structs
class lagom_cfg(C.Structure):
    _fields_ = [("nc", C.c_int32), ("nt", C.c_int32), ("chunk_bytes", C.c_int64)]


class lagom_gemm_geometry(C.Structure):
    _fields_ = [("mu", C.c_int64), ("tb", C.c_int32), ("d_bytes", C.c_double),
                ("tile_m", C.c_int32), ("tile_n", C.c_int32), ("tile_k", C.c_int32), ("threads", C.c_int32),
                ("d_bytes_past_l2", C.c_double)]


class lagom_comm_desc(C.Structure):
    _fields_ = [("op", C.c_int32), ("dtype", C.c_int32), ("srcs", C.POINTER(C.c_void_p)), ("nsrc", C.c_int32),
                ("dsts", C.POINTER(C.c_void_p)), ("ndst", C.c_int32), ("count", C.c_int64), ("comm_id", C.c_int32),
                ("after_comp", C.c_int32), ("lds_staged", C.c_int32), ("fuse_with_prev", C.c_int32)]


class lagom_comm_step(C.Structure):
    _fields_ = [("op", C.c_int32), ("srcs", C.POINTER(C.c_void_p)), ("nsrc", C.c_int32),
                ("dsts", C.POINTER(C.c_void_p)), ("ndst", C.c_int32)]


class lagom_gemm_desc(C.Structure):
    _fields_ = [("A", C.c_void_p), ("B", C.c_void_p), ("C", C.c_void_p), ("M", C.c_int64), ("N", C.c_int64),
                ("K", C.c_int64), ("b_is_nk", C.c_int32), ("out_dtype", C.c_int32), ("after_comm_id", C.c_int32)]


class lagom_timing(C.Structure):
    _fields_ = [("X_us", C.c_double), ("Y_us", C.c_double), ("Z_us", C.c_double),
                ("x_us", C.POINTER(C.c_double)), ("y_us", C.POINTER(C.c_double)),
                ("x_mad_us", C.POINTER(C.c_double)), ("Ysum_us", C.c_double), ("Ysum_mad_us", C.c_double), ("Z_mad_us", C.c_double),
                ("comm_start_us", C.c_double), ("comp_start_us", C.c_double)]


class lagom_sweep_point(C.Structure):
    _fields_ = [("cfg", lagom_cfg), ("comm_alone_us", C.c_double), ("comm_corun_us", C.c_double),
                ("comp_alone_us", C.c_double), ("comp_corun_us", C.c_double), ("z_corun_us", C.c_double),
                ("v_alone", C.c_double), ("v_corun", C.c_double)]


class lagom_table_entry(C.Structure):
    _fields_ = [("cfg", lagom_cfg), ("x_us", C.c_double), ("v", C.c_double)]


class lagom_comm_table(C.Structure):
    _fields_ = [("entries", C.POINTER(lagom_table_entry)), ("n", C.c_int32)]


class lagom_comp_model(C.Structure):
    _fields_ = [("mu", C.c_int64), ("tb", C.c_int32), ("d_bytes", C.c_double), ("theta_us", C.c_double)]


class lagom_penalty(C.Structure):
    _fields_ = [("nt", C.c_int32), ("rho", C.c_double)]


class lagom_model(C.Structure):
    _fields_ = [("lambda_", C.c_int32), ("bw_peak", C.c_double), ("comps", C.POINTER(lagom_comp_model)),
                ("ncomp", C.c_int32), ("tables", C.POINTER(lagom_comm_table)), ("ncomm", C.c_int32),
                ("comp_after_comm", C.POINTER(C.c_int32)), ("comm_after_comp", C.POINTER(C.c_int32)),
                ("corun_share", C.c_double), ("penalty", C.POINTER(lagom_penalty)), ("npenalty", C.c_int32)]


class lagom_pred(C.Structure):
    _fields_ = [("X_us", C.c_double), ("Y_us", C.c_double), ("Z_us", C.c_double),
                ("x_us", C.POINTER(C.c_double)), ("y_us", C.POINTER(C.c_double)), ("g", C.POINTER(C.c_int32))]


class lagom_tune_space(C.Structure):
    _fields_ = [("nc", C.POINTER(C.c_int32)), ("n_nc", C.c_int32), ("nt", C.POINTER(C.c_int32)), ("n_nt", C.c_int32),
                ("chunk", C.POINTER(C.c_int64)), ("n_chunk", C.c_int32)]


class lagom_trace_step(C.Structure):
    _fields_ = [("comm", C.c_int32), ("level_from", C.c_int32), ("level_to", C.c_int32), ("accepted", C.c_int32),
                ("done", C.c_int32), ("xj_prev", C.c_double), ("xj_new", C.c_double), ("X", C.c_double),
                ("Y", C.c_double), ("Z", C.c_double), ("H", C.c_double), ("lr", C.c_double)]


class lagom_trace(C.Structure):
    _fields_ = [("steps", C.POINTER(lagom_trace_step)), ("capacity", C.c_int32), ("n", C.c_int32),
                ("calls", C.c_int32), ("X", C.c_double), ("Y", C.c_double), ("Z", C.c_double),
                ("levels", C.POINTER(C.c_int32))]


class lagom_profile_log(C.Structure):
    _fields_ = [("capacity", C.c_int32), ("ncomm", C.c_int32), ("n", C.c_int32), ("cfgs", C.POINTER(lagom_cfg)),
                ("x_us", C.POINTER(C.c_double)), ("x_mad_us", C.POINTER(C.c_double)),
                ("Y_us", C.POINTER(C.c_double)), ("Y_mad_us", C.POINTER(C.c_double)),
                ("Z_us", C.POINTER(C.c_double)), ("Z_mad_us", C.POINTER(C.c_double)), ("iters", C.POINTER(C.c_int32))]


class lagom_overlap_ctx(C.Structure):
    _fields_ = [("launches", C.POINTER(lagom_comm_desc)), ("nlaunch", C.c_int32),
                ("comps", C.POINTER(lagom_gemm_desc)), ("ncomp", C.c_int32),
                ("comm_stream", C.c_void_p), ("comp_stream", C.c_void_p), ("warmup", C.c_int32), ("iters", C.c_int32),
                ("min_total_us", C.c_double), ("max_iters", C.c_int32), ("log", C.POINTER(lagom_profile_log))]


class lagom_fill_desc(C.Structure):
    _fields_ = [("lambda_", C.c_int32), ("bw_peak", C.c_double), ("mu", C.c_int64), ("tb", C.c_int32), ("d_bytes", C.c_double),
                ("ncomp", C.c_int32), ("ncomm", C.c_int32), ("comm_bytes", C.POINTER(C.c_double)), ("v_cap_frac", C.c_double)]


class lagom_calibration(C.Structure):
    _fields_ = [("sigma", C.c_double), ("theta_us", C.c_double), ("fit_mean", C.c_double), ("fit_max", C.c_double),
                ("held_mean", C.c_double), ("held_max", C.c_double), ("n_fit", C.c_int32), ("n_held", C.c_int32),
                ("npenalty", C.c_int32)]


PROFILE_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(lagom_cfg), C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double))

# --------------------------------------------------------------------------- loading
_lib = None


def lib() -> C.CDLL:
    """The loaded native library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_20656_amd.build` "
                              "(there is no CPU fallback)")
        # PyTorch carries its own copy of the HIP runtime.  Whichever copy is loaded first serves the whole process, and
        # a second one sees no device: load torch's before this library so that tensors, streams and kernels share one.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.lagom_strerror.restype = C.c_char_p
        L.lagom_strerror.argtypes = [C.c_int]
        L.lagom_last_error.restype = C.c_char_p
        L.lagom_comm_kernel.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_void_p), C.c_int, C.POINTER(C.c_void_p), C.c_int,
                                        C.c_int64, C.POINTER(lagom_cfg), C.c_void_p]
        L.lagom_comm_kernel_lds.argtypes = L.lagom_comm_kernel.argtypes
        L.lagom_comm_steps.argtypes = [C.c_int, C.POINTER(lagom_comm_step), C.c_int, C.c_int64, C.POINTER(lagom_cfg), C.c_void_p]
        L.lagom_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]
        L.lagom_gemm_describe.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int, C.POINTER(lagom_gemm_geometry)]
        L.lagom_overlap_run.argtypes = [C.POINTER(lagom_comm_desc), C.c_int, C.POINTER(lagom_cfg), C.c_int,
                                        C.POINTER(lagom_gemm_desc), C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_int, C.c_int, C.c_int, C.POINTER(lagom_timing)]
        L.lagom_contention_sweep.argtypes = [C.POINTER(lagom_comm_desc), C.c_int, C.c_int, C.POINTER(lagom_gemm_desc), C.c_int,
                                             C.POINTER(lagom_cfg), C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                             C.POINTER(lagom_sweep_point)]
        L.lagom_streams_overlap.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int)]
        L.lagom_overlap_steps.argtypes = [C.POINTER(lagom_comm_desc), C.c_int, C.POINTER(lagom_cfg), C.c_int,
                                          C.POINTER(lagom_gemm_desc), C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_double)]
        L.lagom_overlap_steps_graph.argtypes = L.lagom_overlap_steps.argtypes
        L.lagom_comm_bytes.restype = C.c_int64
        L.lagom_comm_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64]
        L.lagom_cost_model.argtypes = [C.POINTER(lagom_model), C.POINTER(lagom_cfg), C.c_int, C.POINTER(lagom_pred)]
        L.lagom_tune.argtypes = [C.POINTER(lagom_tune_space), C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                 C.POINTER(lagom_cfg), C.POINTER(lagom_trace)]
        L.lagom_model_fill.argtypes = [C.POINTER(lagom_sweep_point), C.c_int, C.POINTER(C.c_uint8), C.POINTER(lagom_fill_desc),
                                       C.POINTER(lagom_table_entry), C.POINTER(lagom_comm_table), C.POINTER(lagom_comp_model),
                                       C.POINTER(C.c_double)]
        L.lagom_model_calibrate.argtypes = [C.POINTER(lagom_sweep_point), C.c_int, C.POINTER(C.c_uint8), C.POINTER(lagom_fill_desc),
                                            C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_double), C.c_int,
                                            C.POINTER(C.c_double), C.c_int, C.POINTER(lagom_penalty), C.c_int,
                                            C.POINTER(lagom_calibration)]
        L.lagom_ladder_chunks.argtypes = [C.POINTER(C.c_int64), C.c_int, C.c_int32, C.c_int32, C.c_int64, C.c_int,
                                          C.POINTER(lagom_sweep_point), C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != LAGOM_OK:
        L = lib()
        raise LagomError(rc, f"{L.lagom_strerror(rc).decode()}: {L.lagom_last_error().decode()}")


def _ptr(x) -> int:
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def _stream(s) -> int:
    if s is None:
        return 0
    return int(s.cuda_stream) if hasattr(s, "cuda_stream") else int(s)


def _ptr_array(xs):
    arr = (C.c_void_p * len(xs))()
    for i, x in enumerate(xs):
        arr[i] = _ptr(x)
    return arr


CfgLike = Union[Tuple[int, int, int], lagom_cfg]


def _cfg(c: CfgLike) -> lagom_cfg:
    return c if isinstance(c, lagom_cfg) else lagom_cfg(int(c[0]), int(c[1]), int(c[2]))


def _cfg_array(cfgs: Sequence[CfgLike]):
    arr = (lagom_cfg * max(len(cfgs), 1))()
    for i, c in enumerate(cfgs):
        arr[i] = _cfg(c)
    return arr


# ----------------------------------------------------------------------- entry points
def lagom_comm_kernel(op: int, dt: int, srcs, dsts, count: int, cfg: CfgLike, stream=None) -> None:
    c = _cfg(cfg)
    _check(lib().lagom_comm_kernel(op, dt, _ptr_array(srcs), len(srcs), _ptr_array(dsts), len(dsts),
                                   int(count), C.byref(c), _stream(stream)))


def lagom_comm_kernel_lds(op: int, dt: int, srcs, dsts, count: int, cfg: CfgLike, stream=None) -> None:
    c = _cfg(cfg)
    _check(lib().lagom_comm_kernel_lds(op, dt, _ptr_array(srcs), len(srcs), _ptr_array(dsts), len(dsts),
                                       int(count), C.byref(c), _stream(stream)))


def lagom_comm_steps(dt: int, steps: Sequence[Tuple[int, Sequence, Sequence]], count: int, cfg: CfgLike, stream=None) -> None:
    """steps: (op, srcs, dsts) per local step, all of `count` elements of dt; one kernel launch for all of them."""
    c = _cfg(cfg)
    arr = (lagom_comm_step * max(len(steps), 1))()
    keep = []
    for i, (op, srcs, dsts) in enumerate(steps):
        a, b = _ptr_array(srcs), _ptr_array(dsts)
        keep += [a, b]
        arr[i] = lagom_comm_step(int(op), C.cast(a, C.POINTER(C.c_void_p)), len(srcs), C.cast(b, C.POINTER(C.c_void_p)), len(dsts))
    _check(lib().lagom_comm_steps(dt, arr, len(steps), int(count), C.byref(c), _stream(stream)))


def lagom_gemm(A, B, Cmat, M: int, N: int, K: int, b_is_nk: bool = True, out_dt: int = LAGOM_BF16, stream=None) -> None:
    _check(lib().lagom_gemm(_ptr(A), _ptr(B), _ptr(Cmat), int(M), int(N), int(K), 1 if b_is_nk else 0, out_dt, _stream(stream)))


def lagom_gemm_describe(M: int, N: int, K: int, out_dt: int = LAGOM_BF16) -> lagom_gemm_geometry:
    g = lagom_gemm_geometry()
    _check(lib().lagom_gemm_describe(int(M), int(N), int(K), out_dt, C.byref(g)))
    return g


def lagom_comm_bytes(op: int, dt: int, nsrc: int, ndst: int, count: int) -> int:
    return int(lib().lagom_comm_bytes(op, dt, nsrc, ndst, int(count)))


@dataclass
class CommLaunch:
    op: int
    dtype: int
    srcs: Sequence
    dsts: Sequence
    count: int
    comm_id: int = 0
    after_comp: int = -1        # computation that must have finished before this launch starts
    fuse: bool = False          # issue in the same kernel launch as the previous launch of this communication
    lds_staged: bool = False    # issue through lagom_comm_kernel_lds


@dataclass
class GemmDesc:
    A: object
    B: object
    C: object
    M: int
    N: int
    K: int
    b_is_nk: bool = True
    out_dtype: int = LAGOM_BF16
    after_comm_id: int = -1     # communication that must have finished before this GEMM starts


@dataclass
class Timing:
    X_us: float
    Y_us: float
    Z_us: float
    x_us: List[float]
    y_us: List[float]
    x_mad_us: List[float] = field(default_factory=list)   # spread over the repetitions (median absolute deviation)
    Ysum_us: float = 0.0
    Ysum_mad_us: float = 0.0
    Z_mad_us: float = 0.0
    comm_start_us: float = 0.0                            # common start to the first kernel of either stream
    comp_start_us: float = 0.0


class _Group:
    """C arrays for one overlap group; keeps the pointer arrays alive."""

    def __init__(self, launches: Sequence[CommLaunch], comps: Sequence[GemmDesc]):
        self.keep = []
        self.nlaunch, self.ncomp = len(launches), len(comps)
        self.L = (lagom_comm_desc * max(self.nlaunch, 1))()
        for i, l in enumerate(launches):
            s, d = _ptr_array(l.srcs), _ptr_array(l.dsts)
            self.keep += [s, d]
            self.L[i] = lagom_comm_desc(l.op, l.dtype, C.cast(s, C.POINTER(C.c_void_p)), len(l.srcs),
                                        C.cast(d, C.POINTER(C.c_void_p)), len(l.dsts), int(l.count), int(l.comm_id),
                                        int(l.after_comp), 1 if l.lds_staged else 0, 1 if l.fuse else 0)
        self.G = (lagom_gemm_desc * max(self.ncomp, 1))()
        for i, g in enumerate(comps):
            self.G[i] = lagom_gemm_desc(_ptr(g.A), _ptr(g.B), _ptr(g.C), int(g.M), int(g.N), int(g.K),
                                        1 if g.b_is_nk else 0, int(g.out_dtype), int(g.after_comm_id))


def lagom_streams_overlap(stream_a, stream_b) -> bool:
    out = C.c_int(0)
    _check(lib().lagom_streams_overlap(C.c_void_p(_stream(stream_a)), C.c_void_p(_stream(stream_b)), C.byref(out)))
    return bool(out.value)


def overlapping_streams(tries: int = 8):
    """Two torch streams (default priority) on which kernels run at the same time: new streams are drawn
    until lagom_streams_overlap accepts a pair."""
    import torch
    pool = [torch.cuda.Stream()]
    for _ in range(tries):
        pool.append(torch.cuda.Stream())
        for a in pool[:-1]:
            if lagom_streams_overlap(a, pool[-1]):
                return a, pool[-1]
    raise LagomError(LAGOM_EHIP, "no pair of streams on which kernels overlap (is GPU_MAX_HW_QUEUES 1?)")


def lagom_overlap_run(launches: Sequence[CommLaunch], cfgs: Sequence[CfgLike], comps: Sequence[GemmDesc],
                      comm_stream, comp_stream, warmup: int = 2, iters: int = 10, mode: int = LAGOM_CORUN) -> Timing:
    grp = _Group(launches, comps)
    ncfg = len(cfgs)
    x = (C.c_double * max(ncfg, 1))()
    y = (C.c_double * max(grp.ncomp, 1))()
    xm = (C.c_double * max(ncfg, 1))()
    t = lagom_timing(0.0, 0.0, 0.0, C.cast(x, C.POINTER(C.c_double)), C.cast(y, C.POINTER(C.c_double)),
                     C.cast(xm, C.POINTER(C.c_double)), 0.0, 0.0, 0.0)
    _check(lib().lagom_overlap_run(grp.L, grp.nlaunch, _cfg_array(cfgs), ncfg, grp.G, grp.ncomp,
                                   _stream(comm_stream), _stream(comp_stream), warmup, iters, mode, C.byref(t)))
    return Timing(t.X_us, t.Y_us, t.Z_us, list(x)[:ncfg], list(y)[:grp.ncomp], list(xm)[:ncfg], t.Ysum_us, t.Ysum_mad_us, t.Z_mad_us,
                  t.comm_start_us, t.comp_start_us)


def lagom_overlap_steps(launches: Sequence[CommLaunch], cfgs: Sequence[CfgLike], comps: Sequence[GemmDesc],
                        comm_stream, comp_stream, steps: int) -> float:
    """Device microseconds per repetition of the group over `steps` back-to-back repetitions."""
    return _steps(lib().lagom_overlap_steps, launches, cfgs, comps, comm_stream, comp_stream, steps)


def lagom_overlap_steps_graph(launches: Sequence[CommLaunch], cfgs: Sequence[CfgLike], comps: Sequence[GemmDesc],
                              comm_stream, comp_stream, steps: int) -> float:
    """The same, one repetition captured into a HIP graph and replayed `steps` times."""
    return _steps(lib().lagom_overlap_steps_graph, launches, cfgs, comps, comm_stream, comp_stream, steps)


def _steps(fn, launches, cfgs, comps, comm_stream, comp_stream, steps) -> float:
    grp = _Group(launches, comps)
    out = C.c_double(0.0)
    _check(fn(grp.L, grp.nlaunch, _cfg_array(cfgs), len(cfgs), grp.G, grp.ncomp,
                                     _stream(comm_stream), _stream(comp_stream), int(steps), C.byref(out)))
    return out.value


@dataclass
class SweepPoint:
    cfg: Tuple[int, int, int]
    comm_alone_us: float
    comm_corun_us: float
    comp_alone_us: float
    comp_corun_us: float
    z_corun_us: float
    v_alone: float
    v_corun: float


def lagom_contention_sweep(launches: Sequence[CommLaunch], ncfg: int, comps: Sequence[GemmDesc], points: Sequence[CfgLike],
                           comm_stream, comp_stream, warmup: int = 2, iters: int = 10) -> List[SweepPoint]:
    grp = _Group(launches, comps)
    out = (lagom_sweep_point * len(points))()
    _check(lib().lagom_contention_sweep(grp.L, grp.nlaunch, ncfg, grp.G, grp.ncomp, _cfg_array(points), len(points),
                                        _stream(comm_stream), _stream(comp_stream), warmup, iters, out))
    return [SweepPoint((o.cfg.nc, o.cfg.nt, o.cfg.chunk_bytes), o.comm_alone_us, o.comm_corun_us, o.comp_alone_us,
                       o.comp_corun_us, o.z_corun_us, o.v_alone, o.v_corun) for o in out]


def _sweep_array(points: Sequence["SweepPoint"]):
    arr = (lagom_sweep_point * max(len(points), 1))()
    for i, p in enumerate(points):
        arr[i] = lagom_sweep_point(_cfg(p.cfg), p.comm_alone_us, p.comm_corun_us, p.comp_alone_us, p.comp_corun_us,
                                   p.z_corun_us, p.v_alone, p.v_corun)
    return arr


def _fill_desc(lam, bw_peak, mu, tb, d_bytes, ncomp, comm_bytes, v_cap_frac=0.0):
    cb = (C.c_double * max(len(comm_bytes), 1))(*[float(b) for b in comm_bytes])
    return lagom_fill_desc(int(lam), float(bw_peak), int(mu), int(tb), float(d_bytes), int(ncomp), len(comm_bytes),
                           C.cast(cb, C.POINTER(C.c_double)), float(v_cap_frac)), cb


def _mask(held_out, n):
    if held_out is None:
        return None
    return (C.c_uint8 * max(n, 1))(*[1 if h else 0 for h in held_out])


def lagom_ladder_chunks(chunk_grid: Sequence[int], nc_max: int, nt_ref: int, bytes_per_source: int, kind: int,
                        points: Optional[Sequence["SweepPoint"]] = None) -> List[int]:
    grid = (C.c_int64 * max(len(chunk_grid), 1))(*[int(c) for c in chunk_grid])
    out = (C.c_int64 * max(len(chunk_grid), 1))()
    n = C.c_int32(0)
    pts = _sweep_array(points) if points else None
    _check(lib().lagom_ladder_chunks(grid, len(chunk_grid), int(nc_max), int(nt_ref), int(bytes_per_source), int(kind),
                                     pts, len(points) if points else 0, out, C.byref(n)))
    return list(out)[:n.value]


# ----------------------------------------------------------------- cost model (host)
@dataclass
class CompModel:
    mu: int
    tb: int
    d_bytes: float
    theta_us: float


@dataclass
class Model:
    lam: int
    bw_peak: float                                    # bytes per microsecond
    comps: List[CompModel]
    tables: List[dict] = field(default_factory=list)  # per communication: (nc, nt, chunk) -> (x_us, v)
    comp_after_comm: Optional[Sequence[int]] = None   # per computation: communication it waits for, or -1
    comm_after_comp: Optional[Sequence[int]] = None   # per communication: computation it waits for, or -1
    corun_share: float = 0.0                          # 0 = Eq. 5-6 as printed; see lagom_model in lagom.h
    resident_penalty: dict = field(default_factory=dict)   # NT -> rho; empty = Eq. 6 as printed


@dataclass
class Pred:
    X_us: float
    Y_us: float
    Z_us: float
    x_us: List[float]
    y_us: List[float]
    g: List[List[int]]


class _CModel:
    def __init__(self, m: Model):
        self.comps = (lagom_comp_model * max(len(m.comps), 1))()
        for i, c in enumerate(m.comps):
            self.comps[i] = lagom_comp_model(int(c.mu), int(c.tb), float(c.d_bytes), float(c.theta_us))
        self.entry_arrays = []
        self.tables = (lagom_comm_table * max(len(m.tables), 1))()
        for j, t in enumerate(m.tables):
            arr = (lagom_table_entry * max(len(t), 1))()
            for e, (k, (x, v)) in enumerate(t.items()):
                arr[e] = lagom_table_entry(lagom_cfg(int(k[0]), int(k[1]), int(k[2])), float(x), float(v))
            self.entry_arrays.append(arr)
            self.tables[j] = lagom_comm_table(C.cast(arr, C.POINTER(lagom_table_entry)), len(t))
        self.cac = (C.c_int32 * max(len(m.comps), 1))(*[int(v) for v in m.comp_after_comm]) if m.comp_after_comm is not None else None
        self.cap = (C.c_int32 * max(len(m.tables), 1))(*[int(v) for v in m.comm_after_comp]) if m.comm_after_comp is not None else None
        null = C.POINTER(C.c_int32)()
        pen = list(m.resident_penalty.items())
        self.pen = (lagom_penalty * max(len(pen), 1))(*[lagom_penalty(int(nt), float(rho)) for nt, rho in pen])
        self.c = lagom_model(int(m.lam), float(m.bw_peak), C.cast(self.comps, C.POINTER(lagom_comp_model)), len(m.comps),
                             C.cast(self.tables, C.POINTER(lagom_comm_table)), len(m.tables),
                             C.cast(self.cac, C.POINTER(C.c_int32)) if self.cac is not None else null,
                             C.cast(self.cap, C.POINTER(C.c_int32)) if self.cap is not None else null,
                             float(m.corun_share),
                             C.cast(self.pen, C.POINTER(lagom_penalty)) if pen else C.POINTER(lagom_penalty)(), len(pen))


def lagom_cost_model(model: Model, cfgs: Sequence[CfgLike]) -> Pred:
    cm = _CModel(model)
    n, mcomp = len(cfgs), len(model.comps)
    x = (C.c_double * max(n, 1))()
    y = (C.c_double * max(mcomp, 1))()
    g = (C.c_int32 * max(mcomp * (n + 1), 1))()
    p = lagom_pred(0.0, 0.0, 0.0, C.cast(x, C.POINTER(C.c_double)), C.cast(y, C.POINTER(C.c_double)), C.cast(g, C.POINTER(C.c_int32)))
    _check(lib().lagom_cost_model(C.byref(cm.c), _cfg_array(cfgs), n, C.byref(p)))
    return Pred(p.X_us, p.Y_us, p.Z_us, list(x)[:n], list(y)[:mcomp],
                [[g[i * (n + 1) + s] for s in range(n + 1)] for i in range(mcomp)])


def lagom_model_fill(points: Sequence[SweepPoint], lam: int, bw_peak: float, mu: int, tb: int, d_bytes: float, ncomp: int,
                     comm_bytes: Sequence[float], held_out: Optional[Sequence[bool]] = None, v_cap_frac: float = 0.0,
                     comp_after_comm=None, comm_after_comp=None, corun_share: float = 0.0,
                     resident_penalty: Optional[dict] = None) -> Tuple[Model, float]:
    """The model of one overlap group filled from a sweep; returns (model, t_alone_us)."""
    desc, keep = _fill_desc(lam, bw_peak, mu, tb, d_bytes, ncomp, comm_bytes, v_cap_frac)
    n, ncomm = len(points), len(comm_bytes)
    entries = (lagom_table_entry * max(n * ncomm, 1))()
    tables = (lagom_comm_table * max(ncomm, 1))()
    comps = (lagom_comp_model * max(ncomp, 1))()
    t_alone = C.c_double(0.0)
    _check(lib().lagom_model_fill(_sweep_array(points), n, _mask(held_out, n), C.byref(desc), entries, tables, comps, C.byref(t_alone)))
    py_tables = []
    for j in range(ncomm):
        tj = tables[j]
        py_tables.append({(tj.entries[e].cfg.nc, tj.entries[e].cfg.nt, tj.entries[e].cfg.chunk_bytes): (tj.entries[e].x_us, tj.entries[e].v)
                          for e in range(tj.n)})
    py_comps = [CompModel(c.mu, c.tb, c.d_bytes, c.theta_us) for c in comps[:ncomp]]
    return Model(lam, bw_peak, py_comps, py_tables, comp_after_comm, comm_after_comp, corun_share,
                 dict(resident_penalty) if resident_penalty else {}), t_alone.value


@dataclass
class Calibration:
    sigma: float
    theta_us: float
    fit_mean: float
    fit_max: float
    held_mean: float
    held_max: float
    n_fit: int
    n_held: int
    penalty: Optional[dict] = None      # NT -> rho when candidate rhos were given


def lagom_model_calibrate(points: Sequence[SweepPoint], lam: int, bw_peak: float, mu: int, tb: int, d_bytes: float, ncomp: int,
                          comm_bytes: Sequence[float], sigmas: Sequence[float], held_out: Optional[Sequence[bool]] = None,
                          v_cap_frac: float = 0.0, comp_after_comm=None, comm_after_comp=None,
                          rhos: Optional[Sequence[float]] = None) -> Calibration:
    desc, keep = _fill_desc(lam, bw_peak, mu, tb, d_bytes, ncomp, comm_bytes, v_cap_frac)
    n = len(points)
    cac = (C.c_int32 * max(ncomp, 1))(*[int(v) for v in comp_after_comm]) if comp_after_comm is not None else None
    cap = (C.c_int32 * max(len(comm_bytes), 1))(*[int(v) for v in comm_after_comp]) if comm_after_comp is not None else None
    sg = (C.c_double * max(len(sigmas), 1))(*[float(v) for v in sigmas])
    out = lagom_calibration()
    nrho = len(rhos) if rhos else 0
    rh = (C.c_double * max(nrho, 1))(*[float(v) for v in (rhos or [])])
    room = len(set(int(tuple(p.cfg)[1]) for p in points)) if nrho else 0
    pen = (lagom_penalty * max(room, 1))()
    _check(lib().lagom_model_calibrate(_sweep_array(points), n, _mask(held_out, n), C.byref(desc), cac, cap, sg, len(sigmas),
                                       rh if nrho else None, nrho, pen if nrho else None, room, C.byref(out)))
    penalty = {pen[e].nt: pen[e].rho for e in range(out.npenalty)} if nrho else None
    return Calibration(out.sigma, out.theta_us, out.fit_mean, out.fit_max, out.held_mean, out.held_max, out.n_fit, out.n_held, penalty)


# ------------------------------------------------------------------------ tuner (host)
@dataclass
class Space:
    nc: Sequence[int]
    nt: Sequence[int]
    chunk: Sequence[int]


@dataclass
class TraceStep:
    comm: int
    level_from: int
    level_to: int
    accepted: bool
    done: bool
    xj_prev: float
    xj_new: float
    X: float
    Y: float
    Z: float
    H: float
    lr: float


@dataclass
class TuneResult:
    cfgs: List[Tuple[int, int, int]]
    levels: List[int]
    X: float
    Y: float
    Z: float
    calls: int
    trace: List[TraceStep]
    code: int = LAGOM_OK


@dataclass
class OverlapProfile:
    """Measured ProfileTime: one co-run of the group per call (native callback)."""
    launches: Sequence[CommLaunch]
    comps: Sequence[GemmDesc]
    comm_stream: object
    comp_stream: object
    warmup: int = 1
    iters: int = 5
    min_total_us: float = 0.0      # measure again, longer, when iters * Z stays below this
    max_iters: int = 0
    log_capacity: int = 0          # > 0: record what every call measured; read it back from `.log` after the search
    log: Optional[list] = None     # out: per call {"cfgs", "x", "x_mad", "Y", "Y_mad", "Z", "Z_mad", "iters"}


ProfileLike = Union[Callable[[List[Tuple[int, int, int]]], Tuple[Sequence[float], float]], Model, OverlapProfile]


def lagom_tune(spaces: Sequence[Space], profile: ProfileLike, mode: int = LAGOM_PRIORITY,
               raise_on_callback_error: bool = True) -> TuneResult:
    """`profile` is a Python callable cfgs -> (x list, Y), a ``Model`` (the native cost-model callback is
    used) or an ``OverlapProfile`` (the native measuring callback is used)."""
    L = lib()
    n = len(spaces)
    keep = []
    sp = (lagom_tune_space * max(n, 1))()
    total_levels = 0
    for j, s in enumerate(spaces):
        a = (C.c_int32 * max(len(s.nc), 1))(*[int(v) for v in s.nc])
        b = (C.c_int32 * max(len(s.nt), 1))(*[int(v) for v in s.nt])
        c = (C.c_int64 * max(len(s.chunk), 1))(*[int(v) for v in s.chunk])
        keep += [a, b, c]
        sp[j] = lagom_tune_space(C.cast(a, C.POINTER(C.c_int32)), len(s.nc), C.cast(b, C.POINTER(C.c_int32)), len(s.nt),
                                 C.cast(c, C.POINTER(C.c_int64)), len(s.chunk))
        total_levels += max(len(s.nc), len(s.nt), len(s.chunk))
    cap = total_levels + 2
    steps = (lagom_trace_step * cap)()
    levels = (C.c_int32 * max(n, 1))()
    tr = lagom_trace(C.cast(steps, C.POINTER(lagom_trace_step)), cap, 0, 0, math.nan, math.nan, math.nan,
                     C.cast(levels, C.POINTER(C.c_int32)))
    out = (lagom_cfg * max(n, 1))()

    if isinstance(profile, Model):
        cm = _CModel(profile)
        keep.append(cm)
        fn, user = C.cast(L.lagom_model_profile, C.c_void_p), C.cast(C.pointer(cm.c), C.c_void_p)
    elif isinstance(profile, OverlapProfile):
        grp = _Group(profile.launches, profile.comps)
        plog, plog_arrays = None, None
        if profile.log_capacity > 0:
            cap_l = int(profile.log_capacity)
            plog_arrays = {"cfgs": (lagom_cfg * (cap_l * n))(), "x": (C.c_double * (cap_l * n))(), "x_mad": (C.c_double * (cap_l * n))(),
                           "Y": (C.c_double * cap_l)(), "Y_mad": (C.c_double * cap_l)(), "Z": (C.c_double * cap_l)(),
                           "Z_mad": (C.c_double * cap_l)(), "iters": (C.c_int32 * cap_l)()}
            a = plog_arrays
            plog = lagom_profile_log(cap_l, n, 0, C.cast(a["cfgs"], C.POINTER(lagom_cfg)), C.cast(a["x"], C.POINTER(C.c_double)),
                                     C.cast(a["x_mad"], C.POINTER(C.c_double)), C.cast(a["Y"], C.POINTER(C.c_double)),
                                     C.cast(a["Y_mad"], C.POINTER(C.c_double)), C.cast(a["Z"], C.POINTER(C.c_double)),
                                     C.cast(a["Z_mad"], C.POINTER(C.c_double)), C.cast(a["iters"], C.POINTER(C.c_int32)))
        ctx = lagom_overlap_ctx(C.cast(grp.L, C.POINTER(lagom_comm_desc)), grp.nlaunch,
                                C.cast(grp.G, C.POINTER(lagom_gemm_desc)), grp.ncomp,
                                _stream(profile.comm_stream), _stream(profile.comp_stream), profile.warmup, profile.iters,
                                float(profile.min_total_us), int(profile.max_iters),
                                C.pointer(plog) if plog is not None else C.POINTER(lagom_profile_log)())
        keep += [grp, ctx, plog, plog_arrays]
        fn, user = C.cast(L.lagom_overlap_profile, C.c_void_p), C.cast(C.pointer(ctx), C.c_void_p)
    else:
        def _cb(_user, cfgs, ncomm, x_out, y_out):
            try:
                x, Y = profile([(cfgs[i].nc, cfgs[i].nt, cfgs[i].chunk_bytes) for i in range(ncomm)])
                for i in range(ncomm):
                    x_out[i] = float(x[i])
                y_out[0] = float(Y)
                return 0
            except Exception:
                return 1
        cb = PROFILE_FN(_cb)
        keep.append(cb)
        fn, user = C.cast(cb, C.c_void_p), None
    rc = L.lagom_tune(sp, n, fn, user, mode, out, C.byref(tr))
    if isinstance(profile, OverlapProfile) and profile.log_capacity > 0:
        a = plog_arrays
        profile.log = [{"cfgs": [(a["cfgs"][k * n + j].nc, a["cfgs"][k * n + j].nt, a["cfgs"][k * n + j].chunk_bytes) for j in range(n)],
                        "x": [a["x"][k * n + j] for j in range(n)], "x_mad": [a["x_mad"][k * n + j] for j in range(n)],
                        "Y": a["Y"][k], "Y_mad": a["Y_mad"][k], "Z": a["Z"][k], "Z_mad": a["Z_mad"][k], "iters": a["iters"][k]}
                       for k in range(min(plog.n, plog.capacity))]
    if rc != LAGOM_OK and not (rc == LAGOM_ECALLBACK and not raise_on_callback_error):
        _check(rc)
    trace = [TraceStep(s.comm, s.level_from, s.level_to, bool(s.accepted), bool(s.done), s.xj_prev, s.xj_new,
                       s.X, s.Y, s.Z, s.H, s.lr) for s in steps[:tr.n]]
    return TuneResult([(o.nc, o.nt, o.chunk_bytes) for o in out[:n]], list(levels)[:n], tr.X, tr.Y, tr.Z, tr.calls, trace, rc)
