"""CPU oracle for rooted broadcast schedules -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``bcast_oracle.c`` (plain C, compiled with gcc).
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the GPU library never does, and this package never imports it.

Buffers are a C-contiguous ``numpy.uint8`` array of shape ``[P, capacity]``:
row r is rank r's buffer.  Functions modify it in place and return counts
(and, on request, a trace of every transfer the schedule performed).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from pathlib import Path
from typing import List, Optional

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "bcast_oracle.c"
_HDR = _HERE / "bcast_oracle.h"
_LIB = _HERE / "libbcast_oracle.so"


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, no GPU toolchain involved)."""
    stale = (not _LIB.exists()) or _LIB.stat().st_mtime < max(_SRC.stat().st_mtime, _HDR.stat().st_mtime)
    if force or stale:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", str(_SRC), "-o", str(tmp)]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Xfer(ctypes.Structure):
    _fields_ = [
        ("step", ctypes.c_long),
        ("src_rank", ctypes.c_int),
        ("dst_rank", ctypes.c_int),
        ("chunk", ctypes.c_long),
        ("lo", ctypes.c_ulonglong),
        ("hi", ctypes.c_ulonglong),
    ]


class _Trace(ctypes.Structure):
    _fields_ = [
        ("xfers", ctypes.POINTER(_Xfer)),
        ("xfers_cap", ctypes.c_size_t),
        ("xfers_len", ctypes.c_size_t),
        ("have", ctypes.POINTER(ctypes.c_long)),
        ("have_cap_steps", ctypes.c_size_t),
        ("bytes_copied", ctypes.c_ulonglong),
    ]


@dataclass
class Transfer:
    step: int
    src_rank: int
    dst_rank: int
    chunk: int
    lo: int
    hi: int


@dataclass
class Result:
    """What a schedule did: its step/round/send count and, if traced, details."""

    steps: int
    bytes_copied: int = 0
    transfers: Optional[List[Transfer]] = None
    have: Optional[np.ndarray] = None  # [steps, P] chunks held per chain position after each step
    scatter_rounds: int = 0
    ring_steps: int = 0


_lib = None


def _bind(path):
    """Load one build of the oracle and declare its signatures."""
    lib = ctypes.CDLL(str(path))
    pp = ctypes.POINTER(ctypes.c_void_p)
    tp = ctypes.POINTER(_Trace)
    lib.oracle_naive_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t]
    lib.oracle_naive_bcast.restype = ctypes.c_int
    lib.oracle_chain_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t, tp]
    lib.oracle_chain_bcast.restype = ctypes.c_long
    lib.oracle_direct_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, tp]
    lib.oracle_direct_bcast.restype = ctypes.c_long
    lib.oracle_binomial_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, tp]
    lib.oracle_binomial_bcast.restype = ctypes.c_long
    lib.oracle_knomial_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, tp]
    lib.oracle_knomial_bcast.restype = ctypes.c_long
    lib.oracle_knomial_pipeline_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, tp]
    lib.oracle_knomial_pipeline_bcast.restype = ctypes.c_long
    lib.oracle_chain_reduce_f32.argtypes = [pp, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t, tp]
    lib.oracle_chain_reduce_f32.restype = ctypes.c_long
    lp = ctypes.POINTER(ctypes.c_long)
    lib.oracle_scatter_allgather_bcast.argtypes = [pp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t, lp, lp, tp]
    lib.oracle_scatter_allgather_bcast.restype = ctypes.c_long
    d = ctypes.c_double
    lib.oracle_model_direct.argtypes = [ctypes.c_int, d, d, d]
    lib.oracle_model_chain.argtypes = [ctypes.c_int, d, d, d]
    lib.oracle_model_knomial.argtypes = [ctypes.c_int, ctypes.c_int, d, d, d]
    lib.oracle_model_scatter_allgather.argtypes = [ctypes.c_int, d, d, d]
    lib.oracle_model_chain_pipeline.argtypes = [ctypes.c_int, d, d, d, d]
    lib.oracle_model_knomial_pipeline.argtypes = [ctypes.c_int, ctypes.c_int, d, d, d, d]
    for n in ("direct", "chain", "knomial", "scatter_allgather", "chain_pipeline", "knomial_pipeline"):
        getattr(lib, "oracle_model_" + n).restype = d
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def use_library(path) -> None:
    """Point this module at another build of the oracle (tests use this to
    check that the pins reject deliberately broken variants); None restores
    the regular build."""
    global _lib
    _lib = None if path is None else _bind(path)


def _row_pointers(bufs: Optional[np.ndarray], P: int, M: int):
    if bufs is None:
        return None
    if not (isinstance(bufs, np.ndarray) and bufs.dtype == np.uint8 and bufs.ndim == 2):
        raise TypeError("bufs must be a 2-D numpy uint8 array [P, capacity]")
    if not bufs.flags.c_contiguous or not bufs.flags.writeable:
        raise ValueError("bufs must be C-contiguous and writeable")
    if bufs.shape[0] != P or bufs.shape[1] < M:
        raise ValueError("bufs has shape %r, need [%d, >=%d]" % (bufs.shape, P, M))
    base = bufs.ctypes.data
    stride = bufs.strides[0]
    return (ctypes.c_void_p * P)(*[base + r * stride for r in range(P)])


class _TraceBuf:
    def __init__(self, P: int, want: bool, max_xfers: int, max_steps: int):
        self.c = _Trace()
        self.P = P
        self.want = want
        if want:
            self.x = (_Xfer * max(1, max_xfers))()
            self.h = np.zeros((max(1, max_steps), P), dtype=np.int64)
            assert ctypes.sizeof(ctypes.c_long) == 8
            self.c.xfers = ctypes.cast(self.x, ctypes.POINTER(_Xfer))
            self.c.xfers_cap = max_xfers
            self.c.have = self.h.ctypes.data_as(ctypes.POINTER(ctypes.c_long))
            self.c.have_cap_steps = max_steps

    def result(self, steps: int, with_have: bool = False) -> Result:
        res = Result(steps=int(steps), bytes_copied=int(self.c.bytes_copied))
        if self.want:
            n = min(int(self.c.xfers_len), int(self.c.xfers_cap))
            res.transfers = [
                Transfer(x.step, x.src_rank, x.dst_rank, x.chunk, x.lo, x.hi) for x in self.x[:n]
            ]
            if with_have:
                res.have = self.h[: max(0, steps)].copy()
        return res


def _check(rc: int, what: str) -> int:
    if rc < 0:
        raise ValueError("%s: bad arguments" % what)
    return rc


def naive_bcast(bufs: np.ndarray, root: int, M: int) -> None:
    """Every non-root row's first M bytes become the root row's (the definition)."""
    P = bufs.shape[0]
    _check(_load().oracle_naive_bcast(_row_pointers(bufs, P, M), P, root, M), "naive_bcast")


def chain_bcast(bufs: Optional[np.ndarray], P: int, root: int, M: int, C: int, trace: bool = False) -> Result:
    """Pipelined chain (paper Sec. IV-B, Eq. 5); ``bufs=None`` walks the schedule only."""
    nchunks = -(-M // C) if C > 0 else 0
    tb = _TraceBuf(P, trace, nchunks * max(0, P - 1), nchunks + P)
    steps = _check(_load().oracle_chain_bcast(_row_pointers(bufs, P, M), P, root, M, C, ctypes.byref(tb.c)), "chain_bcast")
    return tb.result(steps, with_have=True)


def direct_bcast(bufs: Optional[np.ndarray], P: int, root: int, M: int, trace: bool = False) -> Result:
    """Direct algorithm (Sec. III-A, Eq. 1): root sends to every other rank in turn."""
    tb = _TraceBuf(P, trace, P, 1)
    n = _check(_load().oracle_direct_bcast(_row_pointers(bufs, P, M), P, root, M, ctypes.byref(tb.c)), "direct_bcast")
    return tb.result(n)


def binomial_bcast(bufs: Optional[np.ndarray], P: int, root: int, M: int, trace: bool = False) -> Result:
    """Binomial tree (Sec. III-A, Eq. 3 with k = 2)."""
    tb = _TraceBuf(P, trace, P, 1)
    n = _check(_load().oracle_binomial_bcast(_row_pointers(bufs, P, M), P, root, M, ctypes.byref(tb.c)), "binomial_bcast")
    return tb.result(n)


def knomial_bcast(bufs: Optional[np.ndarray], P: int, root: int, M: int, k: int, trace: bool = False) -> Result:
    """K-nomial tree (Sec. III-A, Eq. 3) with radix k."""
    tb = _TraceBuf(P, trace, P, 1)
    n = _check(_load().oracle_knomial_bcast(_row_pointers(bufs, P, M), P, root, M, k, ctypes.byref(tb.c)), "knomial_bcast")
    return tb.result(n)


def knomial_pipeline_bcast(bufs: Optional[np.ndarray], P: int, root: int, M: int, C: int, k: int, trace: bool = False) -> Result:
    """Pipelined k-nomial tree: the levels of Eq. 3, chunk by chunk (Sec. IV-B)."""
    nchunks = -(-M // C) if C > 0 else 0
    tb = _TraceBuf(P, trace, nchunks * max(0, P - 1), 1)
    n = _check(_load().oracle_knomial_pipeline_bcast(_row_pointers(bufs, P, M), P, root, M, C, k, ctypes.byref(tb.c)),
               "knomial_pipeline_bcast")
    return tb.result(n)


def chain_reduce_f32(send: Optional[np.ndarray], P: int, root: int, count: int, chunk_elems: int, trace: bool = False):
    """Pipelined chain reduction (fp32 sum) in chain order; ``send`` is a
    C-contiguous float32 array [P, count] (row r = rank r's contribution) or
    None for the schedule only.  Returns (recv, Result)."""
    nchunks = -(-count // chunk_elems) if chunk_elems > 0 else 0
    tb = _TraceBuf(P, trace, nchunks * max(0, P - 1), 1)
    recv = None
    if send is not None:
        assert send.dtype == np.float32 and send.flags["C_CONTIGUOUS"] and send.shape == (P, count)
        rows = (ctypes.c_void_p * P)(*[send.ctypes.data + r * send.strides[0] for r in range(P)])
        recv = np.empty(count, dtype=np.float32)
        n = _load().oracle_chain_reduce_f32(rows, recv.ctypes.data, P, root, count, chunk_elems, ctypes.byref(tb.c))
    else:
        n = _load().oracle_chain_reduce_f32(None, None, P, root, count, chunk_elems, ctypes.byref(tb.c))
    return recv, tb.result(_check(n, "chain_reduce_f32"))


def scatter_allgather_bcast(bufs: Optional[np.ndarray], P: int, root: int, M: int, trace: bool = False) -> Result:
    """Binomial scatter + ring allgather (Sec. III-A, Eq. 4)."""
    tb = _TraceBuf(P, trace, P * P + P, 1)
    sr = ctypes.c_long(0)
    rs = ctypes.c_long(0)
    n = _check(
        _load().oracle_scatter_allgather_bcast(
            _row_pointers(bufs, P, M), P, root, M, ctypes.byref(sr), ctypes.byref(rs), ctypes.byref(tb.c)
        ),
        "scatter_allgather_bcast",
    )
    res = tb.result(n)
    res.scatter_rounds = sr.value
    res.ring_steps = rs.value
    return res


def model_direct(n, M, ts, B):
    return _load().oracle_model_direct(n, M, ts, B)


def model_chain(n, M, ts, B):
    return _load().oracle_model_chain(n, M, ts, B)


def model_knomial(n, k, M, ts, B):
    return _load().oracle_model_knomial(n, k, M, ts, B)


def model_knomial_pipeline(n, k, M, C, ts, B):
    return _load().oracle_model_knomial_pipeline(n, k, M, C, ts, B)


def model_scatter_allgather(n, M, ts, B):
    return _load().oracle_model_scatter_allgather(n, M, ts, B)


def model_chain_pipeline(n, M, C, ts, B):
    return _load().oracle_model_chain_pipeline(n, M, C, ts, B)
