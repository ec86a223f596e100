"""ctypes binding for the gfx950 broadcast library (``lib/libbcast.so``).

Argument marshalling only: every byte is moved by the library's HIP kernels.
Function names and argument order follow ``include/bcast.h`` and
``include/bcast_debug.h``.  Buffers may be
given as integers (device addresses) or as objects with ``data_ptr()`` (torch
tensors); streams as integers (``torch.cuda.current_stream().cuda_stream``),
objects with ``cuda_stream``, or None for the default stream.

There is no CPU fallback: if the shared library is missing, importing this
module raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Sequence, Tuple

LIB_PATH = Path(__file__).resolve().parent / "lib" / "libbcast.so"

BCAST_MAX_RANKS = 64

BCAST_ALGO_AUTO = 0
BCAST_ALGO_CHAIN = 1
BCAST_ALGO_DIRECT = 2
BCAST_ALGO_BINOMIAL = 3
BCAST_ALGO_FANOUT = 4
BCAST_ALGO_SCATTER_ALLGATHER = 5
BCAST_ALGO_KNOMIAL = 6
BCAST_ALGO_KNOMIAL_PIPELINED = 7
ALGO_NAMES = {0: "auto", 1: "chain", 2: "direct", 3: "binomial", 4: "fanout", 5: "scatter_allgather", 6: "knomial", 7: "knomial_pipelined"}

BCAST_OK = 0
BCAST_ERR_ARG = -1
BCAST_ERR_NOMEM = -2
BCAST_ERR_HIP = -3
BCAST_ERR_TIMEOUT = -4
BCAST_ERR_UNTUNED = -5
BCAST_ERR_CAPACITY = -6

# every symbol include/bcast.h and include/bcast_debug.h declare
EXPORTS = [
    "bcast_plan_create", "bcast_run", "bcast_plan_status", "bcast_plan_clear_status", "bcast_plan_info",
    "bcast_plan_destroy", "bcast_plan_set_lanes", "bcast_plan_set_stages", "bcast_plan_set_trip", "bcast_plan_set_block_threads", "bcast_plan_set_radix", "bcast_plan_set_debug", "bcast_plan_debug_set_epoch", "bcast_chain_stage_span", "bcast_reduce_sum_f32", "bcast_reduce_sum_f32_static", "bcast_plan_reserve_reduce", "bcast_allreduce_sum_f32", "bcast_reduce_info", "bcast_plan_set_mode", "bcast_plan_enable_trace", "bcast_plan_read_trace",
    "bcast_plan_handoff_counts", "bcast_plan_set_cache_policy", "bcast_plan_set_chain_waves", "bcast_plan_set_rank_handoff", "bcast_plan_set_stage_store", "bcast_plan_set_replayable", "bcast_memory_regions", "bcast_buffers_alloc", "bcast_buffers_free", "bcast_chain_geometry",
    "bcast_tune", "bcast_tune_load", "bcast_tune_save", "bcast_tune_clear", "bcast_tune_set",
    "bcast_tune_lookup", "bcast_tune_set_log", "bcast_tune_put", "bcast_tune_get", "bcast_tune_count", "bcast_tune_reduce", "bcast_tune_reduce_put", "bcast_tune_reduce_get", "bcast_plan_set_reduce_trip", "bcast_debug_store_pattern", "bcast_debug_load_pattern", "bcast_strerror", "bcast_last_hip_error", "bcast_version",
]


class BcastError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = "%s: %s (status %d)" % (what, _lib.bcast_strerror(status).decode(), status)
        if status == BCAST_ERR_HIP:
            msg += ", hipError %d" % _lib.bcast_last_hip_error()
        super().__init__(msg)


class ChainRequest(ctypes.Structure):
    _fields_ = [("lanes", ctypes.c_int), ("stages", ctypes.c_int), ("trip_bytes", ctypes.c_int), ("block_threads", ctypes.c_int)]


class PlanInfo(ctypes.Structure):
    _fields_ = [
        ("algo", ctypes.c_int),
        ("chunk_bytes", ctypes.c_uint64),
        ("nchunks", ctypes.c_uint64),
        ("stages", ctypes.c_int),
        ("hops_per_stage", ctypes.c_int),
        ("lanes", ctypes.c_int),
        ("rotating_spans", ctypes.c_int),
        ("trip_bytes", ctypes.c_int),
        ("slice_bytes", ctypes.c_uint64),
        ("grid_blocks", ctypes.c_int),
        ("block_threads", ctypes.c_int),
        ("vec_bytes", ctypes.c_int),
        ("launches", ctypes.c_int),
        ("algorithmic_bytes", ctypes.c_uint64),
        ("rank_waves", ctypes.c_int),
        ("stage_store", ctypes.c_int),
        ("rank_handoff", ctypes.c_int),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class TuneEntry(ctypes.Structure):
    _fields_ = [
        ("algo", ctypes.c_int),
        ("chunk_bytes", ctypes.c_uint64),
        ("stages", ctypes.c_int),
        ("trip_bytes", ctypes.c_int),
        ("usec", ctypes.c_double),
        ("chain_chunk_bytes", ctypes.c_uint64),
        ("chain_stages", ctypes.c_int),
        ("chain_trip_bytes", ctypes.c_int),
        ("chain_usec", ctypes.c_double),
        ("rank_waves", ctypes.c_int),
        ("chain_rank_waves", ctypes.c_int),
        ("stage_store", ctypes.c_int),
        ("chain_stage_store", ctypes.c_int),
        ("lanes", ctypes.c_int),
        ("chain_lanes", ctypes.c_int),
        ("spans", ctypes.c_int),
        ("chain_spans", ctypes.c_int),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class ReduceEntry(ctypes.Structure):
    _fields_ = [("chunk_bytes", ctypes.c_uint64), ("stages", ctypes.c_int), ("trip_bytes", ctypes.c_int), ("usec", ctypes.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


BCAST_TUNE_FOLDED = 1 << 16
BCAST_TUNE_NO_RANK_WAVES = 1 << 17


def _load():
    if not LIB_PATH.exists():
        raise ImportError(
            "%s is missing: build it with `python -m paper_1707_09414_amd.build` "
            "(there is no CPU fallback)" % LIB_PATH
        )
    lib = ctypes.CDLL(str(LIB_PATH))
    vp, i, sz, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_uint64
    pvp = ctypes.POINTER(ctypes.c_void_p)
    sigs = {
        "bcast_plan_create": ([pvp, i, sz, sz, i], i),
        "bcast_run": ([vp, pvp, i, sz, vp], i),
        "bcast_plan_status": ([vp, ctypes.POINTER(u64)], i),
        "bcast_plan_clear_status": ([vp], i),
        "bcast_plan_info": ([vp, pvp, sz, ctypes.POINTER(PlanInfo)], i),
        "bcast_plan_destroy": ([vp], i),
        "bcast_plan_set_lanes": ([vp, i], i),
        "bcast_plan_set_stages": ([vp, i], i),
        "bcast_plan_set_radix": ([vp, i], i),
        "bcast_plan_set_trip": ([vp, i], i),
        "bcast_reduce_sum_f32": ([vp, ctypes.POINTER(ctypes.c_void_p), vp, i, sz, vp], i),
        "bcast_reduce_info": ([vp, sz, ctypes.POINTER(PlanInfo)], i),
        "bcast_reduce_sum_f32_static": ([vp, ctypes.POINTER(ctypes.c_void_p), vp, i, sz, vp], i),
        "bcast_plan_reserve_reduce": ([vp, sz, i], i),
        "bcast_allreduce_sum_f32": ([vp, ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p), i, sz, vp], i),
        "bcast_chain_stage_span": ([i, i, i, ctypes.c_uint64, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)], i),
        "bcast_plan_debug_set_epoch": ([vp, ctypes.c_uint64], i),
        "bcast_plan_set_block_threads": ([vp, i], i),
        "bcast_plan_set_debug": ([vp, u64, i], i),
        "bcast_plan_set_mode": ([vp, ctypes.c_uint], i),
        "bcast_plan_set_cache_policy": ([vp, i, i, i, i], i),
        "bcast_plan_set_chain_waves": ([vp, i], i),
        "bcast_plan_set_rank_handoff": ([vp, i], i),
        "bcast_plan_set_replayable": ([vp, i], i),
        "bcast_plan_set_stage_store": ([vp, i], i),
        "bcast_memory_regions": ([ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_size_t)], i),
        "bcast_buffers_alloc": ([i, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_void_p),
                                ctypes.POINTER(ctypes.c_int)], i),
        "bcast_buffers_free": ([i, ctypes.POINTER(ctypes.c_void_p)], i),
        "bcast_plan_enable_trace": ([vp, sz], i),
        "bcast_plan_read_trace": ([vp, ctypes.POINTER(u64), sz], i),
        "bcast_plan_handoff_counts": ([vp, ctypes.POINTER(u64), ctypes.POINTER(u64)], i),
        "bcast_chain_geometry": ([i, sz, sz, i, ctypes.POINTER(ChainRequest), ctypes.POINTER(PlanInfo)], i),
        "bcast_tune": ([i, sz, sz, ctypes.c_uint, vp, ctypes.c_char_p], i),
        "bcast_tune_load": ([ctypes.c_char_p], i),
        "bcast_tune_save": ([ctypes.c_char_p], i),
        "bcast_tune_clear": ([], i),
        "bcast_tune_set": ([i, sz, i, sz, ctypes.c_double], i),
        "bcast_tune_lookup": ([i, sz, ctypes.POINTER(i), ctypes.POINTER(sz), ctypes.POINTER(ctypes.c_double)], i),
        "bcast_tune_set_log": ([ctypes.c_char_p], i),
        "bcast_tune_put": ([i, sz, ctypes.POINTER(TuneEntry)], i),
        "bcast_tune_get": ([i, sz, ctypes.POINTER(TuneEntry)], i),
        "bcast_tune_count": ([], i),
        "bcast_tune_reduce": ([i, sz, sz, vp, ctypes.c_char_p], i),
        "bcast_tune_reduce_put": ([i, sz, ctypes.POINTER(ReduceEntry)], i),
        "bcast_tune_reduce_get": ([i, sz, ctypes.POINTER(ReduceEntry)], i),
        "bcast_plan_set_reduce_trip": ([vp, i], i),
        "bcast_debug_store_pattern": ([pvp, i, sz, vp], i),
        "bcast_debug_load_pattern": ([pvp, i, sz, vp, i, vp], i),
        "bcast_strerror": ([i], ctypes.c_char_p),
        "bcast_last_hip_error": ([], i),
        "bcast_version": ([], ctypes.c_char_p),
    }
    for name, (args, res) in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = res
    return lib


_lib = _load()


def _check(status: int, what: str) -> None:
    if status != BCAST_OK:
        raise BcastError(status, what)


def _ptr(x) -> int:
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    return int(s.cuda_stream) if hasattr(s, "cuda_stream") else int(s)


class RankPointers:
    """The rank buffers' device addresses in the C array ``bcast_run`` takes.
    Building it costs more than a small broadcast takes, so a caller that
    broadcasts into the same buffers many times builds it once and passes it in
    place of the buffer list.  It keeps the buffers alive."""

    def __init__(self, rank_bufs: Sequence):
        self.bufs = list(rank_bufs)
        self.array = (ctypes.c_void_p * len(self.bufs))(*[_ptr(b) for b in self.bufs])

    def __len__(self) -> int:
        return len(self.bufs)


def _ptr_array(rank_bufs):
    if isinstance(rank_bufs, RankPointers):
        return rank_bufs.array
    return (ctypes.c_void_p * len(rank_bufs))(*[_ptr(b) for b in rank_bufs])


class Plan:
    """Owner of one ``bcast_plan_t``; destroyed explicitly or when collected."""

    def __init__(self, handle: int, nranks: int, bytes_: int, chunk_bytes: int, algo: int):
        self.handle = handle
        self.nranks = nranks
        self.bytes = bytes_
        self.chunk_bytes = chunk_bytes
        self.algo = algo

    def destroy(self) -> None:
        if self.handle:
            h, self.handle = self.handle, None
            _check(_lib.bcast_plan_destroy(h), "bcast_plan_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()


def bcast_plan_create(nranks: int, bytes: int, chunk_bytes: int = 0, algo: int = BCAST_ALGO_CHAIN) -> Plan:
    out = ctypes.c_void_p()
    _check(_lib.bcast_plan_create(ctypes.byref(out), nranks, bytes, chunk_bytes, algo), "bcast_plan_create")
    return Plan(out.value, nranks, bytes, chunk_bytes, algo)


def bcast_run(plan: Plan, rank_bufs: Sequence, root: int, bytes: int, stream=None) -> None:
    if len(rank_bufs) != plan.nranks:
        raise BcastError(BCAST_ERR_ARG, "bcast_run: need %d buffers, got %d" % (plan.nranks, len(rank_bufs)))
    _check(_lib.bcast_run(plan.handle, _ptr_array(rank_bufs), root, bytes, _stream(stream)), "bcast_run")


def bcast_run_status(plan: Plan, rank_bufs: Sequence, root: int, bytes: int, stream=None) -> int:
    """Like bcast_run but returns the status code instead of raising."""
    arr = _ptr_array(rank_bufs) if rank_bufs is not None else None
    return _lib.bcast_run(plan.handle, arr, root, bytes, _stream(stream))


def bcast_plan_status(plan: Plan) -> Tuple[int, int]:
    """(status, detail): detail is hop << 32 | chunk of the first wave that gave up."""
    d = ctypes.c_uint64(0)
    return _lib.bcast_plan_status(plan.handle, ctypes.byref(d)), d.value


def bcast_plan_clear_status(plan: Plan) -> None:
    _check(_lib.bcast_plan_clear_status(plan.handle), "bcast_plan_clear_status")


def bcast_plan_info(plan: Plan, bytes: int, rank_bufs: Optional[Sequence] = None) -> dict:
    info = PlanInfo()
    arr = _ptr_array(rank_bufs) if rank_bufs is not None else None
    _check(_lib.bcast_plan_info(plan.handle, arr, bytes, ctypes.byref(info)), "bcast_plan_info")
    return info.as_dict()


def bcast_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def bcast_plan_set_lanes(plan: Plan, lanes: int) -> None:
    _check(_lib.bcast_plan_set_lanes(plan.handle, lanes), "bcast_plan_set_lanes")


def bcast_plan_set_stages(plan: Plan, stages: int) -> None:
    _check(_lib.bcast_plan_set_stages(plan.handle, stages), "bcast_plan_set_stages")


def bcast_plan_set_trip(plan: Plan, trip_bytes: int) -> None:
    _check(_lib.bcast_plan_set_trip(plan.handle, trip_bytes), "bcast_plan_set_trip")


def bcast_plan_set_block_threads(plan: Plan, block_threads: int) -> None:
    _check(_lib.bcast_plan_set_block_threads(plan.handle, block_threads), "bcast_plan_set_block_threads")


def bcast_reduce_sum_f32(plan: Plan, send_bufs, recv_buf, root: int, count: int, stream=None) -> None:
    if len(send_bufs) != plan.nranks:
        raise BcastError(BCAST_ERR_ARG, "bcast_reduce_sum_f32: need %d buffers, got %d" % (plan.nranks, len(send_bufs)))
    _check(_lib.bcast_reduce_sum_f32(plan.handle, _ptr_array(send_bufs), _ptr(recv_buf), root, count, _stream(stream)),
           "bcast_reduce_sum_f32")


def bcast_reduce_sum_f32_static(plan: Plan, send_bufs, recv_buf, root: int, count: int, stream=None) -> None:
    if len(send_bufs) != plan.nranks:
        raise BcastError(BCAST_ERR_ARG, "bcast_reduce_sum_f32_static: need %d buffers, got %d" % (plan.nranks, len(send_bufs)))
    _check(_lib.bcast_reduce_sum_f32_static(plan.handle, _ptr_array(send_bufs), _ptr(recv_buf), root, count, _stream(stream)),
           "bcast_reduce_sum_f32_static")


def bcast_reduce_static_status(plan: Plan, send_bufs, recv_buf, root: int, count: int, stream=None) -> int:
    """Like bcast_reduce_sum_f32_static but returns the status code instead of raising."""
    return _lib.bcast_reduce_sum_f32_static(plan.handle, _ptr_array(send_bufs), _ptr(recv_buf), root, count, _stream(stream))


def bcast_plan_reserve_reduce(plan: Plan, count: int, stages: int) -> None:
    _check(_lib.bcast_plan_reserve_reduce(plan.handle, count, stages), "bcast_plan_reserve_reduce")


def bcast_allreduce_sum_f32(plan: Plan, send_bufs, recv_bufs, root: int, count: int, stream=None) -> None:
    if len(send_bufs) != plan.nranks or len(recv_bufs) != plan.nranks:
        raise BcastError(BCAST_ERR_ARG, "bcast_allreduce_sum_f32: need %d buffers each" % plan.nranks)
    _check(_lib.bcast_allreduce_sum_f32(plan.handle, _ptr_array(send_bufs), _ptr_array(recv_bufs), root, count, _stream(stream)),
           "bcast_allreduce_sum_f32")


def bcast_reduce_status(plan: Plan, send_bufs, recv_buf, root: int, count: int, stream=None) -> int:
    """Like bcast_reduce_sum_f32 but returns the status code instead of raising."""
    arr = _ptr_array(send_bufs) if send_bufs is not None else None
    return _lib.bcast_reduce_sum_f32(plan.handle, arr, _ptr(recv_buf) if recv_buf is not None else None, root, count, _stream(stream))


def bcast_reduce_info(plan: Plan, count: int) -> dict:
    info = PlanInfo()
    _check(_lib.bcast_reduce_info(plan.handle, count, ctypes.byref(info)), "bcast_reduce_info")
    return info.as_dict()


def bcast_chain_stage_span(nranks: int, stages: int, stage: int, chunk: int) -> Tuple[int, int]:
    """(first_hop, last_hop) that `stage` plays for chunk number `chunk`."""
    first, last = ctypes.c_int(0), ctypes.c_int(0)
    _check(_lib.bcast_chain_stage_span(nranks, stages, stage, chunk, ctypes.byref(first), ctypes.byref(last)),
           "bcast_chain_stage_span")
    return first.value, last.value


def bcast_plan_debug_set_epoch(plan: Plan, epoch: int) -> None:
    _check(_lib.bcast_plan_debug_set_epoch(plan.handle, epoch), "bcast_plan_debug_set_epoch")


def bcast_plan_set_radix(plan: Plan, radix: int) -> None:
    _check(_lib.bcast_plan_set_radix(plan.handle, radix), "bcast_plan_set_radix")


def bcast_plan_set_debug(plan: Plan, spin_limit_ticks: int, mute_hop: int) -> None:
    _check(_lib.bcast_plan_set_debug(plan.handle, spin_limit_ticks, mute_hop), "bcast_plan_set_debug")


BCAST_MODE_COUNT = 2
BCAST_MODE_FIXED_SPANS = 16
BCAST_MODE_ROTATE_SPANS = 32


def bcast_plan_set_mode(plan: Plan, mode: int) -> None:
    _check(_lib.bcast_plan_set_mode(plan.handle, mode), "bcast_plan_set_mode")


BCAST_CACHE_STREAM = 2
BCAST_CACHE_AGENT = 16


def bcast_plan_set_cache_policy(plan: Plan, ld_root: int = -1, ld_edge: int = -1, ld_back: int = -1, st_mid: int = -1) -> None:
    _check(_lib.bcast_plan_set_cache_policy(plan.handle, ld_root, ld_edge, ld_back, st_mid), "bcast_plan_set_cache_policy")


BCAST_CHAIN_AUTO = 0
BCAST_CHAIN_WAVE_PER_STAGE = 1
BCAST_CHAIN_WAVE_PER_RANK = 2


def bcast_plan_set_chain_waves(plan: Plan, mode: int) -> None:
    _check(_lib.bcast_plan_set_chain_waves(plan.handle, mode), "bcast_plan_set_chain_waves")


BCAST_HANDOFF_AUTO, BCAST_HANDOFF_CACHE, BCAST_HANDOFF_LDS = 0, 1, 2


def bcast_plan_set_rank_handoff(plan: Plan, mode: int) -> None:
    _check(_lib.bcast_plan_set_rank_handoff(plan.handle, mode), "bcast_plan_set_rank_handoff")


BCAST_STORE_AUTO, BCAST_STORE_THROUGH, BCAST_STORE_BACK = 0, 1, 2
BCAST_SPANS_AUTO, BCAST_SPANS_FIXED, BCAST_SPANS_ROTATE = 0, 1, 2


def bcast_plan_set_stage_store(plan: Plan, mode: int) -> None:
    _check(_lib.bcast_plan_set_stage_store(plan.handle, mode), "bcast_plan_set_stage_store")


BCAST_PLACED_NO, BCAST_PLACED_BY_ORDER, BCAST_PLACED_MEASURED = 0, 1, 2


def bcast_memory_regions() -> Tuple[int, int]:
    """(number of regions of the current device's memory, bytes of each)."""
    n, each = ctypes.c_int(0), ctypes.c_size_t(0)
    _check(_lib.bcast_memory_regions(ctypes.byref(n), ctypes.byref(each)), "bcast_memory_regions")
    return n.value, each.value


def bcast_buffers_alloc(bytes_each: Sequence[int], regions: Sequence[int]) -> Tuple[list, int]:
    """Device buffers placed by region; returns (device addresses, BCAST_PLACED_*)."""
    n = len(bytes_each)
    if len(regions) != n:
        raise BcastError(BCAST_ERR_ARG, "bcast_buffers_alloc: %d sizes, %d regions" % (n, len(regions)))
    ptrs = (ctypes.c_void_p * n)()
    placed = ctypes.c_int(0)
    _check(_lib.bcast_buffers_alloc(n, (ctypes.c_size_t * n)(*bytes_each), (ctypes.c_int * n)(*regions), ptrs, ctypes.byref(placed)),
           "bcast_buffers_alloc")
    return [int(p or 0) for p in ptrs], placed.value


def bcast_buffers_free(ptrs: Sequence[int]) -> None:
    n = len(ptrs)
    _check(_lib.bcast_buffers_free(n, (ctypes.c_void_p * n)(*ptrs)), "bcast_buffers_free")


def bcast_plan_set_replayable(plan: Plan, on: bool) -> None:
    _check(_lib.bcast_plan_set_replayable(plan.handle, 1 if on else 0), "bcast_plan_set_replayable")


def bcast_plan_enable_trace(plan: Plan, entries: int) -> None:
    _check(_lib.bcast_plan_enable_trace(plan.handle, entries), "bcast_plan_enable_trace")


def bcast_plan_read_trace(plan: Plan, entries: int):
    """[(begin, end)] device-clock ticks (100 MHz) per (stage, chunk), stage-major."""
    buf = (ctypes.c_uint64 * (2 * entries))()
    _check(_lib.bcast_plan_read_trace(plan.handle, buf, entries), "bcast_plan_read_trace")
    return [(buf[2 * i], buf[2 * i + 1]) for i in range(entries)]


def bcast_plan_handoff_counts(plan: Plan) -> Tuple[int, int]:
    """(same-XCD, cross-XCD) chain hand-offs counted so far (needs BCAST_MODE_COUNT)."""
    a, b = ctypes.c_uint64(0), ctypes.c_uint64(0)
    _check(_lib.bcast_plan_handoff_counts(plan.handle, ctypes.byref(a), ctypes.byref(b)), "bcast_plan_handoff_counts")
    return a.value, b.value


def bcast_chain_geometry(nranks: int, bytes: int, chunk_bytes: int, max_waves: int, lanes_request: int = 0,
                         stages_request: int = 0, trip_request: int = 0, block_request: int = 0) -> dict:
    info = PlanInfo()
    req = ChainRequest(lanes_request, stages_request, trip_request, block_request)
    _check(_lib.bcast_chain_geometry(nranks, bytes, chunk_bytes, max_waves, ctypes.byref(req), ctypes.byref(info)),
           "bcast_chain_geometry")
    return info.as_dict()


def bcast_tune(nranks: int, min_bytes: int, max_bytes: int, algo_mask: int = 0, stream=None,
               table_path: Optional[str] = None) -> None:
    path = table_path.encode() if table_path else None
    _check(_lib.bcast_tune(nranks, min_bytes, max_bytes, algo_mask, _stream(stream), path), "bcast_tune")


def bcast_tune_load(table_path: str) -> None:
    _check(_lib.bcast_tune_load(str(table_path).encode()), "bcast_tune_load")


def bcast_tune_save(table_path: str) -> None:
    _check(_lib.bcast_tune_save(str(table_path).encode()), "bcast_tune_save")


def bcast_tune_clear() -> None:
    _check(_lib.bcast_tune_clear(), "bcast_tune_clear")


def bcast_tune_set(nranks: int, bytes: int, algo: int, chunk_bytes: int, usec: float = 0.0) -> None:
    _check(_lib.bcast_tune_set(nranks, bytes, algo, chunk_bytes, usec), "bcast_tune_set")


def bcast_tune_lookup(nranks: int, bytes: int) -> Tuple[int, int, float]:
    """(algo, chunk_bytes, usec) of the entry that AUTO would use."""
    a, c, u = ctypes.c_int(0), ctypes.c_size_t(0), ctypes.c_double(0.0)
    _check(_lib.bcast_tune_lookup(nranks, bytes, ctypes.byref(a), ctypes.byref(c), ctypes.byref(u)), "bcast_tune_lookup")
    return a.value, c.value, u.value


def bcast_tune_set_log(log_path: Optional[str]) -> None:
    _check(_lib.bcast_tune_set_log(log_path.encode() if log_path else None), "bcast_tune_set_log")


def bcast_tune_put(nranks: int, bytes: int, **fields) -> None:
    """Install one entry; fields are those of bcast_tune_entry_t."""
    e = TuneEntry(**fields)
    _check(_lib.bcast_tune_put(nranks, bytes, ctypes.byref(e)), "bcast_tune_put")


def bcast_tune_get(nranks: int, bytes: int) -> dict:
    """The entry AUTO / chunk 0 would use for this size (nearest bucket)."""
    e = TuneEntry()
    _check(_lib.bcast_tune_get(nranks, bytes, ctypes.byref(e)), "bcast_tune_get")
    return e.as_dict()


def bcast_tune_reduce(nranks: int, min_bytes: int, max_bytes: int, stream=None, table_path: Optional[str] = None) -> None:
    path = table_path.encode() if table_path else None
    _check(_lib.bcast_tune_reduce(nranks, min_bytes, max_bytes, _stream(stream), path), "bcast_tune_reduce")


def bcast_tune_reduce_put(nranks: int, bytes: int, **fields) -> None:
    e = ReduceEntry(**fields)
    _check(_lib.bcast_tune_reduce_put(nranks, bytes, ctypes.byref(e)), "bcast_tune_reduce_put")


def bcast_tune_reduce_get(nranks: int, bytes: int) -> dict:
    e = ReduceEntry()
    _check(_lib.bcast_tune_reduce_get(nranks, bytes, ctypes.byref(e)), "bcast_tune_reduce_get")
    return e.as_dict()


def bcast_plan_set_reduce_trip(plan: Plan, trip_bytes: int) -> None:
    _check(_lib.bcast_plan_set_reduce_trip(plan.handle, trip_bytes), "bcast_plan_set_reduce_trip")


def bcast_debug_store_pattern(bufs, bytes: int, stream=None) -> None:
    """Overwrite [0, bytes) of every buffer with the dependency-free store pattern (measurement)."""
    _check(_lib.bcast_debug_store_pattern(_ptr_array(bufs), len(bufs), bytes, _stream(stream)), "bcast_debug_store_pattern")


def bcast_debug_load_pattern(bufs, bytes: int, out, write_result: bool, stream=None) -> None:
    """Read every buffer once with the dependency-free load pattern; optionally write the xor fold to out."""
    _check(_lib.bcast_debug_load_pattern(_ptr_array(bufs), len(bufs), bytes, _ptr(out), int(write_result), _stream(stream)),
           "bcast_debug_load_pattern")


def bcast_tune_count() -> int:
    return _lib.bcast_tune_count()


def bcast_strerror(status: int) -> str:
    return _lib.bcast_strerror(status).decode()


def bcast_last_hip_error() -> int:
    return _lib.bcast_last_hip_error()


def bcast_version() -> str:
    return _lib.bcast_version().decode()
