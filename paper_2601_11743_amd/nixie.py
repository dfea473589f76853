"""ctypes binding of libnixie.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Iterable, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnixie.so")

EINVAL, EOVERLAP, ENOMEM, EHIP, ETIMEOUT, EMISMATCH, EBUSY, EUNMAPPED = -1, -2, -3, -4, -5, -6, -7, -8
ORDER_TABLE, ORDER_LARGE_FIRST, ORDER_ADDRESS, ORDER_REVERSE = 0, 1, 2, 3
SPLIT_BY_BYTES, SERIALIZE, DIAG_RING_ONLY, DIAG_STALL_DRAIN, HOST_PLAIN_MEMCPY, IN_PLACE, NO_DIRECT, HOST_SPIN = 1, 2, 4, 8, 16, 32, 64, 128
NO_FLEX_WGS = 256

DECLARED_SYMBOLS = (
    "nixie_layout_create", "nixie_layout_info", "nixie_layout_chunks", "nixie_layout_segments",
    "nixie_layout_destroy", "nixie_plan", "nixie_plan_info", "nixie_plan_destroy", "nixie_switch",
    "nixie_hash_tables", "nixie_verify", "nixie_hash_buffers", "nixie_link_peak",
    "nixie_strerror", "nixie_last_hip_error",
    "nixie_sched_create", "nixie_sched_destroy", "nixie_sched_add_app", "nixie_sched_api_enter",
    "nixie_sched_api_return", "nixie_sched_request", "nixie_sched_tick", "nixie_sched_app_info",
    "nixie_pool_create", "nixie_pool_info", "nixie_pool_destroy", "nixie_space_create", "nixie_space_assign", "nixie_space_map",
    "nixie_space_unmap", "nixie_space_mapped", "nixie_space_destroy",
    "nixie_tier_register", "nixie_tier_unregister", "nixie_host_copy", "nixie_place",
    "nixie_switch_begin", "nixie_switch_wait_in", "nixie_switch_end",
    "nixie_ring_create", "nixie_ring_destroy", "nixie_plan_on_ring",
    "nixie_hash_buffers_noalloc", "nixie_abi_check",
)


class _Alloc(C.Structure):
    _fields_ = [("dev_ptr", C.c_void_p), ("host_ptr", C.c_void_p), ("bytes", C.c_uint64)]


class _Table(C.Structure):
    _fields_ = [("allocs", C.POINTER(_Alloc)), ("count", C.c_uint64)]


class _Opts(C.Structure):
    _fields_ = [("slot_bytes", C.c_uint64), ("out_slots", C.c_uint32), ("order", C.c_uint32),
                ("gather_wgs", C.c_uint32), ("scatter_wgs", C.c_uint32), ("team", C.c_uint32),
                ("drain_threads", C.c_uint32), ("fill_threads", C.c_uint32),
                ("timeout_ms", C.c_uint32), ("flags", C.c_uint32), ("xcd_mask", C.c_uint32), ("flex_wgs", C.c_uint32)]


class _Info(C.Structure):
    _fields_ = [("ring_bytes", C.c_uint64), ("slot_bytes", C.c_uint64),
                ("out_slots", C.c_uint32), ("in_slots", C.c_uint32),
                ("chunks_out", C.c_uint64), ("chunks_in", C.c_uint64),
                ("segments_out", C.c_uint64), ("segments_in", C.c_uint64),
                ("bytes_out", C.c_uint64), ("bytes_in", C.c_uint64),
                ("pinned_ring_bytes", C.c_uint64), ("pinned_ctrl_bytes", C.c_uint64),
                ("gather_wgs", C.c_uint32), ("scatter_wgs", C.c_uint32),
                ("team_out", C.c_uint32), ("team_in", C.c_uint32),
                ("drain_threads", C.c_uint32), ("fill_threads", C.c_uint32),
                ("direct_chunks_out", C.c_uint64), ("direct_chunks_in", C.c_uint64),
                ("direct_bytes_out", C.c_uint64), ("direct_bytes_in", C.c_uint64), ("flex_wgs", C.c_uint32)]


class _Segment(C.Structure):
    _fields_ = [("dev_addr", C.c_uint64), ("host_addr", C.c_uint64),
                ("slot_off", C.c_uint32), ("len", C.c_uint32)]


class _Chunk(C.Structure):
    _fields_ = [("seg_begin", C.c_uint64), ("seg_count", C.c_uint32), ("used_bytes", C.c_uint32),
                ("dep_out", C.c_uint64)]


class _Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "bytes_out", "bytes_in", "ns_total", "ns_out_done", "ns_in_done", "ns_kernel", "ns_launch",
        "drain_wait_ns", "fill_wait_ns", "gather_stall_ticks", "scatter_stall_ticks")] + [
        ("kernels", C.c_uint32), ("gpu_status", C.c_uint32), ("pump_rounds_out", C.c_uint32), ("pump_rounds_in", C.c_uint32),
        ("credit_rtt_ticks_out", C.c_uint32), ("credit_rtt_ticks_in", C.c_uint32)]


class _Report(C.Structure):
    _fields_ = [("checked_out", C.c_uint64), ("checked_in", C.c_uint64),
                ("mismatched_out", C.c_uint64), ("mismatched_in", C.c_uint64),
                ("first_bad_out", C.c_int64), ("first_bad_in", C.c_int64)]


class _LinkPeak(C.Structure):
    _fields_ = [(n, C.c_double) for n in (
        "sdma_d2h", "sdma_h2d", "sdma_d2h_both", "sdma_h2d_both",
        "kernel_d2h", "kernel_h2d", "kernel_d2h_both", "kernel_h2d_both")]


class _ChunkState(C.Structure):
    _fields_ = [("bytes", C.c_uint64), ("app", C.c_uint32), ("tier", C.c_uint32)]


class _Capacity(C.Structure):
    _fields_ = [("gpu_bytes", C.c_uint64), ("pinned_bytes", C.c_uint64)]


class _Placement(C.Structure):
    _fields_ = [("restored_bytes", C.c_uint64), ("restored_from_pageable_bytes", C.c_uint64),
                ("evicted_bytes", C.c_uint64), ("kept_pinned_bytes", C.c_uint64), ("to_pageable_bytes", C.c_uint64),
                ("gpu_used_after", C.c_uint64), ("pinned_used_after", C.c_uint64)]


class _SchedParams(C.Structure):
    _fields_ = [("levels", C.c_uint32), ("allot_ns", C.c_uint64), ("preempt_ns", C.c_uint64), ("idle_ns", C.c_uint64)]


class _SchedDecision(C.Structure):
    _fields_ = [("run", C.c_int32), ("evict", C.c_int32), ("prefetch", C.c_int32), ("switched", C.c_uint32)]


class _SchedApp(C.Structure):
    _fields_ = [("priority", C.c_uint32), ("idle", C.c_uint32), ("pending", C.c_uint32), ("running", C.c_uint32),
                ("exec_ns", C.c_uint64)]


def _as_dict(s: C.Structure) -> dict:
    return {n: getattr(s, n) for n, _ in s._fields_}


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """Load libnixie.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        # Nothing built yet: build once (hipcc cross-compiles, no GPU needed).  Callers that are about to
        # use the GPU load the library before they touch it, since a build starts other programs.
        try:
            from . import build as _build
            _build.build()
        except Exception as e:   # no compiler, or the build failed: there is no CPU fallback
            raise RuntimeError(f"{_LIB_PATH} is missing and could not be built ({e}): run "
                               "paper_2601_11743_amd/build.py (or __graft_entry__.build())") from e
    L = C.CDLL(_LIB_PATH)
    vp, u64, i32 = C.c_void_p, C.c_uint64, C.c_int
    L.nixie_layout_create.argtypes = [C.POINTER(_Table), C.POINTER(_Table), u64, C.POINTER(_Opts), C.POINTER(vp)]
    L.nixie_layout_info.argtypes = [vp, C.POINTER(_Info)]
    L.nixie_layout_chunks.argtypes = [vp, i32, C.POINTER(_Chunk), u64]
    L.nixie_layout_chunks.restype = C.c_int64
    L.nixie_layout_segments.argtypes = [vp, i32, C.POINTER(_Segment), u64]
    L.nixie_layout_segments.restype = C.c_int64
    L.nixie_layout_destroy.argtypes = [vp]
    L.nixie_layout_destroy.restype = None
    L.nixie_plan.argtypes = [C.POINTER(_Table), C.POINTER(_Table), u64, C.POINTER(_Opts), C.POINTER(vp)]
    L.nixie_ring_create.argtypes = [u64, C.POINTER(vp)]
    L.nixie_ring_destroy.argtypes = [vp]
    L.nixie_plan_on_ring.argtypes = [C.POINTER(_Table), C.POINTER(_Table), vp, C.POINTER(_Opts), C.POINTER(vp)]
    L.nixie_plan_info.argtypes = [vp, C.POINTER(_Info)]
    L.nixie_plan_destroy.argtypes = [vp]
    L.nixie_plan_destroy.restype = None
    L.nixie_switch.argtypes = [vp, vp, C.POINTER(_Stats)]
    L.nixie_switch_begin.argtypes = [vp, vp]
    L.nixie_switch_wait_in.argtypes = [vp]
    L.nixie_switch_end.argtypes = [vp, C.POINTER(_Stats)]
    L.nixie_hash_tables.argtypes = [vp, vp, vp, vp]
    L.nixie_verify.argtypes = [vp, vp, vp, vp, C.POINTER(_Report)]
    L.nixie_hash_buffers.argtypes = [vp, vp, u64, i32, vp, vp]
    L.nixie_hash_buffers_noalloc.argtypes = [vp, vp, u64, vp, vp]
    L.nixie_abi_check.argtypes = [u64, u64, u64]
    if L.nixie_abi_check(C.sizeof(_Opts), C.sizeof(_Info), C.sizeof(_Stats)) != 0:
        raise RuntimeError(f"{_LIB_PATH} was built from another version of include/nixie.h than this binding: "
                           "rebuild (python -m paper_2601_11743_amd.build)")
    L.nixie_link_peak.argtypes = [u64, i32, C.POINTER(_LinkPeak)]
    L.nixie_sched_create.argtypes = [C.POINTER(_SchedParams), C.POINTER(vp)]
    L.nixie_sched_destroy.argtypes = [vp]
    L.nixie_sched_destroy.restype = None
    L.nixie_sched_add_app.argtypes = [vp, u64]
    L.nixie_sched_api_enter.argtypes = [vp, i32, u64, i32]
    L.nixie_sched_api_return.argtypes = [vp, i32, u64]
    L.nixie_sched_request.argtypes = [vp, i32, u64]
    L.nixie_sched_tick.argtypes = [vp, u64, C.POINTER(_SchedDecision)]
    L.nixie_sched_app_info.argtypes = [vp, i32, u64, C.POINTER(_SchedApp)]
    L.nixie_tier_register.argtypes = [vp, u64]
    L.nixie_tier_unregister.argtypes = [vp]
    L.nixie_place.argtypes = [C.POINTER(_Capacity), C.POINTER(_ChunkState), u64, C.c_uint32, vp, C.c_uint32,
                              vp, vp, C.POINTER(u64), C.POINTER(_Placement)]
    L.nixie_host_copy.argtypes = [vp, vp, vp, u64, C.c_uint32]
    L.nixie_pool_create.argtypes = [u64, u64, C.POINTER(vp)]
    L.nixie_pool_info.argtypes = [vp, C.POINTER(u64), C.POINTER(u64)]
    L.nixie_pool_destroy.argtypes = [vp]
    L.nixie_space_create.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    L.nixie_space_assign.argtypes = [vp, u64, vp, u64]
    L.nixie_space_map.argtypes = [vp, u64, u64]
    L.nixie_space_unmap.argtypes = [vp, u64, u64]
    L.nixie_space_mapped.argtypes = [vp, u64, u64]
    L.nixie_space_destroy.argtypes = [vp]
    L.nixie_strerror.argtypes = [i32]
    L.nixie_strerror.restype = C.c_char_p
    L.nixie_last_hip_error.argtypes = []
    _lib = L
    return L


def strerror(code: int) -> str:
    return lib().nixie_strerror(code).decode()


class NixieError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        hip = lib().nixie_last_hip_error() if code == EHIP else 0
        super().__init__(f"{what}: {strerror(code)} ({code})" + (f", hipError {hip}" if hip else ""))


class Opts:
    """Keyword view of nixie_opts_t; anything left out is the library default."""

    def __init__(self, **kw):
        self.c = _Opts()
        for k, v in kw.items():
            if not hasattr(self.c, k):
                raise TypeError(f"unknown option {k}")
            setattr(self.c, k, v)


def _table(allocs):
    """allocs: iterable of (dev_ptr, host_ptr, bytes) integers, or a C-contiguous uint64 numpy
    array of shape (n, 3) with the same columns (used as is, no copy)."""
    if isinstance(allocs, np.ndarray):
        a = np.ascontiguousarray(allocs, dtype=np.uint64)
        if a.ndim != 2 or a.shape[1] != 3:
            raise TypeError("allocation table array must have shape (n, 3)")
        n = a.shape[0]
        ptr = C.cast(a.ctypes.data, C.POINTER(_Alloc)) if n else C.cast(None, C.POINTER(_Alloc))
        return _Table(ptr, n), a
    rows = list(allocs or [])
    arr = (_Alloc * max(1, len(rows)))()
    for i, (d, h, b) in enumerate(rows):
        arr[i].dev_ptr, arr[i].host_ptr, arr[i].bytes = d, h, b
    t = _Table(arr, len(rows))
    return t, arr


def _opts_ptr(opts: Opts | None):
    return C.byref(opts.c) if opts is not None else None


class Layout:
    """nixie_layout_*: the planner alone (host only, needs no GPU)."""

    def __init__(self, out_allocs, in_allocs, ring_bytes: int, opts: Opts | None = None):
        self._h = C.c_void_p()
        to, self._ko = _table(out_allocs)
        ti, self._ki = _table(in_allocs)
        rc = lib().nixie_layout_create(C.byref(to), C.byref(ti), ring_bytes, _opts_ptr(opts), C.byref(self._h))
        if rc:
            self._h = None
            raise NixieError(rc, "nixie_layout_create")

    def info(self) -> dict:
        i = _Info()
        rc = lib().nixie_layout_info(self._h, C.byref(i))
        if rc:
            raise NixieError(rc, "nixie_layout_info")
        return _as_dict(i)

    def chunks(self, direction: int) -> np.ndarray:
        n = lib().nixie_layout_chunks(self._h, direction, None, 0)
        if n < 0:
            raise NixieError(int(n), "nixie_layout_chunks")
        arr = (_Chunk * max(1, n))()
        lib().nixie_layout_chunks(self._h, direction, arr, n)
        dt = np.dtype([("seg_begin", "<u8"), ("seg_count", "<u4"), ("used_bytes", "<u4"), ("dep_out", "<u8")])
        return np.frombuffer(arr, dtype=dt, count=n).copy()

    def segments(self, direction: int) -> np.ndarray:
        n = lib().nixie_layout_segments(self._h, direction, None, 0)
        if n < 0:
            raise NixieError(int(n), "nixie_layout_segments")
        arr = (_Segment * max(1, n))()
        lib().nixie_layout_segments(self._h, direction, arr, n)
        dt = np.dtype([("dev_addr", "<u8"), ("host_addr", "<u8"), ("slot_off", "<u4"), ("len", "<u4")])
        return np.frombuffer(arr, dtype=dt, count=n).copy()

    def close(self):
        if self._h:
            lib().nixie_layout_destroy(self._h)
            self._h = None

    __del__ = close


class Ring:
    """nixie_ring_*: pinned payload memory shared by many plans, one switch at a time."""

    def __init__(self, nbytes: int):
        self._h = C.c_void_p()
        self.bytes = nbytes
        rc = lib().nixie_ring_create(nbytes, C.byref(self._h))
        if rc:
            self._h = None
            raise NixieError(rc, "nixie_ring_create")

    def close(self):
        if self._h:
            rc = lib().nixie_ring_destroy(self._h)
            if rc:
                raise NixieError(rc, "nixie_ring_destroy")
            self._h = None


class Plan:
    """nixie_plan / nixie_switch / nixie_hash_tables / nixie_verify / nixie_plan_destroy."""

    def __init__(self, out_allocs, in_allocs, ring_bytes, opts: Opts | None = None):
        """ring_bytes: a size (the plan allocates its own ring) or a Ring (nixie_plan_on_ring)."""
        self._h = C.c_void_p()
        to, self._ko = _table(out_allocs)
        ti, self._ki = _table(in_allocs)
        self.n_out, self.n_in = int(to.count), int(ti.count)
        if isinstance(ring_bytes, Ring):
            self._ring = ring_bytes              # keeps the ring alive as long as the plan
            rc = lib().nixie_plan_on_ring(C.byref(to), C.byref(ti), ring_bytes._h, _opts_ptr(opts), C.byref(self._h))
        else:
            rc = lib().nixie_plan(C.byref(to), C.byref(ti), ring_bytes, _opts_ptr(opts), C.byref(self._h))
        if rc:
            self._h = None
            raise NixieError(rc, "nixie_plan")

    def info(self) -> dict:
        i = _Info()
        rc = lib().nixie_plan_info(self._h, C.byref(i))
        if rc:
            raise NixieError(rc, "nixie_plan_info")
        return _as_dict(i)

    def switch(self, stream: int = 0, check: bool = True) -> dict:
        """stream: raw hipStream_t as an integer (torch.cuda.Stream.cuda_stream), 0 = default."""
        st = _Stats()
        rc = lib().nixie_switch(self._h, C.c_void_p(stream), C.byref(st))
        d = _as_dict(st)
        d["rc"] = rc
        if rc and check:
            raise NixieError(rc, "nixie_switch")
        return d

    def switch_begin(self, stream: int = 0) -> None:
        rc = lib().nixie_switch_begin(self._h, C.c_void_p(stream))
        if rc:
            raise NixieError(rc, "nixie_switch_begin")

    def switch_wait_in(self) -> None:
        rc = lib().nixie_switch_wait_in(self._h)
        if rc:
            raise NixieError(rc, "nixie_switch_wait_in")

    def switch_end(self, check: bool = True) -> dict:
        st = _Stats()
        rc = lib().nixie_switch_end(self._h, C.byref(st))
        if rc and check:
            raise NixieError(rc, "nixie_switch_end")
        d = _as_dict(st)
        d["rc"] = rc
        return d

    def hash_tables(self, stream: int = 0):
        ho = np.zeros(max(1, self.n_out), dtype=np.uint64)
        hi = np.zeros(max(1, self.n_in), dtype=np.uint64)
        rc = lib().nixie_hash_tables(self._h, C.c_void_p(stream), ho.ctypes.data, hi.ctypes.data)
        if rc:
            raise NixieError(rc, "nixie_hash_tables")
        return ho[:self.n_out], hi[:self.n_in]

    def verify(self, expect_out, expect_in, stream: int = 0, check: bool = True) -> dict:
        eo = None if expect_out is None else np.ascontiguousarray(expect_out, dtype=np.uint64)
        ei = None if expect_in is None else np.ascontiguousarray(expect_in, dtype=np.uint64)
        rep = _Report()
        rc = lib().nixie_verify(self._h, C.c_void_p(stream),
                                None if eo is None or eo.size == 0 else eo.ctypes.data,
                                None if ei is None or ei.size == 0 else ei.ctypes.data, C.byref(rep))
        d = _as_dict(rep)
        d["rc"] = rc
        if rc and check:
            raise NixieError(rc, f"nixie_verify {d}")
        return d

    def close(self):
        if self._h:
            lib().nixie_plan_destroy(self._h)
            self._h = None

    __del__ = close


def hash_buffers(ptrs: Sequence[int], sizes: Sequence[int], on_device: bool, stream: int = 0) -> np.ndarray:
    n = len(ptrs)
    p = np.asarray(list(ptrs), dtype=np.uint64)
    b = np.asarray(list(sizes), dtype=np.uint64)
    h = np.zeros(max(1, n), dtype=np.uint64)
    if n:
        rc = lib().nixie_hash_buffers(p.ctypes.data, b.ctypes.data, n, int(on_device), C.c_void_p(stream), h.ctypes.data)
        if rc:
            raise NixieError(rc, "nixie_hash_buffers")
    return h[:n]


def hash_buffers_noalloc(ptrs: Sequence[int], sizes: Sequence[int], hashes_dev: int, stream: int = 0) -> None:
    """Enqueue the hashing of device buffers on stream; hashes_dev: device address of len(ptrs) uint64."""
    n = len(ptrs)
    p = np.asarray(list(ptrs), dtype=np.uint64)
    b = np.asarray(list(sizes), dtype=np.uint64)
    rc = lib().nixie_hash_buffers_noalloc(p.ctypes.data, b.ctypes.data, n, C.c_void_p(stream), C.c_void_p(hashes_dev))
    if rc:
        raise NixieError(rc, "nixie_hash_buffers_noalloc")


def link_peak(nbytes: int = 1 << 30, reps: int = 5) -> dict:
    out = _LinkPeak()
    rc = lib().nixie_link_peak(nbytes, reps, C.byref(out))
    if rc:
        raise NixieError(rc, "nixie_link_peak")
    return _as_dict(out)


def tier_register(host_addr: int, nbytes: int) -> None:
    rc = lib().nixie_tier_register(C.c_void_p(host_addr), nbytes)
    if rc:
        raise NixieError(rc, "nixie_tier_register")


def tier_unregister(host_addr: int) -> None:
    rc = lib().nixie_tier_unregister(C.c_void_p(host_addr))
    if rc:
        raise NixieError(rc, "nixie_tier_unregister")


def host_copy(dst: Sequence[int], src: Sequence[int], sizes: Sequence[int], threads: int = 0) -> None:
    n = len(dst)
    d = np.asarray(list(dst), dtype=np.uint64)
    s = np.asarray(list(src), dtype=np.uint64)
    b = np.asarray(list(sizes), dtype=np.uint64)
    rc = lib().nixie_host_copy(d.ctypes.data, s.ctypes.data, b.ctypes.data, n, threads) if n else 0
    if rc:
        raise NixieError(rc, "nixie_host_copy")


TIER_GPU, TIER_PINNED, TIER_PAGEABLE = 0, 1, 2


def place(gpu_bytes: int, pinned_bytes: int, chunks, incoming_app: int, victim_apps):
    """nixie_place.  chunks: sequence of (bytes, app, tier).  Returns (new_tier list, summary dict,
    order list)."""
    n = len(chunks)
    arr = (_ChunkState * max(1, n))()
    for i, (b, a, t) in enumerate(chunks):
        arr[i] = _ChunkState(b, a, t)
    vic = np.asarray(list(victim_apps), dtype=np.uint32)
    tiers = np.zeros(max(1, n), dtype=np.uint32)
    order = np.zeros(max(1, n), dtype=np.uint64)
    moved, summ = C.c_uint64(0), _Placement()
    cap = _Capacity(gpu_bytes, pinned_bytes)
    rc = lib().nixie_place(C.byref(cap), arr, n, incoming_app, vic.ctypes.data if vic.size else None, vic.size,
                           tiers.ctypes.data, order.ctypes.data, C.byref(moved), C.byref(summ))
    if rc:
        raise NixieError(rc, "nixie_place")
    return [int(t) for t in tiers[:n]], _as_dict(summ), [int(i) for i in order[:moved.value]]


class Pool:
    """nixie_pool_*: physical device memory in equal blocks."""

    def __init__(self, nbytes: int, block_bytes: int = 0):
        self._h = C.c_void_p()
        rc = lib().nixie_pool_create(nbytes, block_bytes, C.byref(self._h))
        if rc:
            self._h = None
            raise NixieError(rc, "nixie_pool_create")
        b, k = C.c_uint64(), C.c_uint64()
        lib().nixie_pool_info(self._h, C.byref(b), C.byref(k))
        self.bytes, self.block_bytes = int(b.value), int(k.value)

    def close(self):
        if self._h:
            rc = lib().nixie_pool_destroy(self._h)
            if rc:
                raise NixieError(rc, "nixie_pool_destroy")
            self._h = None


class Space:
    """nixie_space_*: a reserved device address range that maps a pool's blocks, offset for offset."""

    def __init__(self, pool: Pool):
        self._h, base = C.c_void_p(), C.c_void_p()
        self.pool = pool
        rc = lib().nixie_space_create(pool._h, C.byref(self._h), C.byref(base))
        if rc:
            self._h = None
            raise NixieError(rc, "nixie_space_create")
        self.base = int(base.value)

    def assign(self, offset: int, pool_blocks: Sequence[int]) -> None:
        """Pool block pool_blocks[i] backs block offset / block_bytes + i of this space from now on."""
        pb = np.asarray(list(pool_blocks), dtype=np.uint64)
        rc = lib().nixie_space_assign(self._h, offset, pb.ctypes.data, pb.size)
        if rc:
            raise NixieError(rc, "nixie_space_assign")

    def map(self, offset: int = 0, nbytes: int | None = None) -> None:
        rc = lib().nixie_space_map(self._h, offset, self.pool.bytes - offset if nbytes is None else nbytes)
        if rc:
            raise NixieError(rc, "nixie_space_map")

    def unmap(self, offset: int = 0, nbytes: int | None = None) -> None:
        rc = lib().nixie_space_unmap(self._h, offset, self.pool.bytes - offset if nbytes is None else nbytes)
        if rc:
            raise NixieError(rc, "nixie_space_unmap")

    def mapped(self, offset: int = 0, nbytes: int | None = None) -> bool:
        rc = lib().nixie_space_mapped(self._h, offset, self.pool.bytes - offset if nbytes is None else nbytes)
        if rc < 0:
            raise NixieError(rc, "nixie_space_mapped")
        return bool(rc)

    def close(self):
        if self._h:
            rc = lib().nixie_space_destroy(self._h)
            if rc:
                raise NixieError(rc, "nixie_space_destroy")
            self._h = None


class Sched:
    """nixie_sched_*: idleness detection, priority inference and MLFQ (host only, needs no GPU)."""

    def __init__(self, levels: int = 0, allot_ns: int = 0, preempt_ns: int = 0, idle_ns: int = 0):
        self._h = C.c_void_p()
        p = _SchedParams(levels, allot_ns, preempt_ns, idle_ns)
        rc = lib().nixie_sched_create(C.byref(p), C.byref(self._h))
        if rc:
            self._h = None
            raise NixieError(rc, "nixie_sched_create")

    def _ck(self, rc, what):
        if rc < 0:
            raise NixieError(rc, what)
        return rc

    def add_app(self, now: int) -> int:
        return self._ck(lib().nixie_sched_add_app(self._h, now), "nixie_sched_add_app")

    def api_enter(self, app: int, now: int, blocking: bool) -> None:
        self._ck(lib().nixie_sched_api_enter(self._h, app, now, int(blocking)), "nixie_sched_api_enter")

    def api_return(self, app: int, now: int) -> None:
        self._ck(lib().nixie_sched_api_return(self._h, app, now), "nixie_sched_api_return")

    def request(self, app: int, now: int) -> None:
        self._ck(lib().nixie_sched_request(self._h, app, now), "nixie_sched_request")

    def tick(self, now: int) -> dict:
        d = _SchedDecision()
        self._ck(lib().nixie_sched_tick(self._h, now, C.byref(d)), "nixie_sched_tick")
        return {"run": d.run, "evict": d.evict, "prefetch": d.prefetch, "switched": bool(d.switched)}

    def info(self, app: int, now: int) -> dict:
        a = _SchedApp()
        self._ck(lib().nixie_sched_app_info(self._h, app, now, C.byref(a)), "nixie_sched_app_info")
        return {"priority": a.priority, "t_a": a.exec_ns, "idle": bool(a.idle), "pending": bool(a.pending),
                "running": bool(a.running)}

    def close(self):
        if self._h:
            lib().nixie_sched_destroy(self._h)
            self._h = None

    __del__ = close
