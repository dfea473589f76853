"""ctypes front of ``nixie_oracle.c`` (plain-C CPU oracle).  TEST INFRASTRUCTURE.

The C file states what a context-switch swap computes (paper, "Hierarchical
Memory": exactly one copy of each chunk, moved as a whole between tiers;
"Speeding Up Context Switches": B's chunks go to GPU memory while A's are
evicted to CPU memory).  Here numpy ``uint8`` arrays stand in for both the GPU
allocations and their pageable host backings.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import time
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nixie_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_nixie.so")


def lib_path() -> str:
    return _LIB


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lpthread"])
    return _LIB


class OracleError(RuntimeError):
    def __init__(self, code: int, report: dict | None = None):
        self.code = code
        self.report = report or {}
        super().__init__(f"oracle invariant violated: {_CODES.get(code, code)} {self.report}")


_CODES = {0: "OK", -1: "EINVAL", -2: "ENOMEM", -3: "ESLOT_BUSY", -4: "EBUDGET",
          -5: "ECOUNT", -6: "ERANGE", -7: "ELEFTOVER"}
FAULTS = {"none": 0, "drop_chunk": 1, "short_piece": 2, "slot_shift": 3,
          "double_copy": 4, "overrun": 5, "wrong_direction": 6, "ignore_alias": 7,
          "reuse_busy_slot": 8, "overcommit": 9}


class _Alloc(C.Structure):
    _fields_ = [("dev", C.c_void_p), ("host", C.c_void_p), ("bytes", C.c_uint64)]


class _Report(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "hwm_staged_bytes", "final_staged_bytes", "n_out_chunks", "n_in_chunks",
        "bytes_out", "bytes_in", "count_errors", "steps")]


def _table(pairs: Sequence[tuple[np.ndarray, np.ndarray]]):
    """pairs: (dev_view, host_view) uint8 arrays of equal length, C-contiguous."""
    arr = (_Alloc * max(1, len(pairs)))()
    for i, (d, h) in enumerate(pairs):
        assert d.dtype == np.uint8 and h.dtype == np.uint8 and d.size == h.size
        assert d.flags.c_contiguous and h.flags.c_contiguous
        arr[i].dev = d.ctypes.data
        arr[i].host = h.ctypes.data
        arr[i].bytes = d.size
    return arr, len(pairs)


class Oracle:
    def __init__(self):
        build()
        L = C.CDLL(_LIB)
        L.o_switch_direct.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.o_switch_direct.restype = None
        L.o_mix64.argtypes = [C.c_uint64]
        L.o_mix64.restype = C.c_uint64
        L.o_hash64.argtypes = [C.c_void_p, C.c_uint64]
        L.o_hash64.restype = C.c_uint64
        L.o_hash_table.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_void_p]
        L.o_hash_table.restype = None
        L.o_switch_staged.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64,
                                      C.c_uint64, C.c_uint64, C.c_uint64, C.c_int,
                                      C.c_uint64, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.o_switch_staged.restype = C.c_int
        L.o_switch_staged_mt.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64,
                                         C.c_uint64, C.c_uint64, C.c_int, C.c_void_p]
        L.o_switch_staged_mt.restype = C.c_int
        self._L = L

    # -- result definition ------------------------------------------------
    def switch_direct(self, out_pairs, in_pairs) -> float:
        """Two memcpy loops; returns the seconds the C call took."""
        o, no = _table(out_pairs)
        i, ni = _table(in_pairs)
        t0 = time.perf_counter()
        self._L.o_switch_direct(o, no, i, ni)
        return time.perf_counter() - t0

    # -- staged form with invariant checks --------------------------------
    def switch_staged(self, out_pairs, in_pairs, ring_bytes: int, slot_bytes: int,
                      n_out_slots: int | None = None, pack: bool = True, seed: int = 0,
                      check_bytes: bool = False, fault: str = "none", in_place: bool = False) -> dict:
        """in_place: incoming device ranges may overlap outgoing ones; a chunk is only scattered
        once every GPU byte it overwrites has been staged out."""
        o, no = _table(out_pairs)
        i, ni = _table(in_pairs)
        if n_out_slots is None:
            n_out_slots = (ring_bytes // slot_bytes) // 2 if slot_bytes else 0
        rep = _Report()
        rc = self._L.o_switch_staged(o, no, i, ni, ring_bytes, slot_bytes, n_out_slots,
                                     int(pack), seed & (2**64 - 1), int(check_bytes),
                                     FAULTS[fault], int(in_place), C.byref(rep))
        d = {n: int(getattr(rep, n)) for n, _ in _Report._fields_}
        if rc != 0:
            raise OracleError(rc, d)
        return d

    def switch_staged_mt(self, out_pairs, in_pairs, ring_bytes: int, slot_bytes: int,
                         threads_per_dir: int) -> float:
        o, no = _table(out_pairs)
        i, ni = _table(in_pairs)
        sec = C.c_double(0.0)
        rc = self._L.o_switch_staged_mt(o, no, i, ni, ring_bytes, slot_bytes,
                                        threads_per_dir, C.byref(sec))
        if rc != 0:
            raise OracleError(rc)
        return sec.value

    # -- hash ---------------------------------------------------------------
    def mix64(self, x: int) -> int:
        return int(self._L.o_mix64(x & (2**64 - 1)))

    def hash64(self, data: np.ndarray) -> int:
        data = np.ascontiguousarray(data, dtype=np.uint8)
        return int(self._L.o_hash64(data.ctypes.data, data.size))

    def hash_table(self, pairs, which: str) -> np.ndarray:
        """which = 'dev' or 'host': the side that currently holds the data."""
        t, n = _table(pairs)
        out = np.zeros(max(1, n), dtype=np.uint64)
        self._L.o_hash_table(t, n, 0 if which == "dev" else 1, out.ctypes.data)
        return out[:n]
