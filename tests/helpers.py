"""Arena plumbing shared by the CPU-oracle tests and the GPU parity tests.

No swap arithmetic here: only buffers, red zones, poison and comparisons.
"""
from __future__ import annotations

import numpy as np

import workloads as W

RED = 0xC3          # red-zone byte, both sides
POISON_DEV = 0xA5   # incoming device ranges before the switch
POISON_HOST = 0x5A  # outgoing host ranges before the switch


def aligned_full(n: int, value: int, align: int = 4096) -> np.ndarray:
    """uint8 array of n bytes whose first byte sits on an ``align`` boundary."""
    raw = np.empty(n + align, dtype=np.uint8)
    off = (-raw.ctypes.data) % align
    a = raw[off:off + n]
    a[:] = value
    return a


class HostSet:
    """One application's working set on the CPU: a 'device' stand-in arena and a
    pageable host arena, same layout, red zones between allocations."""

    def __init__(self, sizes, seed: int, resident: str, skew_dev: int = 0, skew_host: int = 0,
                 redzone: int = 256):
        self.sizes = [s if isinstance(s, int) else s[1] for s in sizes]
        self.seed = seed
        self.resident = resident  # 'dev' (to be evicted) or 'host' (to be brought in)
        self.ldev = W.make_layout(self.sizes, redzone=redzone, skew=skew_dev)
        self.lhost = W.make_layout(self.sizes, redzone=redzone, skew=skew_host)
        self.dev = aligned_full(self.ldev.total, RED)
        self.host = aligned_full(self.lhost.total, RED)
        src, lsrc = (self.dev, self.ldev) if resident == "dev" else (self.host, self.lhost)
        dst, ldst, poison = ((self.host, self.lhost, POISON_HOST) if resident == "dev"
                             else (self.dev, self.ldev, POISON_DEV))
        W.fill_content(src, lsrc, seed)
        for o, b in zip(ldst.offsets, ldst.sizes):
            dst[o:o + b] = poison

    def pairs(self):
        return [(self.dev[od:od + b], self.host[oh:oh + b])
                for od, oh, b in zip(self.ldev.offsets, self.lhost.offsets, self.sizes)]

    def expected(self, i: int) -> np.ndarray:
        return W.content_bytes(self.seed, i, self.sizes[i])

    def check_moved(self):
        """Destination side holds the generated content; red zones untouched."""
        dst, ldst = (self.host, self.lhost) if self.resident == "dev" else (self.dev, self.ldev)
        for i, (o, b) in enumerate(zip(ldst.offsets, ldst.sizes)):
            got = dst[o:o + b]
            exp = self.expected(i)
            if not np.array_equal(got, exp):
                bad = int(np.flatnonzero(got != exp)[0])
                raise AssertionError(f"allocation {i} ({b} B) differs first at byte {bad}")
        self.check_redzones()

    def check_redzones(self):
        for arena, lay in ((self.dev, self.ldev), (self.host, self.lhost)):
            mask = np.ones(arena.size, dtype=bool)
            for o, b in zip(lay.offsets, lay.sizes):
                mask[o:o + b] = False
            if not (arena[mask] == RED).all():
                bad = int(np.flatnonzero(mask & (arena != RED))[0])
                raise AssertionError(f"red zone overwritten at arena byte {bad}")


class AliasedPair:
    """In-place switch inputs: application A (GPU resident) and application B (in pageable memory)
    whose device ranges lie in ONE shared device arena, so B's allocations partly or wholly reuse
    the GPU memory A gives up.  Host arenas are separate.  expected_dev() is the arena a correct
    switch leaves: B's content written over the initial arena (numpy slicing, no swap code)."""

    def __init__(self, sizes_a, sizes_b, seed: int, skew_a: int = 0, skew_b: int = 0, shift_b: int = 0,
                 redzone: int = 256):
        self.sizes_a, self.sizes_b, self.seed = list(sizes_a), list(sizes_b), seed
        self.la = W.make_layout(self.sizes_a, redzone=redzone, skew=skew_a)
        lb = W.make_layout(self.sizes_b, redzone=redzone, skew=skew_b)
        self.lb = W.Layout([o + shift_b for o in lb.offsets], lb.sizes, lb.total + shift_b, redzone)
        total = max(self.la.total, self.lb.total)
        self.dev = aligned_full(total, RED)
        W.fill_content(self.dev, self.la, seed)                 # A is resident
        self.dev0 = self.dev.copy()
        self.lha = W.make_layout(self.sizes_a, redzone=redzone)
        self.lhb = W.make_layout(self.sizes_b, redzone=redzone)
        self.host_a = aligned_full(self.lha.total, RED)
        self.host_b = aligned_full(self.lhb.total, RED)
        for o, b in zip(self.lha.offsets, self.sizes_a):
            self.host_a[o:o + b] = POISON_HOST
        W.fill_content(self.host_b, self.lhb, seed + 1)         # B waits in pageable memory

    def pairs_a(self, dev=None):
        dev = self.dev if dev is None else dev
        return [(dev[od:od + b], self.host_a[oh:oh + b])
                for od, oh, b in zip(self.la.offsets, self.lha.offsets, self.sizes_a)]

    def pairs_b(self, dev=None):
        dev = self.dev if dev is None else dev
        return [(dev[od:od + b], self.host_b[oh:oh + b])
                for od, oh, b in zip(self.lb.offsets, self.lhb.offsets, self.sizes_b)]

    def expected_dev(self) -> np.ndarray:
        e = self.dev0.copy()
        for i, (o, b) in enumerate(zip(self.lb.offsets, self.sizes_b)):
            e[o:o + b] = W.content_bytes(self.seed + 1, i, b)
        return e

    def expected_host_a(self) -> np.ndarray:
        e = aligned_full(self.lha.total, RED)
        for i, (o, b) in enumerate(zip(self.lha.offsets, self.sizes_a)):
            e[o:o + b] = W.content_bytes(self.seed, i, b)
        return e

    def check(self, dev=None):
        dev = self.dev if dev is None else dev
        exp_h, exp_d = self.expected_host_a(), self.expected_dev()
        if not np.array_equal(self.host_a, exp_h):
            bad = int(np.flatnonzero(self.host_a != exp_h)[0])
            raise AssertionError(f"evicted set differs first at host arena byte {bad}")
        if not np.array_equal(dev, exp_d):
            bad = int(np.flatnonzero(dev != exp_d)[0])
            raise AssertionError(f"device arena differs first at byte {bad}")
