"""Large working sets built in place: HBM arenas filled by torch, pageable arenas from mmap.

Input generation only.  torch is used for device memory and its random generators; nothing
here chunks, copies or hashes a working set the way the swap does.
"""
from __future__ import annotations

import ctypes
import mmap

import numpy as np

from .sets import Layout, make_layout

_MADV_HUGEPAGE = 14
_libc = ctypes.CDLL(None, use_errno=True)


def pageable_arena(nbytes: int, fill: int | None = 0) -> np.ndarray:
    """Anonymous private mapping (ordinary pageable memory), huge pages requested,
    faulted in up front so that a timed run does not measure the page allocator."""
    nbytes = max(nbytes, mmap.PAGESIZE)
    mm = mmap.mmap(-1, nbytes, flags=mmap.MAP_PRIVATE | mmap.MAP_ANONYMOUS)
    arr = np.frombuffer(mm, dtype=np.uint8)
    _libc.madvise(ctypes.c_void_p(arr.ctypes.data), ctypes.c_size_t(nbytes), _MADV_HUGEPAGE)
    if fill is not None:
        step = 1 << 30
        for a in range(0, nbytes, step):
            arr[a:a + step] = fill
    return arr


def device_view(address: int, nbytes: int, device: str = "cuda:0"):
    """A uint8 torch tensor over device memory that torch did not allocate (the caller keeps it
    alive and mapped for as long as the tensor is used)."""
    import torch

    class _Raw:
        __cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (address, False), "version": 2}

    return torch.as_tensor(_Raw(), device=device)


class BigSet:
    """One application's working set at full size: an HBM arena (torch uint8) and a pageable
    arena with the same layout (256 B aligned bases, red zones between allocations)."""

    def __init__(self, sizes, seed: int, resident: str, content: str, device: str = "cuda:0",
                 redzone: int = 256, red: int = 0xC3, poison_dev: int = 0xA5, poison_host: int = 0x5A,
                 share_dev: "BigSet | None" = None, dev_arena=None, pinned_host: bool = False):
        """share_dev: for an in-place switch -- this (host-resident) set gets no HBM of its own; its
        device ranges lie in the other set's arena, which must have the same layout.
        dev_arena: a uint8 device tensor supplied by the caller (for instance a view of a mapped
        address space) that becomes this set's HBM arena.  A GPU-resident set is generated into it;
        a host-resident set only takes its addresses and never touches it, since the memory behind
        it may be another application's.
        pinned_host: the host arena is pinned, GPU-addressable memory (the pinned tier) instead of
        pageable memory."""
        import torch
        self.sizes = [s if isinstance(s, int) else s[1] for s in sizes]
        self.names = [("" if isinstance(s, int) else s[0]) for s in sizes]
        self.seed, self.resident, self.red = seed, resident, red
        self.layout: Layout = make_layout(self.sizes, redzone=redzone)
        if dev_arena is not None:
            assert dev_arena.dtype == torch.uint8 and dev_arena.numel() >= self.layout.total and share_dev is None
        if dev_arena is not None and resident == "dev":
            self.dev = dev_arena[:self.layout.total]
            self.dev.fill_(red)
        else:
            self.dev = torch.full((self.layout.total,), red, dtype=torch.uint8, device=device)
        if pinned_host:
            self.host_t = torch.empty(max(self.layout.total, 4096), dtype=torch.uint8, pin_memory=True)
            self.host = self.host_t.numpy()
            self.host[:] = red
        else:
            self.host = pageable_arena(self.layout.total, fill=red)
            self.host_t = torch.from_numpy(self.host)
        g = torch.Generator(device=device)
        g.manual_seed(seed)
        for o, b in zip(self.layout.offsets, self.sizes):
            v = self.dev[o:o + b]
            if content == "bf16_normal" and b % 2 == 0 and b > 0:
                v.view(torch.bfloat16).normal_(0.0, 0.02, generator=g)
            elif b > 0:
                v.random_(0, 256, generator=g)
        torch.cuda.synchronize()
        if resident == "host":       # B starts in pageable memory; its HBM ranges are poisoned
            step = 1 << 30
            for a in range(0, self.layout.total, step):
                self.host_t[a:a + step].copy_(self.dev[a:a + step])
            if share_dev is not None:
                assert resident == "host" and share_dev.layout.offsets == self.layout.offsets \
                    and share_dev.sizes == self.sizes, "in-place sets must share one layout"
                self.dev = share_dev.dev          # the generator's scratch arena is dropped here
            elif dev_arena is not None:
                self.dev = dev_arena[:self.layout.total]     # likewise; addresses only
            else:
                for o, b in zip(self.layout.offsets, self.sizes):
                    self.dev[o:o + b] = poison_dev
        else:                        # A is GPU resident; its pageable ranges are poisoned
            for o, b in zip(self.layout.offsets, self.sizes):
                self.host[o:o + b] = poison_host
        torch.cuda.synchronize()

    @property
    def total_bytes(self) -> int:
        return sum(self.sizes)

    def rows(self):
        bd, bh = self.dev.data_ptr(), self.host.ctypes.data
        return [(bd + o, bh + o, b) for o, b in zip(self.layout.offsets, self.sizes)]

    def rows_np(self) -> np.ndarray:
        """The allocation table as a (n, 3) uint64 array: device address, host address, bytes."""
        offs = np.asarray(self.layout.offsets, dtype=np.uint64)
        out = np.empty((len(self.sizes), 3), dtype=np.uint64)
        out[:, 0] = np.uint64(self.dev.data_ptr()) + offs
        out[:, 1] = np.uint64(self.host.ctypes.data) + offs
        out[:, 2] = np.asarray(self.sizes, dtype=np.uint64)
        return out

    def dev_view(self, i: int):
        o, b = self.layout.offsets[i], self.sizes[i]
        return self.dev[o:o + b]

    def host_view(self, i: int) -> np.ndarray:
        o, b = self.layout.offsets[i], self.sizes[i]
        return self.host[o:o + b]

    def allocations_equal(self) -> bool:
        """Every allocation's HBM bytes against its pageable bytes (no red zones: for arenas whose
        gaps belong to someone else)."""
        import torch
        for o, b in zip(self.layout.offsets, self.sizes):
            step = 1 << 30
            for a in range(o, o + b, step):
                e = min(a + step, o + b)
                if not torch.equal(self.dev[a:e], self.host_t[a:e].to(self.dev.device)):
                    return False
        return True

    def arenas_equal(self) -> bool:
        """Whole-arena compare, HBM against pageable (contents and red zones), in 1 GiB steps."""
        import torch
        step = 1 << 30
        for a in range(0, self.layout.total, step):
            if not torch.equal(self.dev[a:a + step], self.host_t[a:a + step].to(self.dev.device)):
                return False
        return True
