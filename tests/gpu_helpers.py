"""GPU-side plumbing for the parity tests: device arenas (torch is used for memory only)."""
from __future__ import annotations

import numpy as np
import torch

from tests.helpers import HostSet


class GpuSet:
    """A HostSet whose 'device' arena really lives in HBM.

    ``hs.dev`` (numpy) is the image uploaded before the switch; ``download()`` reads HBM back
    through torch's own copy path, independent of the library under test."""

    def __init__(self, sizes, seed: int, resident: str, **kw):
        self.hs = HostSet(sizes, seed, resident, **kw)
        self.dev_t = torch.from_numpy(self.hs.dev).to("cuda:0")
        assert self.dev_t.data_ptr() % 256 == 0
        torch.cuda.synchronize()

    def rows(self):
        base_d, base_h = self.dev_t.data_ptr(), self.hs.host.ctypes.data
        return [(base_d + od, base_h + oh, b)
                for od, oh, b in zip(self.hs.ldev.offsets, self.hs.lhost.offsets, self.hs.sizes)]

    def download(self) -> np.ndarray:
        torch.cuda.synchronize()
        return self.dev_t.cpu().numpy()


def first_diff(a: np.ndarray, b: np.ndarray) -> str:
    if a.shape != b.shape:
        return f"shapes {a.shape} vs {b.shape}"
    bad = np.flatnonzero(a != b)
    return "equal" if bad.size == 0 else f"{bad.size} bytes differ, first at {int(bad[0])}"


class RawDevice:
    """Upload / download for device addresses that no torch tensor owns (mapped spaces): plain
    hipMemcpy of the HIP runtime the library itself is linked to, looked up through its handle."""

    def __init__(self, lib_path: str):
        import ctypes
        self._c = ctypes
        self._rt = ctypes.CDLL(lib_path)
        self._rt.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        self._rt.hipDeviceSynchronize.argtypes = []

    def upload(self, dev_addr: int, data: np.ndarray) -> None:
        data = np.ascontiguousarray(data, dtype=np.uint8)
        rc = self._rt.hipMemcpy(dev_addr, data.ctypes.data, data.size, 1)   # hipMemcpyHostToDevice
        assert rc == 0, f"hipMemcpy H2D failed: {rc}"

    def download(self, dev_addr: int, nbytes: int) -> np.ndarray:
        out = np.empty(nbytes, dtype=np.uint8)
        assert self._rt.hipDeviceSynchronize() == 0
        rc = self._rt.hipMemcpy(out.ctypes.data, dev_addr, nbytes, 2)       # hipMemcpyDeviceToHost
        assert rc == 0, f"hipMemcpy D2H failed: {rc}"
        return out
