"""Device memory for tests that hand the library caller-owned device pointers: plain hipMalloc / hipMemcpy
through ctypes on the HIP runtime the library itself is linked against (a second HIP runtime in the process,
such as the one bundled with torch, does not see the GPU once this one has initialised it)."""
from __future__ import annotations

import ctypes as C

import numpy as np

import paper_2302_07863_amd as pkg

_hip = None
H2D, D2H = 1, 2


def hip():
    global _hip
    if _hip is None:
        pkg.lib()                                   # loads libbild.so and, with it, libamdhip64
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t]
        _hip.hipFree.argtypes = [C.c_void_p]
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipMemset.argtypes = [C.c_void_p, C.c_int, C.c_size_t]
    return _hip


class DeviceArray:
    """A device copy of a numpy array (or `nbytes` of zeroed device memory)."""

    def __init__(self, host: np.ndarray | None = None, nbytes: int = 0):
        self.ptr = C.c_void_p()
        self.nbytes = int(host.nbytes if host is not None else nbytes)
        assert hip().hipMalloc(C.byref(self.ptr), max(self.nbytes, 16)) == 0
        if host is not None:
            h = np.ascontiguousarray(host)
            assert hip().hipMemcpy(self.ptr, h.ctypes.data, self.nbytes, H2D) == 0
        else:
            assert hip().hipMemset(self.ptr, 0, max(self.nbytes, 16)) == 0

    def to_host(self, dtype, count: int) -> np.ndarray:
        out = np.zeros(count, dtype=dtype)
        assert out.nbytes <= self.nbytes
        assert hip().hipDeviceSynchronize() == 0
        assert hip().hipMemcpy(out.ctypes.data, self.ptr, out.nbytes, D2H) == 0
        return out

    def free(self):
        if self.ptr:
            hip().hipFree(self.ptr)
            self.ptr = C.c_void_p()

    __del__ = free
