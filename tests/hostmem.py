"""Pinned host memory of an exact size for the GPU tests (torch's pinned allocator rounds
large requests up to a power of two, which matters when a test needs most of what the
machine allows).  Plain ctypes over the HIP runtime; test infrastructure only."""
import ctypes

import numpy as np

_hip = None


def _lib():
    global _hip
    if _hip is None:
        h = ctypes.CDLL("libamdhip64.so")
        h.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
        h.hipHostMalloc.restype = ctypes.c_int
        h.hipHostFree.argtypes = [ctypes.c_void_p]
        h.hipHostFree.restype = ctypes.c_int
        _hip = h
    return _hip


class Pinned:
    """nbytes of pinned host memory; .array(dtype, shape) views it; free() releases it."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        p = ctypes.c_void_p()
        rc = _lib().hipHostMalloc(ctypes.byref(p), self.nbytes, 0)
        if rc != 0 or not p.value:
            raise MemoryError(f"hipHostMalloc({self.nbytes}) failed with {rc}")
        self.ptr = p.value

    def array(self, dtype, shape, offset_bytes: int = 0):
        count = int(np.prod(shape))
        buf = (ctypes.c_uint8 * (count * np.dtype(dtype).itemsize)).from_address(self.ptr + offset_bytes)
        return np.frombuffer(buf, dtype=dtype, count=count).reshape(shape)

    def free(self):
        if self.ptr:
            _lib().hipHostFree(ctypes.c_void_p(self.ptr))
            self.ptr = 0
