"""Page-locked host buffers of an exact size, straight from hipHostMalloc.

PyTorch's pinned allocator rounds every request up to a power of two (a 37.5 GiB staging area would
pin 64 GiB) and keeps freed blocks cached; the multi-GiB KV staging areas of the large workloads are
therefore allocated here and wrapped as tensors.  Plumbing only: nothing of the method lives here.
"""
from __future__ import annotations

import ctypes

import numpy as np

_hip = None


def _lib():
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
        _hip.hipHostMalloc.restype = ctypes.c_int
        _hip.hipHostFree.argtypes = [ctypes.c_void_p]
        _hip.hipHostFree.restype = ctypes.c_int
    return _hip


class PinnedBuffer:
    """nbytes of page-locked host memory; free() (or garbage collection) releases it."""

    def __init__(self, nbytes: int):
        import torch
        torch.cuda.init()                                   # make sure a HIP context exists
        p = ctypes.c_void_p()
        rc = _lib().hipHostMalloc(ctypes.byref(p), max(int(nbytes), 16), 0)
        if rc != 0 or not p.value:
            raise MemoryError(f"hipHostMalloc({nbytes}) failed with HIP error {rc}")
        self.ptr, self.nbytes = p.value, int(nbytes)

    def tensor(self, shape, dtype):
        """A torch CPU tensor over the start of the buffer (no copy).  Keep this object alive."""
        import torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        assert n <= self.nbytes
        raw = (ctypes.c_byte * max(n, 1)).from_address(self.ptr)
        t = torch.frombuffer(raw, dtype=dtype, count=int(np.prod(shape))) if n else torch.empty(0, dtype=dtype)
        return t.view(shape)

    def free(self):
        if self.ptr:
            _lib().hipHostFree(self.ptr)
            self.ptr = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass
