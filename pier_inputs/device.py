"""Device-side input synthesis: allocates workload state with torch and fills it with
the counter-based generator of csrc/pier_inputs.hip.  No optimizer arithmetic."""
import ctypes
import os

import torch

from . import shapes

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpier_inputs.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build      # nothing built yet: build once
            _build.build()
        L = ctypes.CDLL(_LIB_PATH)
        L.pier_inputs_fill_normal.restype = ctypes.c_int
        L.pier_inputs_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                              ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                              ctypes.c_float, ctypes.c_void_p]
        L.pier_inputs_host_alloc.restype = ctypes.c_int
        L.pier_inputs_host_alloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t]
        L.pier_inputs_host_free.restype = ctypes.c_int
        L.pier_inputs_host_free.argtypes = [ctypes.c_void_p]
        L.pier_inputs_device_alloc.restype = ctypes.c_int
        L.pier_inputs_device_alloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t]
        L.pier_inputs_device_free.restype = ctypes.c_int
        L.pier_inputs_device_free.argtypes = [ctypes.c_void_p]
        _lib = L
    return _lib


class RawDeviceBlock:
    """One hipMalloc'd block of exactly ``nbytes`` (its own allocation, not a slice of a cached
    segment); ``ptr`` is the device address.  Freed with the object."""

    def __init__(self, nbytes):
        p = ctypes.c_void_p()
        rc = _load().pier_inputs_device_alloc(ctypes.byref(p), nbytes)
        if rc != 0 or not p.value:
            raise MemoryError("hipMalloc of %d bytes failed with hipError %d" % (nbytes, rc))
        self.ptr, self.nbytes = p.value, nbytes

    def __del__(self):
        if getattr(self, "ptr", None):
            _load().pier_inputs_device_free(self.ptr)
            self.ptr = None


class _PinnedBlock:
    """Owner of one hipHostMalloc'd block; the tensor made from it keeps this object alive."""

    def __init__(self, nbytes):
        p = ctypes.c_void_p()
        rc = _load().pier_inputs_host_alloc(ctypes.byref(p), nbytes)
        if rc != 0 or not p.value:
            raise MemoryError("hipHostMalloc of %d bytes failed with hipError %d" % (nbytes, rc))
        self.ptr, self.nbytes = p.value, nbytes

    def __del__(self):
        if getattr(self, "ptr", None):
            _load().pier_inputs_host_free(self.ptr)
            self.ptr = None


def pinned_empty(numel, dtype=torch.float32):
    """A host tensor in pinned memory of exactly numel elements (no rounding of the request,
    unlike torch's pinned allocator); torch does not know it is pinned, HIP does."""
    import numpy as np
    esize = torch.empty(0, dtype=dtype).element_size()
    block = _PinnedBlock(max(1, numel) * esize)
    raw = (ctypes.c_uint8 * block.nbytes).from_address(block.ptr)
    raw._pier_owner = block                     # the ctypes array is the numpy array's base
    t = torch.from_numpy(np.frombuffer(raw, dtype=np.uint8)).view(dtype)[:max(1, numel)]
    return t


def fill_normal(t, *, seed, stream, step, std, first_elem=0, hip_stream=None):
    """Fills the contiguous device tensor ``t`` (float32 or bfloat16) with elements
    [first_elem, first_elem + t.numel()) of draw (seed, stream, step)."""
    assert t.is_cuda and t.is_contiguous() and t.dtype in (torch.float32, torch.bfloat16)
    s = hip_stream if hip_stream is not None else torch.cuda.current_stream()
    rc = _load().pier_inputs_fill_normal(t.data_ptr(), t.numel(), first_elem,
                                         1 if t.dtype == torch.bfloat16 else 0, seed, stream, step, std,
                                         s.cuda_stream or None)
    if rc != 0:
        raise RuntimeError("pier_inputs_fill_normal failed with hipError %d" % rc)
    return t


class FlatList:
    """A tensor list carved out of one flat device allocation: ``flat`` is the whole
    buffer, ``tensors[i]`` a view of numel[i] elements.  Each tensor starts on a
    16-byte boundary when every numel is a multiple of 4 (true for the GPT shapes);
    ``pad`` > 0 inserts that many unused elements between tensors."""

    def __init__(self, numels, dtype=torch.float32, device="cuda", pad=0, zero=True, pinned=False):
        self.numels = list(numels)
        self.starts = []
        off = 0
        for n in self.numels:
            self.starts.append(off)
            off += n + pad
        total = max(off, 1)
        if pinned:
            self.flat = pinned_empty(total, dtype)
            if zero:
                self.flat.zero_()
        else:
            self.flat = (torch.zeros if zero else torch.empty)(total, dtype=dtype, device=device)
        self.tensors = [self.flat[s:s + n] for s, n in zip(self.starts, self.numels)]

    @classmethod
    def wrap(cls, flat, numels, address_class=None):
        """A tensor list over an existing flat buffer (tensors back to back, no padding)."""
        fl = cls.__new__(cls)
        fl.numels = list(numels)
        fl.starts, off = [], 0
        for n in fl.numels:
            fl.starts.append(off)
            off += n
        assert flat.numel() >= max(off, 1)
        fl.flat = flat
        fl.cls = address_class
        fl.tensors = [flat[s:s + n] for s, n in zip(fl.starts, fl.numels)]
        return fl

    def fill_normal(self, *, seed, stream, step, std, hip_stream=None):
        """One draw over the flat buffer (padding included), so element e of the
        buffer is element e of the draw."""
        fill_normal(self.flat, seed=seed, stream=stream, step=step, std=std, hip_stream=hip_stream)
        return self


def init_params(flat_list, w):
    """Parameters ~ N(0, param_std) from the workload's seed."""
    return flat_list.fill_normal(seed=w.seed, stream=shapes.PARAM_STREAM, step=0, std=w.param_std)
