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
            raise ImportError("libpier_inputs.so is not built: run `python -m pier_inputs.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.pier_inputs_fill_normal.restype = ctypes.c_int
        L.pier_inputs_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                              ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                              ctypes.c_float, ctypes.c_void_p]
        _lib = L
    return _lib


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
            self.flat = torch.empty(total, dtype=dtype, pin_memory=True)
            if zero:
                self.flat.zero_()
        else:
            self.flat = (torch.zeros if zero else torch.empty)(total, dtype=dtype, device=device)
        self.tensors = [self.flat[s:s + n] for s, n in zip(self.starts, self.numels)]

    def fill_normal(self, *, seed, stream, step, std, hip_stream=None):
        """One draw over the flat buffer (padding included), so element e of the
        buffer is element e of the draw."""
        fill_normal(self.flat, seed=seed, stream=stream, step=step, std=std, hip_stream=hip_stream)
        return self


def init_params(flat_list, w):
    """Parameters ~ N(0, param_std) from the workload's seed."""
    return flat_list.fill_normal(seed=w.seed, stream=shapes.PARAM_STREAM, step=0, std=w.param_std)
