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

    def fill_normal(self, *, seed, stream, step, std, hip_stream=None):
        """One draw over the flat buffer (padding included), so element e of the
        buffer is element e of the draw."""
        fill_normal(self.flat, seed=seed, stream=stream, step=step, std=std, hip_stream=hip_stream)
        return self


def init_params(flat_list, w):
    """Parameters ~ N(0, param_std) from the workload's seed."""
    return flat_list.fill_normal(seed=w.seed, stream=shapes.PARAM_STREAM, step=0, std=w.param_std)


class PlacedState:
    """All buffers of one workload - theta, m, v, gradient per replica, anchor and M -
    as FlatLists.  With ``arena`` (a paper_2511_17849_amd.HbmArena) the buffers are carved
    out of it by address class.  Measured on MI355X at GPT-2 XL size: a launch streams fastest
    when its buffers lie in exactly two classes, half in each - for the AdamW launch theta_g, m_g
    in one class and v_g, grad_g in another (6.40-6.55 TB/s against 6.33-6.39 with one buffer per
    class and 5.6-6.1 with all four in one), for the outer step the G thetas, the anchor and M
    split five and five over two classes (6.47-6.54 TB/s against 6.35-6.42 over three classes).
      policy "two_class" (default): the library's pier_placement_plan - theta_g and m_g, back to
        back, in class g mod 2; the anchor and M in whichever of classes 0 and 1 then holds fewer
        of the outer step's buffers; v_g and grad_g, back to back, in class 2 while it has room,
        else in the class of {0, 1} theta_g is not in.
      policy "pairs": theta_g, m_g in class g mod 3, v_g, grad_g in class (g + 1) mod 3, anchor
        and M where the fewest thetas are (the outer step's buffers then span three classes).
      policy "spread": class(theta_g) = g, class(m_g) = g + 1, class(v_g) = g + 2, class(grad_g) = g.
    With fewer classes than a policy names, classes are taken modulo their number.  Without an
    arena the buffers are separate allocations made kind by kind.
    outer="device" | "pinned" | None places anchor and M on the device, in pinned host
    memory (flat arrays for the offload path), or nowhere."""

    def __init__(self, numels, G, grad_dtype=torch.float32, arena=None, outer="device", shared_grad=False,
                 policy="two_class"):
        self.numels = list(numels)
        N = sum(self.numels)
        ncls = arena.n_classes if arena is not None else 1

        def make(dtype, cls):
            fl = FlatList.__new__(FlatList)
            fl.numels = list(self.numels)
            fl.starts, off = [], 0
            for n in fl.numels:
                fl.starts.append(off)
                off += n
            if arena is None:
                fl.flat = torch.empty(max(N, 1), dtype=dtype, device="cuda")
                fl.cls = None
            else:
                fl.flat, fl.cls = arena.alloc(max(N, 1), dtype, cls)
            fl.tensors = [fl.flat[s:s + n] for s, n in zip(fl.starts, fl.numels)]
            return fl

        def make_outer(classes_of_theta, candidates):
            if outer == "device":
                load = {c: sum(1 for x in classes_of_theta if x == c) for c in candidates}
                ca = min(candidates, key=lambda c: load[c])
                load[ca] += 1
                cm = min(candidates, key=lambda c: load[c])
                self.A, self.Mo = make(torch.float32, ca), make(torch.float32, cm)
            elif outer == "pinned":
                self.A = FlatList(self.numels, pinned=True, zero=False)
                self.Mo = FlatList(self.numels, pinned=True, zero=False)
            else:
                self.A = self.Mo = None

        self.P, self.M1, self.V, self.Gd = [], [], [], []
        if policy == "two_class":
            # the library's own plan (pier_placement_plan), followed in the order it was made
            if arena is not None:
                from paper_2511_17849_amd import binding as _pier
                plan, ca, cm = _pier.pier_placement_plan(arena.room(max(N, 1)), G, shared_grad, outer == "device")
            else:
                plan, ca, cm = [dict(theta=None, m=None, v=None, grad=None)] * G, None, None
            for g in range(G):          # theta_g and m_g back to back
                self.P.append(make(torch.float32, plan[g]["theta"]))
                self.M1.append(make(torch.float32, plan[g]["m"]))
            if outer == "device":
                self.A, self.Mo = make(torch.float32, ca), make(torch.float32, cm)
            elif outer == "pinned":
                self.A = FlatList(self.numels, pinned=True, zero=False)
                self.Mo = FlatList(self.numels, pinned=True, zero=False)
            else:
                self.A = self.Mo = None
            shared = None
            for g in range(G):          # v_g and grad_g back to back
                self.V.append(make(torch.float32, plan[g]["v"]))
                if shared_grad:
                    shared = shared or make(grad_dtype, plan[g]["grad"])
                    self.Gd.append(shared)
                else:
                    self.Gd.append(make(grad_dtype, plan[g]["grad"]))
        else:
            if policy == "pairs":
                kp, km, kv, kg = 0, 0, 1, 1
            elif policy == "spread":
                kp, km, kv, kg = 0, 1, 2, 0
            else:
                raise ValueError("unknown placement policy %r" % (policy,))
            for g in range(G):
                self.P.append(make(torch.float32, g + kp))
                self.M1.append(make(torch.float32, g + km))
            for g in range(G):
                self.V.append(make(torch.float32, g + kv))
            make_outer([g % ncls for g in range(G)], list(range(ncls)))
            if shared_grad:
                self.Gd = [make(grad_dtype, kg)] * G
            else:
                self.Gd = [make(grad_dtype, g + kg) for g in range(G)]
        for fl in self.M1 + self.V + ([self.Mo] if self.Mo is not None else []):
            fl.flat.zero_()
