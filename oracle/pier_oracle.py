"""ctypes front end of the CPU oracle (oracle/pier_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and
by the ``cpu_baseline`` leg of ``bench.py``.  It neither imports nor is imported
by the HIP package.  All arrays are contiguous numpy arrays updated in place.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pier_oracle.c")
_LIB = os.path.join(_HERE, "libpier_oracle.so")

# No FMA contraction, no reassociation: one IEEE binary32 operation per
# operator, in source order.
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fno-unsafe-math-optimizations",
          "-shared", "-fPIC", "-Wall", "-Wextra"]

WARMUP, PIER = 0, 1


def build(force=False):
    """Compile the oracle with gcc; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Oracle:
    """The oracle's functions bound to one compiled library (the default build, or
    a deliberately broken copy a test compiled to check that the pins notice)."""
    WARMUP, PIER = WARMUP, PIER

    def __init__(self, path=None):
        L = ctypes.CDLL(path or build())
        f32p = ctypes.POINTER(ctypes.c_float)
        i64, f32, i32 = ctypes.c_int64, ctypes.c_float, ctypes.c_int
        L.pier_oracle_adamw.argtypes = [f32p, f32p, f32p, f32p, i64, f32, f32, f32, f32, f32, i64, f32]
        L.pier_oracle_adamw.restype = None
        L.pier_oracle_adamw_bf16.argtypes = [f32p, f32p, f32p, ctypes.POINTER(ctypes.c_uint16), i64,
                                             f32, f32, f32, f32, f32, i64, f32]
        L.pier_oracle_adamw_bf16.restype = None
        L.pier_oracle_outer.argtypes = [ctypes.POINTER(f32p), i32, f32p, f32p, i64, f32, f32, i32]
        L.pier_oracle_outer.restype = None
        L.pier_oracle_phase.argtypes = [i64, i64]
        L.pier_oracle_phase.restype = i32
        L.pier_oracle_mu.argtypes = [i64, i64]
        L.pier_oracle_mu.restype = f32
        L.pier_oracle_outer_lr.argtypes = [i64, i64]
        L.pier_oracle_outer_lr.restype = f32
        L.pier_oracle_outer_scalars.argtypes = [i64, i64, ctypes.POINTER(i32), f32p, f32p]
        L.pier_oracle_outer_scalars.restype = None
        f64 = ctypes.c_double
        L.pier_oracle_sumsq.argtypes = [f32p, i64, f64]
        L.pier_oracle_sumsq.restype = f64
        L.pier_oracle_sumsq_bf16.argtypes = [ctypes.POINTER(ctypes.c_uint16), i64, f64]
        L.pier_oracle_sumsq_bf16.restype = f64
        L.pier_oracle_clip_coef.argtypes = [f64, f32]
        L.pier_oracle_clip_coef.restype = f32
        L.pier_oracle_inner_lr.argtypes = [i64, i64, f32, f32, f64]
        L.pier_oracle_inner_lr.restype = f32
        L.pier_oracle_to_bf16.argtypes = [f32p, ctypes.POINTER(ctypes.c_uint16), i64]
        L.pier_oracle_to_bf16.restype = None
        self._L = L

    def adamw(self, p, m, v, g, *, lr, beta1, beta2, eps, weight_decay, step, grad_scale=1.0):
        """One inner AdamW step, in place on p, m, v.  ``g`` is float32, or uint16
        holding bfloat16 bit patterns."""
        n = p.size
        assert m.size == n and v.size == n and g.size == n
        if g.dtype == np.uint16:
            assert g.flags.c_contiguous
            self._L.pier_oracle_adamw_bf16(_f32(p), _f32(m), _f32(v),
                                           g.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), n,
                                           lr, beta1, beta2, eps, weight_decay, step, grad_scale)
        else:
            self._L.pier_oracle_adamw(_f32(p), _f32(m), _f32(v), _f32(g), n,
                                      lr, beta1, beta2, eps, weight_decay, step, grad_scale)

    def outer(self, thetas, a, M, *, mu, lr, phase):
        """One outer step over the list ``thetas`` of group models, in place."""
        G = len(thetas)
        n = a.size
        assert G >= 1 and M.size == n and all(t.size == n for t in thetas)
        arr = (ctypes.POINTER(ctypes.c_float) * G)(*[_f32(t) for t in thetas])
        self._L.pier_oracle_outer(arr, G, _f32(a), _f32(M), n, mu, lr, int(phase))

    def sumsq(self, g, acc=0.0):
        """acc + sum of squares of the gradient array g (float32, or uint16 bfloat16 bits),
        accumulated in double in index order; chain calls over a tensor list."""
        if g.dtype == np.uint16:
            assert g.flags.c_contiguous
            return self._L.pier_oracle_sumsq_bf16(g.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), g.size, acc)
        return self._L.pier_oracle_sumsq(_f32(g), g.size, acc)

    def clip_coef(self, sumsq, max_norm):
        """fp32 factor the gradients are multiplied by: min(1, max_norm / (sqrt(sumsq) + 1e-6))."""
        return self._L.pier_oracle_clip_coef(sumsq, max_norm)

    def to_bf16(self, x):
        """bfloat16 bit patterns (uint16) of the float32 array x, round to nearest even."""
        out = np.empty(x.size, np.uint16)
        self._L.pier_oracle_to_bf16(_f32(x), out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), x.size)
        return out

    def phase(self, t, T):
        return self._L.pier_oracle_phase(t, T)

    def mu(self, t, T):
        return self._L.pier_oracle_mu(t, T)

    def outer_lr(self, t, T):
        return self._L.pier_oracle_outer_lr(t, T)

    def inner_lr(self, t, T, lr_max, lr_min, warmup_frac=0.02):
        return self._L.pier_oracle_inner_lr(t, T, lr_max, lr_min, warmup_frac)

    def outer_scalars(self, t, T):
        """(phase, mu, lr) that the synchronisation at iteration t of T uses."""
        ph, m_, l_ = ctypes.c_int(), ctypes.c_float(), ctypes.c_float()
        self._L.pier_oracle_outer_scalars(t, T, ctypes.byref(ph), ctypes.byref(m_), ctypes.byref(l_))
        return ph.value, m_.value, l_.value


def _f32(a):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous):
        raise TypeError("oracle arrays must be contiguous float32 numpy arrays")
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


_default = None


def default():
    """The oracle every module-level function below uses: the library built from pier_oracle.c
    with CFLAGS, or the one PIER_ORACLE_LIB names (another build of the same source, e.g. the
    instrumented one tests/test_oracle_sanitized.py makes)."""
    global _default
    if _default is None:
        _default = Oracle(os.environ.get("PIER_ORACLE_LIB") or None)
    return _default


def adamw(*a, **k):
    return default().adamw(*a, **k)


def outer(*a, **k):
    return default().outer(*a, **k)


def sumsq(g, acc=0.0):
    return default().sumsq(g, acc)


def clip_coef(sumsq_, max_norm):
    return default().clip_coef(sumsq_, max_norm)


def to_bf16(x):
    return default().to_bf16(x)


def phase(t, T):
    return default().phase(t, T)


def mu(t, T):
    return default().mu(t, T)


def outer_lr(t, T):
    return default().outer_lr(t, T)


def outer_scalars(t, T):
    return default().outer_scalars(t, T)


def inner_lr(t, T, lr_max, lr_min, warmup_frac=0.02):
    return default().inner_lr(t, T, lr_max, lr_min, warmup_frac)
