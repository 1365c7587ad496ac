"""ctypes binding of libpier.so.  Functions carry the names of include/pier.h and do
argument marshalling only: lists of torch tensors become arrays of device pointers,
streams become hipStream_t handles, status codes become exceptions.  Every step of
the optimizer path runs in the HIP library."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpier.so")

PIER_PHASE_WARMUP, PIER_PHASE_PIER = 0, 1
PIER_LOC_DEVICE, PIER_LOC_HOST_PINNED = 0, 1
PIER_MODE_PIER, PIER_MODE_DILOCO = 0, 1


class PierError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (status, message))
        self.status = status


class AdamwHP(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("step", ctypes.c_int64)]


class OuterHP(ctypes.Structure):
    _fields_ = [("outer_lr", ctypes.c_float), ("mu", ctypes.c_float), ("phase", ctypes.c_int)]


class TrainCfg(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("r", ctypes.c_int64), ("mode", ctypes.c_int),
                ("lr_max", ctypes.c_float), ("lr_min", ctypes.c_float), ("warmup_frac", ctypes.c_double),
                ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("clip_norm", ctypes.c_float),
                ("chunk_bytes", ctypes.c_size_t), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("h2d_stream", ctypes.c_void_p),
                ("d2h_stream", ctypes.c_void_p)]


class OffloadStats(ctypes.Structure):
    _fields_ = [("h2d_bytes", ctypes.c_double), ("d2h_bytes", ctypes.c_double),
                ("h2d_ms", ctypes.c_double), ("d2h_ms", ctypes.c_double),
                ("kernel_ms", ctypes.c_double), ("wall_ms", ctypes.c_double),
                ("n_pieces", ctypes.c_int), ("n_slots", ctypes.c_int), ("compute_ms", ctypes.c_double)]


_lib = None


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        # nothing built yet: build once (hipcc cross-compiles without a GPU); there is no
        # other implementation to fall back to, so a failed build is a hard error
        try:
            from . import build as _build
            _build.build()
        except Exception as e:
            raise ImportError("libpier.so is not built and building it failed (%s): run "
                              "`python -m paper_2511_17849_amd.build`; there is no fallback path" % e)
    # torch ships its own HIP runtime; import it first so that libpier binds to the
    # runtime that owns torch's allocations and streams
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    pp = ctypes.POINTER(ctypes.c_void_p)
    sig = {
        "pier_abi_version": (i32, []),
        "pier_last_error": (ctypes.c_char_p, []),
        "pier_status_string": (ctypes.c_char_p, [i32]),
        "pier_ctx_create": (i32, [ctypes.POINTER(vp), i32, ctypes.POINTER(i64), i32]),
        "pier_ctx_destroy": (i32, [vp]),
        "pier_ctx_numel": (i64, [vp]),
        "pier_ctx_set_launch": (i32, [vp, i64, i32, i32, i32]),
        "pier_ctx_set_occupancy": (i32, [vp, i32, i32]),
        "pier_ctx_set_offload_writeback": (i32, [vp, i32]),
        "pier_placement_plan": (i32, [i32, ctypes.POINTER(i64), i32, i32, i32, vp,
                                      ctypes.POINTER(i32), ctypes.POINTER(i32)]),
        "pier_bind_replica": (i32, [vp, i32, pp, pp, pp, pp, i32]),
        "pier_bind_shadow": (i32, [vp, i32, pp]),
        "pier_bind_outer": (i32, [vp, i32, pp, pp]),
        "pier_inner_adamw": (i32, [vp, i32, ctypes.POINTER(AdamwHP), vp]),
        "pier_inner_adamw_clipped": (i32, [vp, i32, ctypes.POINTER(AdamwHP), f32, vp]),
        "pier_inner_adamw_clipped_static": (i32, [vp, i32, ctypes.POINTER(AdamwHP), f32, vp]),
        "pier_ctx_set_norm_fold": (i32, [vp, i32]),
        "pier_grad_norm_last": (i32, [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(f32), vp]),
        "pier_outer_step": (i32, [vp, ctypes.POINTER(OuterHP), vp]),
        "pier_offload_workspace_bytes": (i32, [vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]),
        "pier_offload_stream": (i32, [vp, ctypes.POINTER(OuterHP), ctypes.c_size_t, vp, ctypes.c_size_t,
                                      vp, vp, vp, ctypes.POINTER(OffloadStats)]),
        "pier_hbm_probe": (i32, [vp, ctypes.c_size_t, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int32), i32, vp]),
        "pier_hbm_probe_summary": (i32, [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]),
        "pier_hbm_classify": (i32, [ctypes.POINTER(ctypes.c_double), i32, ctypes.POINTER(ctypes.c_int32)]),
        "pier_mu_schedule": (f32, [i64, i64]),
        "pier_outer_lr_schedule": (f32, [i64, i64]),
        "pier_outer_schedule": (i32, [i64, i64, ctypes.POINTER(OuterHP)]),
        "pier_inner_lr_schedule": (f32, [i64, i64, f32, f32, ctypes.c_double]),
        "pier_train_step": (i32, [vp, ctypes.POINTER(TrainCfg), i64, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    if L.pier_abi_version() != ABI_VERSION:
        raise ImportError("libpier.so has ABI version %d, this binding expects %d: rebuild with "
                          "`python -m paper_2511_17849_amd.build`" % (L.pier_abi_version(), ABI_VERSION))
    _lib = L
    return L


def pier_last_error():
    return _load().pier_last_error().decode()


def pier_status_string(status):
    return _load().pier_status_string(int(status)).decode()


def _check(status):
    if status != 0:
        raise PierError(pier_status_string(status), pier_last_error())


class PierCtx:
    """Handle of a pier_ctx.  Keeps the bound tensors alive."""

    def __init__(self, handle):
        self.handle = handle
        self._keep = {}

    def __del__(self):
        try:
            pier_ctx_destroy(self)
        except Exception:
            pass


def _ptr_array(items):
    """Host array of pointers from torch tensors, raw ints or None."""
    vals = []
    for x in items:
        if x is None:
            vals.append(None)
        elif isinstance(x, int):
            vals.append(x or None)
        else:
            vals.append(x.data_ptr() or None)
    return (ctypes.c_void_p * len(vals))(*vals)


def _stream(s):
    """hipStream_t of a torch.cuda.Stream, a raw handle, or None (null stream)."""
    if s is None:
        return None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


def pier_ctx_create(numel, n_replicas):
    L = _load()
    arr = (ctypes.c_int64 * len(numel))(*[int(n) for n in numel])
    h = ctypes.c_void_p()
    _check(L.pier_ctx_create(ctypes.byref(h), len(numel), arr, int(n_replicas)))
    return PierCtx(h)


def pier_ctx_destroy(ctx):
    if ctx.handle:
        h, ctx.handle = ctx.handle, None
        ctx._keep.clear()
        _check(_load().pier_ctx_destroy(h))


def pier_ctx_numel(ctx):
    return _load().pier_ctx_numel(ctx.handle)


def pier_ctx_set_launch(ctx, chunk_elems=0, unroll=0, max_grid=0, nontemporal=-1):
    _check(_load().pier_ctx_set_launch(ctx.handle, int(chunk_elems), int(unroll), int(max_grid),
                                       int(nontemporal)))


def pier_ctx_set_offload_writeback(ctx, trailing):
    _check(_load().pier_ctx_set_offload_writeback(ctx.handle, int(trailing)))


def pier_ctx_set_occupancy(ctx, wg_threads=0, lds_bytes=-1):
    _check(_load().pier_ctx_set_occupancy(ctx.handle, int(wg_threads), int(lds_bytes)))


# The keep-alive references are replaced only after the library has accepted the new
# pointers: after a failed re-bind it still uses the old ones.
def pier_bind_replica(ctx, replica, p, m, v, grad, grad_is_bf16=False):
    keep = (list(p), list(m), list(v), list(grad))
    _check(_load().pier_bind_replica(ctx.handle, int(replica), _ptr_array(p), _ptr_array(m),
                                     _ptr_array(v), _ptr_array(grad), 1 if grad_is_bf16 else 0))
    ctx._keep[("rep", replica)] = keep


def pier_bind_shadow(ctx, replica, w_bf16):
    """w_bf16: list of bfloat16 device tensors (one per model tensor), or None to unbind."""
    keep = list(w_bf16) if w_bf16 is not None else None
    _check(_load().pier_bind_shadow(ctx.handle, int(replica), _ptr_array(w_bf16) if w_bf16 is not None else None))
    ctx._keep[("shadow", replica)] = keep


def pier_bind_outer(ctx, loc, anchor, momentum):
    if loc == PIER_LOC_HOST_PINNED and not isinstance(anchor, (list, tuple)):
        anchor, momentum = [anchor], [momentum]
    keep = (list(anchor), list(momentum))
    _check(_load().pier_bind_outer(ctx.handle, int(loc), _ptr_array(anchor), _ptr_array(momentum)))
    ctx._keep["outer"] = keep


def pier_inner_adamw(ctx, replica, *, lr, beta1, beta2, eps, weight_decay, step, grad_scale=1.0,
                     stream=None):
    hp = AdamwHP(lr, beta1, beta2, eps, weight_decay, grad_scale, int(step))
    _check(_load().pier_inner_adamw(ctx.handle, int(replica), ctypes.byref(hp), _stream(stream)))


def pier_inner_adamw_clipped(ctx, replica, *, lr, beta1, beta2, eps, weight_decay, step, max_norm,
                             grad_scale=1.0, stream=None):
    hp = AdamwHP(lr, beta1, beta2, eps, weight_decay, grad_scale, int(step))
    _check(_load().pier_inner_adamw_clipped(ctx.handle, int(replica), ctypes.byref(hp), max_norm,
                                            _stream(stream)))


def pier_inner_adamw_clipped_static(ctx, replica, *, lr, beta1, beta2, eps, weight_decay, step, max_norm,
                                    grad_scale=1.0, stream=None):
    hp = AdamwHP(lr, beta1, beta2, eps, weight_decay, grad_scale, int(step))
    _check(_load().pier_inner_adamw_clipped_static(ctx.handle, int(replica), ctypes.byref(hp), max_norm,
                                                   _stream(stream)))


def pier_ctx_set_norm_fold(ctx, n_partials=0):
    _check(_load().pier_ctx_set_norm_fold(ctx.handle, int(n_partials)))


def pier_grad_norm_last(ctx, replica, stream=None):
    """(norm, coefficient) of the replica's latest clipped step; synchronises the stream."""
    norm, coef = ctypes.c_double(), ctypes.c_float()
    _check(_load().pier_grad_norm_last(ctx.handle, int(replica), ctypes.byref(norm), ctypes.byref(coef),
                                       _stream(stream)))
    return norm.value, coef.value


def pier_outer_step(ctx, *, outer_lr, mu, phase, stream=None):
    hp = OuterHP(outer_lr, mu, int(phase))
    _check(_load().pier_outer_step(ctx.handle, ctypes.byref(hp), _stream(stream)))


def pier_offload_workspace_bytes(ctx, chunk_bytes):
    out = ctypes.c_size_t()
    _check(_load().pier_offload_workspace_bytes(ctx.handle, int(chunk_bytes), ctypes.byref(out)))
    return out.value


def pier_offload_stream(ctx, *, outer_lr, mu, phase, chunk_bytes, workspace, compute_stream=None,
                        h2d_stream=None, d2h_stream=None, want_stats=False):
    """workspace: a torch uint8/float tensor on the device (or (ptr, nbytes))."""
    hp = OuterHP(outer_lr, mu, int(phase))
    if isinstance(workspace, tuple):
        wptr, wbytes = workspace
    else:
        wptr, wbytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    stats = OffloadStats() if want_stats else None
    _check(_load().pier_offload_stream(ctx.handle, ctypes.byref(hp), int(chunk_bytes), wptr or None,
                                       int(wbytes), _stream(compute_stream), _stream(h2d_stream),
                                       _stream(d2h_stream), ctypes.byref(stats) if want_stats else None))
    return stats


ABI_VERSION = 3     # PIER_ABI_VERSION of the header this binding was written against


def pier_abi_version():
    return _load().pier_abi_version()


def pier_placement_plan(room, n_replicas, shared_grad=False, outer_on_device=True):
    """Address class of every model-sized buffer.  ``room[c]``: buffers class c still holds.
    Returns (replicas, anchor_class, momentum_class), replicas a list of dicts with the keys
    theta, m, v, grad; the two classes are -1 when the outer state is not on the device."""
    room = [int(r) for r in room]
    arr = (ctypes.c_int64 * len(room))(*room)
    rep = (ctypes.c_int32 * (4 * int(n_replicas)))()
    a, m = ctypes.c_int32(), ctypes.c_int32()
    _check(_load().pier_placement_plan(len(room), arr, int(n_replicas), int(bool(shared_grad)),
                                       int(bool(outer_on_device)), ctypes.cast(rep, ctypes.c_void_p),
                                       ctypes.byref(a), ctypes.byref(m)))
    reps = [dict(theta=rep[4 * g], m=rep[4 * g + 1], v=rep[4 * g + 2], grad=rep[4 * g + 3])
            for g in range(int(n_replicas))]
    return reps, a.value, m.value


def pier_hbm_probe(arena, granule_bytes, stream=None):
    """Class id of every granule of the device tensor ``arena`` (its contents are overwritten)."""
    nbytes = arena.numel() * arena.element_size()
    n = int(nbytes // granule_bytes)
    out = (ctypes.c_int32 * max(n, 1))()
    _check(_load().pier_hbm_probe(arena.data_ptr() or None, nbytes, int(granule_bytes), out, n, _stream(stream)))
    return list(out[:n])


def pier_hbm_probe_summary():
    """dict(best_rate, threshold, n_classes, n_pairs) of this thread's latest probe / classification."""
    b, t = ctypes.c_double(), ctypes.c_double()
    c, n = ctypes.c_int32(), ctypes.c_int32()
    _check(_load().pier_hbm_probe_summary(ctypes.byref(b), ctypes.byref(t), ctypes.byref(c), ctypes.byref(n)))
    return dict(best_rate=b.value, threshold=t.value, n_classes=c.value, n_pairs=n.value)


def pier_hbm_classify(rates):
    """Class id of every granule from a full table of pair rates (n x n nested lists or array)."""
    rows = [list(map(float, row)) for row in rates]
    n = len(rows)
    flat = (ctypes.c_double * (n * n))(*[x for row in rows for x in row])
    out = (ctypes.c_int32 * max(n, 1))()
    _check(_load().pier_hbm_classify(flat, n, out))
    return list(out[:n])


def pier_mu_schedule(t, T):
    return _load().pier_mu_schedule(int(t), int(T))


def pier_outer_lr_schedule(t, T):
    return _load().pier_outer_lr_schedule(int(t), int(T))


def pier_inner_lr_schedule(t, T, lr_max, lr_min, warmup_frac=0.02):
    return _load().pier_inner_lr_schedule(int(t), int(T), lr_max, lr_min, warmup_frac)


def pier_train_step(ctx, t, *, T, r, mode=PIER_MODE_PIER, lr_max, lr_min, warmup_frac=0.02, beta1, beta2, eps,
                    weight_decay, clip_norm=0.0, chunk_bytes=0, workspace=None, h2d_stream=None,
                    d2h_stream=None, stream=None):
    wptr = workspace.data_ptr() if workspace is not None else None
    wbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    cfg = TrainCfg(int(T), int(r), int(mode), lr_max, lr_min, warmup_frac, beta1, beta2, eps, weight_decay,
                   clip_norm, int(chunk_bytes), wptr, wbytes, _stream(h2d_stream), _stream(d2h_stream))
    _check(_load().pier_train_step(ctx.handle, ctypes.byref(cfg), int(t), _stream(stream)))


def pier_outer_schedule(t, T):
    hp = OuterHP()
    _check(_load().pier_outer_schedule(int(t), int(T), ctypes.byref(hp)))
    return hp
