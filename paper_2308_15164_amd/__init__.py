"""MI355X-native ABS-SGD data-parallel hot path: thin Python binding.

Every function here has the name and the meaning of the C entry point declared
in ``include/abs_sgd.h`` and does argument marshalling only: tensors become
device pointers, streams become ``hipStream_t`` handles, return codes become
Python values or exceptions.  All arithmetic runs in the HIP kernels of
``libabs_sgd.so``; there is no fallback path, and importing the module fails
loudly when the library has not been built.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# ABS_SGD_LIB points the binding at another build of the same library (tuning variants)
LIB_PATH = os.environ.get("ABS_SGD_LIB") or os.path.join(_HERE, "libabs_sgd.so")

ABS_OK, ABS_EMPTY, ABS_EINVAL, ABS_EHIP = 0, 1, -1, -2
ABS_F32, ABS_BF16 = 0, 1
ABS_MAX_K = 64

# name -> (restype, argtypes): every symbol include/abs_sgd.h declares
_vp, _i64, _int, _f = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
_pi64 = ctypes.POINTER(ctypes.c_int64)
_pvp = ctypes.POINTER(ctypes.c_void_p)
SYMBOLS = {
    "abs_version": (_int, []),
    "abs_last_hip_error": (_int, []),
    "abs_error_string": (ctypes.c_char_p, [_int]),
    "abs_row_elems": (_i64, []),
    "abs_set_launch_tuning": (_int, [_int, _int]),
    "abs_set_launch_slice_bytes": (_int, [_i64]),
    "abs_launch_count": (_i64, []),
    "abs_slice_workgroups": (_i64, [_i64, _i64, _int]),
    "abs_set_cache_policy": (_int, [_int, _int]),
    "abs_accumulate": (_int, [_vp, _vp, _int, _i64, _i64, _pi64, _vp]),
    "abs_accumulate_batch": (_int, [_vp, _pvp, _int, _int, _i64, _pi64, _pi64, _vp]),
    "abs_accumulate_jobs": (_int, [_vp, _int, _int, _i64, _int, _vp]),
    "abs_accumulate_jobs_mt": (_int, [_vp, _vp, _int, _int, _vp]),
    "abs_layout_upload": (_int, [_vp]),
    "abs_ctx_set_launch_tuning": (_int, [_vp, _int, _int]),
    "abs_ctx_set_cache_policy": (_int, [_vp, _int, _int]),
    "abs_ctx_accumulate_step": (_int, [_vp, _pvp, ctypes.POINTER(ctypes.c_int), _pi64, _int, _int]),
    "abs_ctx_accumulate_step_mt": (_int, [_vp, _pvp, ctypes.POINTER(ctypes.c_int), _pi64, _int]),
    "abs_sync_update": (_int, [_vp, _vp, _pvp, _pi64, _int, _i64, _f, _f, _f, _vp]),
    "abs_sync_update_dc": (_int, [_vp, _vp, _vp, _pvp, _pi64, _int, _i64, _f, _f, _f, _f, _vp]),
    "abs_sync_update_adam": (_int, [_vp, _vp, _vp, _pvp, _pi64, _int, _i64, _f, _f, _f, _f, _f, _i64, _vp]),
    "abs_layout_create": (_int, [_pvp, _int, _pi64]),
    "abs_layout_destroy": (_int, [_vp]),
    "abs_layout_num_tensors": (_int, [_vp]),
    "abs_layout_total": (_i64, [_vp]),
    "abs_layout_num_chunks": (_i64, [_vp]),
    "abs_layout_tile": (_i64, [_vp]),
    "abs_layout_chunk": (_int, [_vp, _i64, ctypes.POINTER(_int), _pi64, _pi64]),
    "abs_tensorset_create": (_int, [_pvp, _vp, _pvp, _int]),
    "abs_tensorset_destroy": (_int, [_vp]),
    "abs_accumulate_mt": (_int, [_vp, _vp, _vp, _i64, _pi64, _vp]),
    "abs_accumulate_batch_mt": (_int, [_vp, _vp, _pvp, _int, _pi64, _pi64, _vp]),
    "abs_sync_update_mt": (_int, [_vp, _vp, _vp, _pvp, _pi64, _int, _f, _f, _f, _vp]),
    "abs_suggest_accumulate_streams": (_int, [_i64, _int]),
    "abs_sync_update_dcm": (_int, [_vp, _vp, _pvp, _pi64, _int, _i64, _f, _f, _f, _f, _f, _vp]),
    "abs_sync_update_dcm_mt": (_int, [_vp, _vp, _vp, _pvp, _pi64, _int, _f, _f, _f, _f, _f, _vp]),
    "abs_ctx_sync_update_dcm": (_int, [_vp, _vp, _vp, _f, _f, _f, _f]),
    "abs_ctx_sync_update_dcm_mt": (_int, [_vp, _vp, _vp, _f, _f, _f, _f]),
    "abs_sync_update_dc_mt": (_int, [_vp, _vp, _vp, _vp, _pvp, _pi64, _int, _f, _f, _f, _f, _vp]),
    "abs_sync_update_adam_mt": (_int, [_vp, _vp, _vp, _vp, _pvp, _pi64, _int, _f, _f, _f, _f, _f, _i64, _vp]),
    "abs_sync_update_lars_mt": (_int, [_vp, _vp, _vp, _vp, _pvp, _pi64, _int, _f, _f, _f, _f, _vp]),
    "abs_sync_update_lars_mt_noalloc": (_int, [_vp, _vp, _vp, _vp, _pvp, _pi64, _int, _f, _f, _f, _f, _vp]),
    "abs_ctx_create": (_int, [_pvp, _int, _i64, _pvp, _pvp, _vp, _vp]),
    "abs_ctx_create_mt": (_int, [_pvp, _int, _vp, _pvp, _pvp, _vp, _vp]),
    "abs_ctx_destroy": (_int, [_vp]),
    "abs_ctx_set_accumulate_streams": (_int, [_vp, _pvp, _int]),
    "abs_ctx_accumulate": (_int, [_vp, _int, _vp, _int, _i64]),
    "abs_ctx_accumulate_mt": (_int, [_vp, _int, _vp, _i64]),
    "abs_ctx_accumulate_batch": (_int, [_vp, _int, _pvp, _int, _int, _pi64]),
    "abs_ctx_accumulate_batch_mt": (_int, [_vp, _int, _pvp, _int, _pi64]),
    "abs_ctx_sync_update": (_int, [_vp, _vp, _vp, _f, _f, _f]),
    "abs_ctx_sync_update_mt": (_int, [_vp, _vp, _vp, _f, _f, _f]),
    "abs_ctx_sync_update_dc": (_int, [_vp, _vp, _vp, _vp, _f, _f, _f, _f]),
    "abs_ctx_sync_update_dc_mt": (_int, [_vp, _vp, _vp, _vp, _f, _f, _f, _f]),
    "abs_ctx_sync_update_adam": (_int, [_vp, _vp, _vp, _vp, _f, _f, _f, _f, _f, _i64]),
    "abs_ctx_sync_update_adam_mt": (_int, [_vp, _vp, _vp, _vp, _f, _f, _f, _f, _f, _i64]),
    "abs_ctx_sync_update_lars_mt": (_int, [_vp, _vp, _vp, _vp, _f, _f, _f, _f]),
    "abs_swap_buffers": (_int, [_vp]),
    "abs_ctx_counts": (_int, [_vp, _int, _pi64]),
}


class AbsError(RuntimeError):
    def __init__(self, fn, rc):
        self.rc = rc
        detail = ""
        if rc == ABS_EHIP:
            detail = f" (hipError_t {lib().abs_last_hip_error()})"
        super().__init__(f"{fn}: {lib().abs_error_string(rc).decode()}{detail}")


_lib = None


def lib():
    """The loaded C library.  Raises if it has not been built: there is no
    other implementation behind this package."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2308_15164_amd.build` "
                "(hipcc, gfx950). This package has no CPU or PyTorch fallback.")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(fn, rc, allow_empty=False):
    if rc == ABS_OK:
        return True
    if rc == ABS_EMPTY and allow_empty:
        return False
    raise AbsError(fn, rc)


def _dev_ptr(t):
    """Device address of a torch tensor (or a raw integer address)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise TypeError("expected a tensor in GPU memory")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    return t.data_ptr()


def _stream_handle(stream):
    """hipStream_t of a torch stream; None means torch's current stream."""
    if isinstance(stream, int):
        return stream
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _dtype_of(t, dtype=None):
    if dtype is not None:
        return dtype
    import torch
    if t.dtype == torch.float32:
        return ABS_F32
    if t.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        return ABS_BF16
    raise TypeError(f"gradient dtype {t.dtype} is neither fp32 nor bf16")


def _ptr_array(ptrs):
    return (ctypes.c_void_p * len(ptrs))(*ptrs)


def _i64_array(vals):
    return (ctypes.c_int64 * len(vals))(*[int(v) for v in vals])


def abs_version():
    return lib().abs_version()


def abs_row_elems():
    return lib().abs_row_elems()


def abs_set_launch_tuning(blocks_per_cu=0, max_rows_per_tile=4):
    """See abs_set_launch_tuning in abs_sgd.h; the defaults are the library's own."""
    return _check("abs_set_launch_tuning",
                  lib().abs_set_launch_tuning(int(blocks_per_cu), int(max_rows_per_tile)))


def abs_set_launch_slice_bytes(nbytes=1 << 30):
    """See abs_set_launch_slice_bytes in abs_sgd.h; the default is the library's own; 0 = never cut."""
    return _check("abs_set_launch_slice_bytes", lib().abs_set_launch_slice_bytes(int(nbytes)))


def abs_launch_count():
    """Kernel launches this thread has enqueued through the library so far."""
    return int(lib().abs_launch_count())


def abs_suggest_accumulate_streams(P, K):
    """1 or 2: accumulate streams that pay for K workers with P-element accumulators."""
    return int(lib().abs_suggest_accumulate_streams(int(P), int(K)))


def abs_set_cache_policy(accumulate_mode=-1, update_mode=-1):
    """-1 auto, 0 cached, 1 streaming; see abs_set_cache_policy in abs_sgd.h."""
    return _check("abs_set_cache_policy", lib().abs_set_cache_policy(int(accumulate_mode), int(update_mode)))


class Count:
    """Host-side int64 sample counter handed to abs_accumulate by address."""

    def __init__(self, value=0):
        self._c = ctypes.c_int64(int(value))

    @property
    def value(self):
        return self._c.value

    @value.setter
    def value(self, v):
        self._c.value = int(v)


def abs_accumulate(acc, grad, n_samples, count, stream=None, P=None, grad_dtype=None):
    """acc (+)= n_samples * grad; count += n_samples.  See abs_accumulate in abs_sgd.h."""
    n = acc.numel() if P is None else int(P)
    rc = lib().abs_accumulate(_dev_ptr(acc), _dev_ptr(grad), _dtype_of(grad, grad_dtype), n,
                              int(n_samples), ctypes.byref(count._c), _stream_handle(stream))
    return _check("abs_accumulate", rc)


def abs_accumulate_batch(acc, grads, n_samples, count, stream=None, P=None, grad_dtype=None):
    """Fold the J gradients `grads` (sample counts `n_samples`) into acc in one pass."""
    n = acc.numel() if P is None else int(P)
    rc = lib().abs_accumulate_batch(_dev_ptr(acc), _ptr_array([_dev_ptr(g) for g in grads]),
                                    _dtype_of(grads[0], grad_dtype), len(grads), n, _i64_array(n_samples),
                                    ctypes.byref(count._c), _stream_handle(stream))
    return _check("abs_accumulate_batch", rc)


class _JobC(ctypes.Structure):
    """struct abs_job / abs_job_mt (the two have the same layout: five pointer-sized or int fields)."""
    _fields_ = [("acc", ctypes.c_void_p), ("grads", ctypes.c_void_p), ("n_samples", ctypes.c_void_p),
                ("J", ctypes.c_int), ("count", ctypes.c_void_p)]


def _job_array(accs, grads, n_samples, counts):
    """accs[w], grads[w][j], n_samples[w][j], counts[w] (Count) -> (array of abs_job, keep-alive list)."""
    keep, arr = [], (_JobC * len(accs))()
    for w, (a, gs, ns, c) in enumerate(zip(accs, grads, n_samples, counts)):
        gp, np_ = _ptr_array(list(gs)) if len(gs) else None, _i64_array(ns) if len(ns) else None
        keep += [gp, np_]
        arr[w] = _JobC(a, ctypes.cast(gp, ctypes.c_void_p) if gp is not None else None,
                       ctypes.cast(np_, ctypes.c_void_p) if np_ is not None else None, len(gs),
                       ctypes.cast(ctypes.pointer(c._c), ctypes.c_void_p))
    return arr, keep


def abs_accumulate_jobs(accs, grads, n_samples, counts, fold=8, stream=None, P=None, grad_dtype=None):
    """One launch sequence for several workers: job w folds grads[w] (sample counts
    n_samples[w]) into accs[w] and advances counts[w].  See abs_accumulate_jobs in abs_sgd.h."""
    n = accs[0].numel() if P is None else int(P)
    first = next((g for gs in grads for g in gs), None)
    dt = grad_dtype if grad_dtype is not None else _dtype_of(first)
    arr, keep = _job_array([_dev_ptr(a) for a in accs], [[_dev_ptr(g) for g in gs] for gs in grads],
                           n_samples, counts)
    rc = lib().abs_accumulate_jobs(arr, len(accs), dt, n, int(fold), _stream_handle(stream))
    return _check("abs_accumulate_jobs", rc)


def abs_accumulate_jobs_mt(layout, accs, grads, n_samples, counts, fold=8, stream=None):
    """abs_accumulate_jobs over a ragged layout: accs[w] and grads[w][j] are TensorSets."""
    arr, keep = _job_array([a.handle.value for a in accs], [[g.handle.value for g in gs] for gs in grads],
                           n_samples, counts)
    rc = lib().abs_accumulate_jobs_mt(layout.handle, arr, len(accs), int(fold), _stream_handle(stream))
    return _check("abs_accumulate_jobs_mt", rc)


def abs_sync_update(params, momentum, acc, counts, lr, mu, wd, stream=None, P=None):
    """Fused weighted combine of acc[K] + delayed momentum-SGD update.
    Returns False when the total count is zero (nothing applied)."""
    n = params.numel() if P is None else int(P)
    ptrs = _ptr_array([_dev_ptr(a) for a in acc])
    rc = lib().abs_sync_update(_dev_ptr(params), _dev_ptr(momentum), ptrs, _i64_array(counts),
                               len(acc), n, float(lr), float(mu), float(wd), _stream_handle(stream))
    return _check("abs_sync_update", rc, allow_empty=True)


def abs_sync_update_dc(params, params_prev, momentum, acc, counts, lr, mu, wd, lam, stream=None, P=None):
    """abs_sync_update with delayed gradient compensation; params_prev holds x_{t-1}."""
    n = params.numel() if P is None else int(P)
    ptrs = _ptr_array([_dev_ptr(a) for a in acc])
    rc = lib().abs_sync_update_dc(_dev_ptr(params), _dev_ptr(params_prev), _dev_ptr(momentum), ptrs,
                                  _i64_array(counts), len(acc), n, float(lr), float(mu), float(wd),
                                  float(lam), _stream_handle(stream))
    return _check("abs_sync_update_dc", rc, allow_empty=True)


def abs_sync_update_adam(params, exp_avg, exp_avg_sq, acc, counts, lr, beta1, beta2, eps, wd, step,
                         stream=None, P=None):
    """Adam on the delayed weighted average; step counts the applied updates from 1."""
    n = params.numel() if P is None else int(P)
    ptrs = _ptr_array([_dev_ptr(a) for a in acc])
    rc = lib().abs_sync_update_adam(_dev_ptr(params), _dev_ptr(exp_avg), _dev_ptr(exp_avg_sq), ptrs,
                                    _i64_array(counts), len(acc), n, float(lr), float(beta1), float(beta2),
                                    float(eps), float(wd), int(step), _stream_handle(stream))
    return _check("abs_sync_update_adam", rc, allow_empty=True)


class Layout:
    """abs_layout: tensor sizes of a ragged parameter vector and its chunk table."""

    def __init__(self, sizes):
        self.sizes = [int(s) for s in sizes]
        h = ctypes.c_void_p()
        _check("abs_layout_create",
               lib().abs_layout_create(ctypes.byref(h), len(self.sizes), _i64_array(self.sizes)))
        self.handle = h

    def num_tensors(self):
        return lib().abs_layout_num_tensors(self.handle)

    def total(self):
        return lib().abs_layout_total(self.handle)

    def num_chunks(self):
        return lib().abs_layout_num_chunks(self.handle)

    def tile(self):
        return lib().abs_layout_tile(self.handle)

    def upload(self):
        return _check("abs_layout_upload", lib().abs_layout_upload(self.handle))

    def chunk(self, c):
        t, off, ln = ctypes.c_int(), ctypes.c_int64(), ctypes.c_int64()
        _check("abs_layout_chunk", lib().abs_layout_chunk(self.handle, c, ctypes.byref(t),
                                                         ctypes.byref(off), ctypes.byref(ln)))
        return t.value, off.value, ln.value

    def close(self):
        if self.handle is not None:
            lib().abs_layout_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class TensorSet:
    """abs_tensorset: the T base pointers of one logical vector over a Layout."""

    def __init__(self, layout, tensors, dtype=None):
        self.layout = layout
        self.tensors = list(tensors)         # keeps the memory alive
        if len(self.tensors) != len(layout.sizes):
            raise ValueError("one tensor per layout entry expected")
        for t, s in zip(self.tensors, layout.sizes):
            if not isinstance(t, int) and t is not None and t.numel() != s:
                raise ValueError("tensor size does not match the layout")
        first = next((t for t in self.tensors if t is not None and not isinstance(t, int)), None)
        self.dtype = _dtype_of(first, dtype) if (first is not None or dtype is not None) else ABS_F32
        h = ctypes.c_void_p()
        ptrs = _ptr_array([_dev_ptr(t) for t in self.tensors])
        _check("abs_tensorset_create",
               lib().abs_tensorset_create(ctypes.byref(h), layout.handle, ptrs, self.dtype))
        self.handle = h

    def close(self):
        if self.handle is not None:
            lib().abs_tensorset_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def abs_accumulate_mt(layout, acc, grad, n_samples, count, stream=None):
    rc = lib().abs_accumulate_mt(layout.handle, acc.handle, grad.handle, int(n_samples),
                                 ctypes.byref(count._c), _stream_handle(stream))
    return _check("abs_accumulate_mt", rc)


def abs_accumulate_batch_mt(layout, acc, grads, n_samples, count, stream=None):
    rc = lib().abs_accumulate_batch_mt(layout.handle, acc.handle, _ptr_array([g.handle.value for g in grads]),
                                       len(grads), _i64_array(n_samples), ctypes.byref(count._c),
                                       _stream_handle(stream))
    return _check("abs_accumulate_batch_mt", rc)


def abs_sync_update_mt(layout, params, momentum, acc, counts, lr, mu, wd, stream=None):
    sets = _ptr_array([a.handle.value for a in acc])
    rc = lib().abs_sync_update_mt(layout.handle, params.handle, momentum.handle, sets,
                                  _i64_array(counts), len(acc), float(lr), float(mu), float(wd),
                                  _stream_handle(stream))
    return _check("abs_sync_update_mt", rc, allow_empty=True)


def abs_sync_update_dcm(params, momentum, acc, counts, lr, mu, wd, lam, lr_prev, stream=None, P=None):
    """Compensated abs_sync_update with x_t - x_{t-1} = -lr_prev * momentum (no x_{t-1} buffer)."""
    n = params.numel() if P is None else int(P)
    ptrs = _ptr_array([_dev_ptr(a) for a in acc])
    rc = lib().abs_sync_update_dcm(_dev_ptr(params), _dev_ptr(momentum), ptrs, _i64_array(counts),
                                   len(acc), n, float(lr), float(mu), float(wd), float(lam),
                                   float(lr_prev), _stream_handle(stream))
    return _check("abs_sync_update_dcm", rc, allow_empty=True)


def abs_sync_update_dcm_mt(layout, params, momentum, acc, counts, lr, mu, wd, lam, lr_prev, stream=None):
    sets = _ptr_array([a.handle.value for a in acc])
    rc = lib().abs_sync_update_dcm_mt(layout.handle, params.handle, momentum.handle, sets,
                                      _i64_array(counts), len(acc), float(lr), float(mu), float(wd),
                                      float(lam), float(lr_prev), _stream_handle(stream))
    return _check("abs_sync_update_dcm_mt", rc, allow_empty=True)


def abs_sync_update_dc_mt(layout, params, params_prev, momentum, acc, counts, lr, mu, wd, lam,
                          stream=None):
    sets = _ptr_array([a.handle.value for a in acc])
    rc = lib().abs_sync_update_dc_mt(layout.handle, params.handle, params_prev.handle, momentum.handle,
                                     sets, _i64_array(counts), len(acc), float(lr), float(mu),
                                     float(wd), float(lam), _stream_handle(stream))
    return _check("abs_sync_update_dc_mt", rc, allow_empty=True)


def abs_sync_update_adam_mt(layout, params, exp_avg, exp_avg_sq, acc, counts, lr, beta1, beta2, eps, wd,
                            step, stream=None):
    sets = _ptr_array([a.handle.value for a in acc])
    rc = lib().abs_sync_update_adam_mt(layout.handle, params.handle, exp_avg.handle, exp_avg_sq.handle, sets,
                                       _i64_array(counts), len(acc), float(lr), float(beta1), float(beta2),
                                       float(eps), float(wd), int(step), _stream_handle(stream))
    return _check("abs_sync_update_adam_mt", rc, allow_empty=True)


def abs_sync_update_lars_mt(layout, params, momentum, gbar, acc, counts, lr, mu, wd, eta, stream=None):
    """LARS per tensor of the layout on the delayed weighted average; gbar is workspace."""
    sets = _ptr_array([a.handle.value for a in acc])
    rc = lib().abs_sync_update_lars_mt(layout.handle, params.handle, momentum.handle, gbar.handle, sets,
                                       _i64_array(counts), len(acc), float(lr), float(mu), float(wd),
                                       float(eta), _stream_handle(stream))
    return _check("abs_sync_update_lars_mt", rc, allow_empty=True)


def abs_sync_update_lars_mt_noalloc(layout, params, momentum, gbar, acc, counts, lr, mu, wd, eta, stream=None):
    """abs_sync_update_lars_mt with its scratch in the library's fixed device array (no allocation)."""
    sets = _ptr_array([a.handle.value for a in acc])
    rc = lib().abs_sync_update_lars_mt_noalloc(layout.handle, params.handle, momentum.handle, gbar.handle, sets,
                                               _i64_array(counts), len(acc), float(lr), float(mu), float(wd),
                                               float(eta), _stream_handle(stream))
    return _check("abs_sync_update_lars_mt_noalloc", rc, allow_empty=True)


class Context:
    """abs_ctx: the double buffer.  acc_A / acc_B are K tensors each (flat form)
    or K TensorSets each over `layout` (ragged form)."""

    def __init__(self, acc_A, acc_B, stream_acc, stream_upd, layout=None, P=None):
        self.layout = layout
        self.K = len(acc_A)
        self._keep = (list(acc_A), list(acc_B), stream_acc, stream_upd)
        h = ctypes.c_void_p()
        sa, su = _stream_handle(stream_acc), _stream_handle(stream_upd)
        if layout is None:
            n = acc_A[0].numel() if P is None else int(P)
            rc = lib().abs_ctx_create(ctypes.byref(h), self.K, n,
                                      _ptr_array([_dev_ptr(a) for a in acc_A]),
                                      _ptr_array([_dev_ptr(a) for a in acc_B]), sa, su)
            _check("abs_ctx_create", rc)
        else:
            rc = lib().abs_ctx_create_mt(ctypes.byref(h), self.K, layout.handle,
                                         _ptr_array([a.handle.value for a in acc_A]),
                                         _ptr_array([a.handle.value for a in acc_B]), sa, su)
            _check("abs_ctx_create_mt", rc)
        self.handle = h

    def abs_set_accumulate_streams(self, streams):
        self._keep = self._keep + (list(streams),)
        arr = _ptr_array([_stream_handle(s) for s in streams])
        return _check("abs_ctx_set_accumulate_streams",
                      lib().abs_ctx_set_accumulate_streams(self.handle, arr, len(streams)))

    def abs_set_launch_tuning(self, blocks_per_cu=0, max_rows_per_tile=4):
        return _check("abs_ctx_set_launch_tuning",
                      lib().abs_ctx_set_launch_tuning(self.handle, int(blocks_per_cu), int(max_rows_per_tile)))

    def abs_set_cache_policy(self, accumulate_mode=-1, update_mode=-1):
        return _check("abs_ctx_set_cache_policy",
                      lib().abs_ctx_set_cache_policy(self.handle, int(accumulate_mode), int(update_mode)))

    def abs_accumulate_step(self, grads, m, n_samples, fold=8, grad_dtype=None):
        """Step 2 of all K workers in one call: grads / n_samples list worker 0's m[0]
        gradients, then worker 1's m[1], ... (device pointers, or TensorSets for a ragged context)."""
        mc = (ctypes.c_int * len(m))(*[int(v) for v in m])
        if self.layout is None:
            first = grads[0] if len(grads) else None
            dt = grad_dtype if grad_dtype is not None else _dtype_of(first)
            rc = lib().abs_ctx_accumulate_step(self.handle, _ptr_array([_dev_ptr(g) for g in grads]), mc,
                                               _i64_array(n_samples), dt, int(fold))
            return _check("abs_ctx_accumulate_step", rc)
        rc = lib().abs_ctx_accumulate_step_mt(self.handle, _ptr_array([g.handle.value for g in grads]), mc,
                                              _i64_array(n_samples), int(fold))
        return _check("abs_ctx_accumulate_step_mt", rc)

    def abs_accumulate(self, k, grad, n_samples, grad_dtype=None):
        if self.layout is None:
            rc = lib().abs_ctx_accumulate(self.handle, int(k), _dev_ptr(grad),
                                          _dtype_of(grad, grad_dtype), int(n_samples))
            return _check("abs_ctx_accumulate", rc)
        rc = lib().abs_ctx_accumulate_mt(self.handle, int(k), grad.handle, int(n_samples))
        return _check("abs_ctx_accumulate_mt", rc)

    def abs_accumulate_batch(self, k, grads, n_samples, grad_dtype=None):
        if self.layout is None:
            rc = lib().abs_ctx_accumulate_batch(self.handle, int(k), _ptr_array([_dev_ptr(g) for g in grads]),
                                                _dtype_of(grads[0], grad_dtype), len(grads),
                                                _i64_array(n_samples))
            return _check("abs_ctx_accumulate_batch", rc)
        rc = lib().abs_ctx_accumulate_batch_mt(self.handle, int(k), _ptr_array([g.handle.value for g in grads]),
                                               len(grads), _i64_array(n_samples))
        return _check("abs_ctx_accumulate_batch_mt", rc)

    def abs_sync_update(self, params, momentum, lr, mu, wd):
        if self.layout is None:
            rc = lib().abs_ctx_sync_update(self.handle, _dev_ptr(params), _dev_ptr(momentum),
                                           float(lr), float(mu), float(wd))
            return _check("abs_ctx_sync_update", rc, allow_empty=True)
        rc = lib().abs_ctx_sync_update_mt(self.handle, params.handle, momentum.handle,
                                          float(lr), float(mu), float(wd))
        return _check("abs_ctx_sync_update_mt", rc, allow_empty=True)

    def abs_sync_update_dc(self, params, params_prev, momentum, lr, mu, wd, lam):
        if self.layout is None:
            rc = lib().abs_ctx_sync_update_dc(self.handle, _dev_ptr(params), _dev_ptr(params_prev),
                                              _dev_ptr(momentum), float(lr), float(mu), float(wd),
                                              float(lam))
            return _check("abs_ctx_sync_update_dc", rc, allow_empty=True)
        rc = lib().abs_ctx_sync_update_dc_mt(self.handle, params.handle, params_prev.handle,
                                             momentum.handle, float(lr), float(mu), float(wd), float(lam))
        return _check("abs_ctx_sync_update_dc_mt", rc, allow_empty=True)

    def abs_sync_update_dcm(self, params, momentum, lr, mu, wd, lam):
        if self.layout is None:
            rc = lib().abs_ctx_sync_update_dcm(self.handle, _dev_ptr(params), _dev_ptr(momentum), float(lr),
                                               float(mu), float(wd), float(lam))
            return _check("abs_ctx_sync_update_dcm", rc, allow_empty=True)
        rc = lib().abs_ctx_sync_update_dcm_mt(self.handle, params.handle, momentum.handle, float(lr),
                                              float(mu), float(wd), float(lam))
        return _check("abs_ctx_sync_update_dcm_mt", rc, allow_empty=True)

    def abs_sync_update_adam(self, params, exp_avg, exp_avg_sq, lr, beta1, beta2, eps, wd, step):
        if self.layout is None:
            rc = lib().abs_ctx_sync_update_adam(self.handle, _dev_ptr(params), _dev_ptr(exp_avg),
                                                _dev_ptr(exp_avg_sq), float(lr), float(beta1), float(beta2),
                                                float(eps), float(wd), int(step))
            return _check("abs_ctx_sync_update_adam", rc, allow_empty=True)
        rc = lib().abs_ctx_sync_update_adam_mt(self.handle, params.handle, exp_avg.handle, exp_avg_sq.handle,
                                               float(lr), float(beta1), float(beta2), float(eps), float(wd),
                                               int(step))
        return _check("abs_ctx_sync_update_adam_mt", rc, allow_empty=True)

    def abs_sync_update_lars(self, params, momentum, gbar, lr, mu, wd, eta):
        rc = lib().abs_ctx_sync_update_lars_mt(self.handle, params.handle, momentum.handle, gbar.handle,
                                               float(lr), float(mu), float(wd), float(eta))
        return _check("abs_ctx_sync_update_lars_mt", rc, allow_empty=True)

    def abs_swap_buffers(self):
        return _check("abs_swap_buffers", lib().abs_swap_buffers(self.handle))

    def counts(self, which=0):
        out = (ctypes.c_int64 * self.K)()
        _check("abs_ctx_counts", lib().abs_ctx_counts(self.handle, int(which), out))
        return [int(v) for v in out]

    def close(self):
        if self.handle is not None:
            lib().abs_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def abs_swap_buffers(ctx):
    """End of an iteration: cross-stream joins, generations trade places."""
    return ctx.abs_swap_buffers()


__all__ = ["abs_swap_buffers", "abs_set_cache_policy", "abs_suggest_accumulate_streams", "lib", "AbsError", "Count", "Layout", "TensorSet", "Context", "abs_accumulate",
           "abs_accumulate_batch", "abs_accumulate_batch_mt", "abs_accumulate_jobs", "abs_accumulate_jobs_mt", "abs_sync_update", "abs_sync_update_dc", "abs_sync_update_dcm", "abs_sync_update_dcm_mt", "abs_sync_update_adam", "abs_sync_update_adam_mt", "abs_sync_update_lars_mt", "abs_sync_update_lars_mt_noalloc", "abs_accumulate_mt", "abs_sync_update_mt",
           "abs_sync_update_dc_mt", "abs_version",
           "abs_row_elems", "abs_set_launch_tuning", "ABS_OK", "ABS_EMPTY", "ABS_EINVAL", "ABS_EHIP", "ABS_F32",
           "ABS_BF16", "ABS_MAX_K", "SYMBOLS", "LIB_PATH"]
