"""ctypes binding of include/plora.h: same names, argument marshalling only.

Functions return the library's status code (and outputs where the C call has out-parameters).
Device buffers are passed as integers (tensor.data_ptr()), streams as integers
(torch.cuda.current_stream().cuda_stream).  PagedLoraPool is a convenience wrapper that raises
PloraError on a negative status and keeps the objects it must keep alive.
"""
import ctypes as C
import os

import numpy as np

__all__ = ["PLORA_OK", "PLORA_ERR_INVAL", "PLORA_ERR_NOMEM", "PLORA_ERR_EXISTS", "PLORA_ERR_NOTFOUND",
           "PLORA_ERR_BUSY", "PLORA_ERR_HIP", "PLORA_ERR_LIMIT", "PLORA_F16", "PLORA_BF16", "PLORA_F32", "PLORA_POOL_PLACEMENT_ONLY",
           "plora_pool_create", "plora_pool_destroy", "plora_adapter_bytes", "plora_load_adapter",
           "plora_adapter_ready", "plora_wait_adapter", "plora_sync_adapter", "plora_evict", "plora_adapter_pages", "plora_compact", "plora_batch_begin", "plora_batch_info",
           "plora_shrink", "plora_expand", "plora_delta", "plora_delta_static", "plora_batch_end", "plora_pool_stats", "plora_pool_set_option",
           "plora_profile", "plora_profile_read", "plora_probe_stream", "plora_probe_h2d", "plora_last_hip", "plora_version", "PloraError", "PagedLoraPool", "lib", "LIB_PATH",
           "plora_predictor_create", "plora_predictor_destroy", "plora_predictor_observe", "plora_predictor_observed",
           "plora_predictor_predict", "plora_predictor_train", "plora_predictor_train_batch",
           "plora_predictor_param_count", "plora_predictor_get_params", "plora_predictor_set_params",
           "plora_predictor_loss_grad", "plora_predictor_set_threads", "LstmPredictor",
           "plora_manager_create", "plora_manager_destroy", "plora_manager_set_adapter", "plora_manager_set_prediction",
           "plora_manager_request", "plora_manager_prefetch", "plora_manager_scores", "plora_manager_residents",
           "plora_manager_state", "plora_manager_get_stats", "plora_manager_log", "ResidencyManager",
           "plora_suggest_page_bytes"]

PLORA_OK, PLORA_ERR_INVAL, PLORA_ERR_NOMEM, PLORA_ERR_EXISTS = 0, -1, -2, -3
PLORA_ERR_NOTFOUND, PLORA_ERR_BUSY, PLORA_ERR_HIP, PLORA_ERR_LIMIT = -4, -5, -6, -7
PLORA_F16, PLORA_BF16, PLORA_F32 = 0, 1, 2
PLORA_POOL_PLACEMENT_ONLY = 1
_STATUS = {0: "OK", -1: "INVAL", -2: "NOMEM", -3: "EXISTS", -4: "NOTFOUND", -5: "BUSY", -6: "HIP", -7: "LIMIT"}

LIB_PATH = os.environ.get("PLORA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libplora.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libplora.so is not built: run `python -m paper_2512_20210_amd.build` "
                      "(or __graft_entry__.build()); there is no fallback implementation")
lib = C.CDLL(LIB_PATH)


class _Layout(C.Structure):
    _fields_ = [("n_slots", C.c_int32), ("d_in", C.POINTER(C.c_int32)), ("d_out", C.POINTER(C.c_int32)),
                ("dtype", C.c_int32), ("max_adapters", C.c_int32), ("max_rank", C.c_int32)]


class _Stats(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in ("page_bytes", "n_pages", "used_pages", "free_pages", "resident_adapters",
                                          "resident_bytes", "internal_frag_bytes", "loads", "evictions",
                                          "nomem_failures", "h2d_bytes", "h2d_copies")] + [("h2d_ms", C.c_double), ("staged_loads", C.c_uint64), ("fused_launches", C.c_uint64),
                                                                                        ("fused_timeouts", C.c_uint64), ("compacted_adapters", C.c_uint64),
                                                                                        ("compacted_pages", C.c_uint64), ("compact_ms", C.c_double)]


_vp, _i32, _u32, _u64, _f32 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float
lib.plora_pool_create.argtypes = [C.c_size_t, _u32, C.POINTER(_Layout), _vp, _u32, C.POINTER(_vp)]
lib.plora_pool_destroy.argtypes = [_vp]
lib.plora_adapter_bytes.argtypes = [_vp, _i32]
lib.plora_adapter_bytes.restype = _u64
lib.plora_load_adapter.argtypes = [_vp, _i32, _i32, _f32, _vp, _vp, C.POINTER(C.POINTER(_i32)), C.POINTER(_u32)]
lib.plora_adapter_ready.argtypes = [_vp, _i32]
lib.plora_wait_adapter.argtypes = [_vp, _i32, _vp]
lib.plora_evict.argtypes = [_vp, _i32]
lib.plora_compact.argtypes = [_vp, _vp, _u32, C.POINTER(_u32), C.POINTER(_u32)]
lib.plora_adapter_pages.argtypes = [_vp, _i32, C.POINTER(C.POINTER(_i32)), C.POINTER(_u32)]
lib.plora_sync_adapter.argtypes = [_vp, _i32]
lib.plora_batch_begin.argtypes = [_vp, _vp, _i32, _vp, C.POINTER(_vp)]
lib.plora_batch_info.argtypes = [_vp, C.POINTER(_i32), C.POINTER(_i32), C.POINTER(C.POINTER(_i32)),
                                 C.POINTER(C.POINTER(_i32)), C.POINTER(C.POINTER(_i32))]
lib.plora_shrink.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp, _vp]
lib.plora_expand.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp, _vp]
lib.plora_delta.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp]
lib.plora_delta_static.argtypes = [_vp, _vp, _i32, _i32, _vp, _vp, _vp]
lib.plora_batch_end.argtypes = [_vp, _vp]
lib.plora_pool_stats.argtypes = [_vp, C.POINTER(_Stats)]
lib.plora_pool_set_option.argtypes = [_vp, C.c_char_p, C.c_int64]
lib.plora_profile.argtypes = [_vp, C.c_int]
lib.plora_profile_read.argtypes = [_vp, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
lib.plora_probe_stream.argtypes = [_u64, _u64, _u32, _u32, _i32, _vp, C.POINTER(C.c_double)]
lib.plora_probe_h2d.argtypes = [_u64, _i32, _vp, C.POINTER(C.c_double)]
lib.plora_last_hip.argtypes = []
lib.plora_version.argtypes = []


class _ManagerConfig(C.Structure):
    _fields_ = [("alpha", C.c_double), ("beta", C.c_double), ("gamma", C.c_double), ("theta", C.c_double), ("window", C.c_int32)]


class _ManagerStats(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in ("hits", "misses", "loads", "evictions", "failed_loads", "skipped_busy", "waited_for_busy",
                                          "prefetch_loads", "useful_prefetches", "wasted_prefetches", "prefetch_no_room",
                                          "util_samples")] + [(k, C.c_double) for k in ("page_util_sum", "page_util_min",
                                                                                         "byte_util_sum", "byte_util_min")]


lib.plora_manager_create.argtypes = [_vp, _i32, C.POINTER(_ManagerConfig), C.POINTER(_vp)]
lib.plora_manager_destroy.argtypes = [_vp]
lib.plora_manager_set_adapter.argtypes = [_vp, _i32, _i32, _f32, _vp]
lib.plora_manager_set_prediction.argtypes = [_vp, _vp]
lib.plora_manager_request.argtypes = [_vp, _i32, _vp, C.POINTER(_i32)]
lib.plora_manager_prefetch.argtypes = [_vp, _vp, _vp, C.POINTER(_i32)]
lib.plora_manager_scores.argtypes = [_vp, _vp, _vp, _i32, C.POINTER(_i32)]
lib.plora_manager_residents.argtypes = [_vp, _vp, _i32, C.POINTER(_i32)]
lib.plora_manager_state.argtypes = [_vp, _i32]
lib.plora_manager_get_stats.argtypes = [_vp, C.POINTER(_ManagerStats)]
lib.plora_manager_log.argtypes = [_vp, _vp, C.c_int64, C.POINTER(C.c_int64), _i32]
lib.plora_suggest_page_bytes.argtypes = [C.POINTER(_Layout), _vp, _vp, _i32, C.c_double, C.c_size_t, C.c_size_t,
                                         C.POINTER(C.c_size_t), C.POINTER(C.c_double)]


class _PredictorConfig(C.Structure):
    _fields_ = [("n_adapters", C.c_int32), ("window", C.c_int32), ("hidden", C.c_int32), ("layers", C.c_int32),
                ("replay", C.c_int32), ("batch", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("seed", C.c_uint64)]


_fp = C.POINTER(C.c_float)
lib.plora_predictor_create.argtypes = [C.POINTER(_PredictorConfig), C.POINTER(_vp)]
lib.plora_predictor_destroy.argtypes = [_vp]
lib.plora_predictor_observe.argtypes = [_vp, _vp, _i32]
lib.plora_predictor_observed.argtypes = [_vp]
lib.plora_predictor_observed.restype = C.c_int64
lib.plora_predictor_predict.argtypes = [_vp, _vp]
lib.plora_predictor_train.argtypes = [_vp, _i32, _fp]
lib.plora_predictor_train_batch.argtypes = [_vp, _vp, _i32, _fp]
lib.plora_predictor_param_count.argtypes = [_vp]
lib.plora_predictor_param_count.restype = C.c_int64
lib.plora_predictor_get_params.argtypes = [_vp, _vp]
lib.plora_predictor_set_params.argtypes = [_vp, _vp]
lib.plora_predictor_loss_grad.argtypes = [_vp, _vp, _vp, _fp, _vp]
lib.plora_predictor_set_threads.argtypes = [_vp, _i32]


def _ptr_array(ptrs):
    return (C.c_void_p * len(ptrs))(*[int(p) for p in ptrs])


def plora_pool_create(page_bytes, n_pages, d_in, d_out, dtype, max_adapters, max_rank, slab_ptr=None, flags=0):
    """-> (status, pool handle)."""
    di = np.ascontiguousarray(d_in, dtype=np.int32)
    do = np.ascontiguousarray(d_out, dtype=np.int32)
    lay = _Layout(len(di), di.ctypes.data_as(C.POINTER(C.c_int32)), do.ctypes.data_as(C.POINTER(C.c_int32)),
                  dtype, max_adapters, max_rank)
    h = C.c_void_p()
    rc = lib.plora_pool_create(page_bytes, n_pages, C.byref(lay), slab_ptr, flags, C.byref(h))
    return rc, h


def plora_pool_destroy(pool):
    return lib.plora_pool_destroy(pool)


def plora_adapter_bytes(pool, rank):
    return lib.plora_adapter_bytes(pool, rank)


def plora_load_adapter(pool, aid, rank, scale, pinned_host_ptr, copy_stream=None):
    """-> (status, page table as an int32 numpy copy or None)."""
    pt = C.POINTER(C.c_int32)()
    n = C.c_uint32(0)
    rc = lib.plora_load_adapter(pool, aid, rank, scale, pinned_host_ptr, copy_stream, C.byref(pt), C.byref(n))
    if rc:
        return rc, None
    return rc, np.ctypeslib.as_array(pt, shape=(n.value,)).copy()


def plora_adapter_ready(pool, aid):
    return lib.plora_adapter_ready(pool, aid)


def plora_wait_adapter(pool, aid, stream=None):
    return lib.plora_wait_adapter(pool, aid, stream)


def plora_sync_adapter(pool, aid):
    return lib.plora_sync_adapter(pool, aid)


def plora_evict(pool, aid):
    return lib.plora_evict(pool, aid)


def plora_adapter_pages(pool, aid):
    """-> (status, copy of the adapter's page table as an int32 array)."""
    pt, n = C.POINTER(_i32)(), _u32(0)
    rc = lib.plora_adapter_pages(pool, aid, C.byref(pt), C.byref(n))
    if rc != PLORA_OK:
        return rc, None
    return rc, np.ctypeslib.as_array(pt, shape=(n.value,)).copy() if n.value else np.empty(0, np.int32)


def plora_compact(pool, stream=None, max_pages=0):
    """-> (status, pages moved, adapters moved)."""
    pages, adapters = _u32(0), _u32(0)
    rc = lib.plora_compact(pool, stream, max_pages, C.byref(pages), C.byref(adapters))
    return rc, pages.value, adapters.value


def plora_batch_begin(pool, tok2adapter, stream=None):
    """tok2adapter: host int32 array. -> (status, batch handle)."""
    t2a = np.ascontiguousarray(tok2adapter, dtype=np.int32)
    b = C.c_void_p()
    rc = lib.plora_batch_begin(pool, t2a.ctypes.data_as(C.c_void_p), len(t2a), stream, C.byref(b))
    return rc, b


def plora_batch_info(batch):
    """-> (status, perm, seg_adapter, seg_start) as numpy copies."""
    ns, npm = C.c_int32(0), C.c_int32(0)
    perm, sa, ss = C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)()
    rc = lib.plora_batch_info(batch, C.byref(ns), C.byref(npm), C.byref(perm), C.byref(sa), C.byref(ss))
    if rc:
        return rc, None, None, None

    def arr(p, n):
        return np.ctypeslib.as_array(p, shape=(n,)).copy() if n else np.zeros(0, np.int32)
    return rc, arr(perm, npm.value), arr(sa, ns.value), arr(ss, ns.value + 1)


def plora_shrink(pool, batch, slot0, n_slots, x_ptrs, v_ptrs, stream=None):
    return lib.plora_shrink(pool, batch, slot0, n_slots, _ptr_array(x_ptrs), _ptr_array(v_ptrs), stream)


def plora_expand(pool, batch, slot0, n_slots, v_ptrs, y_ptrs, stream=None):
    return lib.plora_expand(pool, batch, slot0, n_slots, _ptr_array(v_ptrs), _ptr_array(y_ptrs), stream)


def plora_delta(pool, batch, slot0, n_slots, x_ptrs, v_ptrs, y_ptrs, stream=None):
    return lib.plora_delta(pool, batch, slot0, n_slots, _ptr_array(x_ptrs), _ptr_array(v_ptrs), _ptr_array(y_ptrs), stream)


def plora_delta_static(pool, batch, slot0, n_slots, x_ptrs, y_ptrs, stream=None):
    return lib.plora_delta_static(pool, batch, slot0, n_slots, _ptr_array(x_ptrs), _ptr_array(y_ptrs), stream)


def plora_batch_end(pool, batch):
    return lib.plora_batch_end(pool, batch)


def plora_pool_stats(pool):
    """-> (status, dict)."""
    st = _Stats()
    rc = lib.plora_pool_stats(pool, C.byref(st))
    return rc, {k: getattr(st, k) for k, _ in _Stats._fields_}


def plora_pool_set_option(pool, key, value):
    return lib.plora_pool_set_option(pool, key.encode(), int(value))


def plora_profile(pool, enable):
    return lib.plora_profile(pool, int(enable))


def plora_profile_read(pool):
    """-> (status, ms[3], launches[3]) for the shrink kernels, the expand kernels and the one-launch form."""
    ms = (C.c_double * 3)()
    n = (C.c_uint64 * 3)()
    rc = lib.plora_profile_read(pool, ms, n)
    return rc, list(ms), list(n)


def plora_probe_stream(w_bytes, y_bytes, w_tile, y_tile, iters, stream=None):
    """-> (status, ms per launch)."""
    ms = C.c_double(0.0)
    rc = lib.plora_probe_stream(w_bytes, y_bytes, w_tile, y_tile, iters, stream, C.byref(ms))
    return rc, ms.value


def plora_probe_h2d(nbytes, iters, stream=None):
    """-> (status, ms per copy)."""
    ms = C.c_double(0.0)
    rc = lib.plora_probe_h2d(nbytes, iters, stream, C.byref(ms))
    return rc, ms.value


def plora_last_hip():
    return lib.plora_last_hip()


def plora_version():
    return lib.plora_version()


class PloraError(RuntimeError):
    def __init__(self, call, code):
        extra = " (hipError %d)" % plora_last_hip() if code == PLORA_ERR_HIP else ""
        super().__init__("%s -> %s%s" % (call, _STATUS.get(code, code), extra))
        self.code = code


def _check(call, rc):
    if rc < 0:
        raise PloraError(call, rc)
    return rc


class PagedLoraPool:
    """Raises on errors, keeps host blobs and pointer arrays alive; no arithmetic of its own."""

    def __init__(self, page_bytes, n_pages, d_in, d_out, dtype, max_adapters, max_rank, slab=None,
                 placement_only=False):
        self.d_in, self.d_out = list(d_in), list(d_out)
        self.dtype, self.max_rank, self.max_adapters = dtype, max_rank, max_adapters
        self.page_bytes, self.n_pages = page_bytes, n_pages
        self._slab = slab  # a torch tensor, kept alive
        rc, self.h = plora_pool_create(page_bytes, n_pages, d_in, d_out, dtype, max_adapters, max_rank,
                                       None if slab is None else slab.data_ptr(),
                                       PLORA_POOL_PLACEMENT_ONLY if placement_only else 0)
        _check("plora_pool_create", rc)
        self._blobs = {}

    def close(self):
        if self.h:
            _check("plora_pool_destroy", plora_pool_destroy(self.h))
            self.h = None

    def adapter_bytes(self, rank):
        return plora_adapter_bytes(self.h, rank)

    def load(self, aid, rank, scale, pinned_blob=None, copy_stream=None):
        """pinned_blob: page-locked torch tensor (or None for a placement-only pool)."""
        ptr = None if pinned_blob is None else pinned_blob.data_ptr()
        rc, pt = plora_load_adapter(self.h, aid, rank, scale, ptr, copy_stream)
        _check("plora_load_adapter", rc)
        self._blobs[aid] = pinned_blob
        return pt

    def ready(self, aid):
        return _check("plora_adapter_ready", plora_adapter_ready(self.h, aid)) == 1

    def wait(self, aid, stream=None):
        _check("plora_wait_adapter", plora_wait_adapter(self.h, aid, stream))

    def evict(self, aid):
        _check("plora_evict", plora_evict(self.h, aid))
        self._blobs.pop(aid, None)

    def page_table(self, aid):
        rc, pt = plora_adapter_pages(self.h, aid)
        _check("plora_adapter_pages", rc)
        return pt

    def compact(self, stream=None, max_pages=0):
        rc, pages, adapters = plora_compact(self.h, stream, max_pages)
        _check("plora_compact", rc)
        return pages, adapters

    def batch_begin(self, tok2adapter, stream=None):
        rc, b = plora_batch_begin(self.h, tok2adapter, stream)
        _check("plora_batch_begin", rc)
        return b

    def batch_info(self, batch):
        rc, perm, sa, ss = plora_batch_info(batch)
        _check("plora_batch_info", rc)
        return perm, sa, ss

    def shrink(self, batch, slot0, x_tensors, v_tensors, stream=None):
        _check("plora_shrink", plora_shrink(self.h, batch, slot0, len(x_tensors), [t.data_ptr() for t in x_tensors],
                                            [t.data_ptr() for t in v_tensors], stream))

    def expand(self, batch, slot0, v_tensors, y_tensors, stream=None):
        _check("plora_expand", plora_expand(self.h, batch, slot0, len(y_tensors), [t.data_ptr() for t in v_tensors],
                                            [t.data_ptr() for t in y_tensors], stream))

    def delta(self, batch, slot0, x_tensors, v_tensors, y_tensors, stream=None):
        _check("plora_delta", plora_delta(self.h, batch, slot0, len(x_tensors), [t.data_ptr() for t in x_tensors],
                                          [t.data_ptr() for t in v_tensors], [t.data_ptr() for t in y_tensors], stream))

    def delta_static(self, batch, slot0, x_tensors, y_tensors, stream=None):
        _check("plora_delta_static", plora_delta_static(self.h, batch, slot0, len(x_tensors), [t.data_ptr() for t in x_tensors],
                                                        [t.data_ptr() for t in y_tensors], stream))

    def batch_end(self, batch):
        _check("plora_batch_end", plora_batch_end(self.h, batch))

    def stats(self):
        rc, st = plora_pool_stats(self.h)
        _check("plora_pool_stats", rc)
        return st

    def profile(self, enable):
        _check("plora_profile", plora_profile(self.h, enable))

    def profile_read(self):
        rc, ms, n = plora_profile_read(self.h)
        _check("plora_profile_read", rc)
        return ms, n

    def set_option(self, key, value):
        _check("plora_pool_set_option", plora_pool_set_option(self.h, key, value))


# ---------------------------------------------------------------------------------------------
# traffic predictor (host only)
# ---------------------------------------------------------------------------------------------
def plora_predictor_create(n_adapters, window=8, hidden=64, layers=2, replay=10000, batch=64, lr=1e-3, beta1=0.9,
                           beta2=0.999, eps=1e-8, seed=0):
    cfg = _PredictorConfig(n_adapters, window, hidden, layers, replay, batch, lr, beta1, beta2, eps, seed)
    out = C.c_void_p()
    rc = lib.plora_predictor_create(C.byref(cfg), C.byref(out))
    return rc, out.value


def plora_predictor_destroy(pred):
    return lib.plora_predictor_destroy(pred)


def plora_predictor_observe(pred, ids):
    a = np.ascontiguousarray(ids, dtype=np.int32)
    return lib.plora_predictor_observe(pred, a.ctypes.data, len(a))


def plora_predictor_observed(pred):
    return lib.plora_predictor_observed(pred)


def plora_predictor_predict(pred, n_adapters):
    out = np.empty(n_adapters, np.float32)
    rc = lib.plora_predictor_predict(pred, out.ctypes.data)
    return rc, out


def plora_predictor_train(pred, steps):
    loss = C.c_float()
    rc = lib.plora_predictor_train(pred, steps, C.byref(loss))
    return rc, loss.value


def plora_predictor_train_batch(pred, target_pos):
    a = np.ascontiguousarray(target_pos, dtype=np.int32)
    loss = C.c_float()
    rc = lib.plora_predictor_train_batch(pred, a.ctypes.data, len(a), C.byref(loss))
    return rc, loss.value


def plora_predictor_set_threads(pred, threads):
    return lib.plora_predictor_set_threads(pred, threads)


def plora_predictor_param_count(pred):
    return lib.plora_predictor_param_count(pred)


def plora_predictor_get_params(pred):
    out = np.empty(lib.plora_predictor_param_count(pred), np.float32)
    rc = lib.plora_predictor_get_params(pred, out.ctypes.data)
    return rc, out


def plora_predictor_set_params(pred, params):
    a = np.ascontiguousarray(params, dtype=np.float32)
    if a.size != lib.plora_predictor_param_count(pred):
        return PLORA_ERR_INVAL
    return lib.plora_predictor_set_params(pred, a.ctypes.data)


def plora_predictor_loss_grad(pred, seq, target, want_grad=True):
    s = np.ascontiguousarray(seq, dtype=np.float32)
    t = np.ascontiguousarray(target, dtype=np.float32)
    loss = C.c_float()
    grad = np.empty(lib.plora_predictor_param_count(pred), np.float32) if want_grad else None
    rc = lib.plora_predictor_loss_grad(pred, s.ctypes.data, t.ctypes.data, C.byref(loss), None if grad is None else grad.ctypes.data)
    return rc, loss.value, grad


class LstmPredictor:
    """The library's predictor behind the interface the prefetch manager expects: predict(ids of the
    coming interval) returns p_hat computed from the intervals seen so far, and only then records the
    coming interval's requests (they become history once the interval is over) and trains."""

    def __init__(self, n_adapters, window=8, hidden=64, layers=2, replay=10000, batch=64, lr=1e-3, seed=0,
                 train_steps=1, threads=1):
        self.n, self.train_steps = int(n_adapters), int(train_steps)
        rc, self.h = plora_predictor_create(n_adapters, window, hidden, layers, replay, batch, lr, seed=seed)
        _check("plora_predictor_create", rc)
        _check("plora_predictor_set_threads", plora_predictor_set_threads(self.h, threads))
        self.last_loss = None

    def predict(self, next_interval_ids):
        rc, p_hat = plora_predictor_predict(self.h, self.n)
        _check("plora_predictor_predict", rc)
        _check("plora_predictor_observe", plora_predictor_observe(self.h, next_interval_ids))
        if self.train_steps:
            rc, self.last_loss = plora_predictor_train(self.h, self.train_steps)
            _check("plora_predictor_train", rc)
        return p_hat

    def close(self):
        if self.h:
            plora_predictor_destroy(self.h)
            self.h = None


# ---------------------------------------------------------------------------------------------
# residency policy (host only)
# ---------------------------------------------------------------------------------------------
def plora_manager_create(pool, n_adapters, alpha=0.4, beta=0.3, gamma=0.3, theta=0.5, window=1000):
    cfg = _ManagerConfig(alpha, beta, gamma, theta, window)
    out = C.c_void_p()
    rc = lib.plora_manager_create(pool, n_adapters, C.byref(cfg), C.byref(out))
    return rc, out.value


def plora_manager_destroy(mgr):
    return lib.plora_manager_destroy(mgr)


def plora_manager_set_adapter(mgr, aid, rank, scale, pinned_host_ptr=None):
    return lib.plora_manager_set_adapter(mgr, aid, rank, scale, pinned_host_ptr)


def plora_manager_set_prediction(mgr, p_hat):
    if p_hat is None:
        return lib.plora_manager_set_prediction(mgr, None)
    a = np.ascontiguousarray(p_hat, dtype=np.float32)
    return lib.plora_manager_set_prediction(mgr, a.ctypes.data)


def plora_manager_request(mgr, aid, copy_stream=None):
    """-> (status, hit)."""
    hit = C.c_int32(0)
    rc = lib.plora_manager_request(mgr, aid, copy_stream, C.byref(hit))
    return rc, hit.value


def plora_manager_prefetch(mgr, p_hat, prefetch_stream=None):
    """-> (status, number of loads started)."""
    a = np.ascontiguousarray(p_hat, dtype=np.float32)
    n = C.c_int32(0)
    rc = lib.plora_manager_prefetch(mgr, a.ctypes.data, prefetch_stream, C.byref(n))
    return rc, n.value


def plora_manager_residents(mgr):
    n = C.c_int32(0)
    rc = lib.plora_manager_residents(mgr, None, 0, C.byref(n))
    ids = np.empty(n.value, np.int32)
    if rc == 0 and n.value:
        rc = lib.plora_manager_residents(mgr, ids.ctypes.data, n.value, C.byref(n))
    return rc, ids


def plora_manager_scores(mgr):
    """-> (status, ids ascending, scores)."""
    n = C.c_int32(0)
    rc = lib.plora_manager_scores(mgr, None, None, 0, C.byref(n))
    ids, sc = np.empty(n.value, np.int32), np.empty(n.value, np.float64)
    if rc == 0 and n.value:
        rc = lib.plora_manager_scores(mgr, ids.ctypes.data, sc.ctypes.data, n.value, C.byref(n))
    return rc, ids, sc


def plora_manager_state(mgr, aid):
    return lib.plora_manager_state(mgr, aid)


def plora_manager_get_stats(mgr):
    st = _ManagerStats()
    rc = lib.plora_manager_get_stats(mgr, C.byref(st))
    return rc, {k: getattr(st, k) for k, _ in _ManagerStats._fields_}


def plora_manager_log(mgr, clear=False):
    """-> (status, int32 array of (kind, id) pairs; kind 0 = load, 1 = evict)."""
    n = C.c_int64(0)
    rc = lib.plora_manager_log(mgr, None, 0, C.byref(n), 0)
    out = np.empty((n.value, 2), np.int32)
    if rc == 0:
        rc = lib.plora_manager_log(mgr, out.ctypes.data if n.value else None, n.value, C.byref(n), int(clear))
    return rc, out


class ResidencyManager:
    """The library's residency policy (load on demand, eviction by score, threshold prefetching) with
    errors raised; no arithmetic of its own."""

    def __init__(self, pool, ranks, scales, blob_of=None, alpha=0.4, beta=0.3, gamma=0.3, theta=0.5, window=1000,
                 copy_stream=None, prefetch_stream=None):
        """pool: PagedLoraPool; ranks / scales: per adapter id; blob_of(id) -> page-locked torch tensor (None for
        a placement-only pool)."""
        self.pool, self.theta = pool, theta
        self.copy_stream, self.prefetch_stream = copy_stream, prefetch_stream
        rc, self.h = plora_manager_create(pool.h, len(ranks), alpha, beta, gamma, theta, window)
        _check("plora_manager_create", rc)
        self._blobs = []
        for i, (r, sc) in enumerate(zip(ranks, scales)):
            blob = blob_of(i) if blob_of is not None else None
            self._blobs.append(blob)
            _check("plora_manager_set_adapter", plora_manager_set_adapter(self.h, i, int(r), float(sc), None if blob is None else blob.data_ptr()))

    def close(self):
        if self.h:
            plora_manager_destroy(self.h)
            self.h = None

    def request(self, aid):
        rc, hit = plora_manager_request(self.h, int(aid), self.copy_stream)
        _check("plora_manager_request", rc)
        return bool(hit)

    def prefetch(self, p_hat):
        rc, n = plora_manager_prefetch(self.h, p_hat, self.prefetch_stream)
        _check("plora_manager_prefetch", rc)
        return n

    def set_prediction(self, p_hat):
        _check("plora_manager_set_prediction", plora_manager_set_prediction(self.h, p_hat))

    def residents(self):
        rc, ids = plora_manager_residents(self.h)
        _check("plora_manager_residents", rc)
        return ids

    def scores(self):
        rc, ids, sc = plora_manager_scores(self.h)
        _check("plora_manager_scores", rc)
        return dict(zip(ids.tolist(), sc.tolist()))

    def state(self, aid):
        return _check("plora_manager_state", plora_manager_state(self.h, int(aid)))

    def stats(self):
        rc, st = plora_manager_get_stats(self.h)
        _check("plora_manager_get_stats", rc)
        return st

    def log(self, clear=False):
        rc, a = plora_manager_log(self.h, clear)
        _check("plora_manager_log", rc)
        return [tuple(x) for x in a.tolist()]


def plora_suggest_page_bytes(d_in, d_out, dtype, ranks, weights, max_internal_frag=0.02, min_page=4096, max_page=2 << 20):
    """-> (status, page_bytes, expected internal fragmentation at that page size)."""
    di = np.ascontiguousarray(d_in, dtype=np.int32)
    do = np.ascontiguousarray(d_out, dtype=np.int32)
    lay = _Layout(len(di), di.ctypes.data_as(C.POINTER(C.c_int32)), do.ctypes.data_as(C.POINTER(C.c_int32)), dtype, 1, 1)
    r = np.ascontiguousarray(ranks, dtype=np.int32)
    w = np.ascontiguousarray(weights, dtype=np.float64)
    if len(r) != len(w):
        return PLORA_ERR_INVAL, 0, 0.0
    page, frag = C.c_size_t(0), C.c_double(0.0)
    rc = lib.plora_suggest_page_bytes(C.byref(lay), r.ctypes.data, w.ctypes.data, len(r), max_internal_frag, min_page, max_page,
                                      C.byref(page), C.byref(frag))
    return rc, page.value, frag.value
