"""ctypes binding of libngc.so: same names as include/ngc.h, argument marshalling only.

Device buffers are torch tensors (torch is used for HBM allocation and streams
only); host arrays are NumPy.  Every function returns what the C call returns
through its output arguments and raises NgcError on a negative status.  If the
shared library has not been built the import of this module fails: there is no
CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
# torch owns the device memory handed to the library and ships its own HIP runtime; it is
# imported first so that libngc.so binds to that same runtime instead of loading a second one.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
# NGC_LIB names another build of the same library (the host-sanitizer build of build.py)
LIB_PATH = os.environ.get("NGC_LIB") or os.path.join(_HERE, "libngc.so")

NGC_OK = 0
NGC_ERR_INVALID = -1
NGC_ERR_UNDECODABLE = -2
NGC_ERR_SINGULAR = -3
NGC_ERR_HIP = -4
NGC_ERR_NOMEM = -5
NGC_ERR_STATE = -6

NGC_LOSS_LSQ, NGC_LOSS_LOGISTIC, NGC_LOSS_MLP2 = 0, 1, 2
NGC_CODE_CYCLIC, NGC_CODE_FRACREP = 0, 1
NGC_KERNEL_NAMES = ("grad", "reduce", "encode", "decode", "update", "mlp", "probe", "tail", "rounds")
NGC_KERNEL_COUNT = len(NGC_KERNEL_NAMES)

EXPORTS = (
    "ngc_create", "ngc_destroy", "ngc_set_code", "ngc_get_code", "ngc_get_shape", "ngc_build_code",
    "ngc_set_mlp2_shape", "ngc_partition_grads", "ngc_partition_grads_static", "ngc_encode", "ngc_select_decode_vec",
    "ngc_select_decode_vec_first", "ngc_set_decode_guard", "ngc_decode", "ngc_encode_decode", "ngc_coded_rounds", "ngc_update",
    "ngc_iteration", "ngc_tail_lds_bytes", "ngc_sync",
    "ngc_worker_task_count", "ngc_worker_schedule", "ngc_worker_grads", "ngc_worker_encode",
    "ngc_select_from_progress", "ngc_build_decoding_table", "ngc_decoding_row_index",
    "ngc_get_decoding_row", "ngc_decode_lookup", "ngc_latency_cdf_gc", "ngc_latency_cdf_ngc", "ngc_latency_simulate",
    "ngc_profile_enable", "ngc_profile_read", "ngc_profile_launches", "ngc_probe_copy", "ngc_probe_read",
    "ngc_strerror", "ngc_last_error",
)

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libngc.so is not built (%s missing): run `python -m paper_2212_08580_amd.build` "
        "or __graft_entry__.build(); there is no CPU fallback" % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _i64, _u64, _dbl = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64,
                             ctypes.c_double)
_lib.ngc_create.argtypes = [ctypes.POINTER(_vp), _i, _i, _i, ctypes.POINTER(_i), _i64, _vp]
_lib.ngc_destroy.argtypes = [_vp]
_lib.ngc_destroy.restype = None
_lib.ngc_set_code.argtypes = [_vp, _i, _vp]
_lib.ngc_get_code.argtypes = [_vp, _i, _vp]
_lib.ngc_build_code.argtypes = [_vp, _i, _u64]
_lib.ngc_get_shape.argtypes = [_vp, ctypes.POINTER(_i), ctypes.POINTER(_i), ctypes.POINTER(_i),
                               ctypes.POINTER(_i64), ctypes.POINTER(_i)]
_lib.ngc_set_mlp2_shape.argtypes = [_vp, _i, _i, _i]
_lib.ngc_set_decode_guard.argtypes = [_vp, _dbl]
_lib.ngc_partition_grads.argtypes = [_vp, _i, _vp, _vp, _vp, _i64, _vp]
_lib.ngc_partition_grads_static.argtypes = _lib.ngc_partition_grads.argtypes
_lib.ngc_encode.argtypes = [_vp, _vp, _i, _vp]
_lib.ngc_select_decode_vec.argtypes = [_vp, _vp, ctypes.POINTER(_i), _vp, ctypes.POINTER(_dbl)]
_lib.ngc_select_decode_vec_first.argtypes = _lib.ngc_select_decode_vec.argtypes
_lib.ngc_decode.argtypes = [_vp, _i, _vp, _vp, _vp]
_lib.ngc_encode_decode.argtypes = [_vp, _vp, _i, _vp, _vp, _vp]
_lib.ngc_coded_rounds.argtypes = [_vp, _vp, _i64, _i, _vp, _vp, _i64, _vp, _vp, _vp]
_lib.ngc_tail_lds_bytes.argtypes = [_vp, _i, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
_lib.ngc_update.argtypes = [_vp, _vp, _vp, _dbl]
_lib.ngc_iteration.argtypes = [_vp, _i, _vp, _vp, _vp, _i64, _vp, _dbl, _vp, _vp, _vp,
                               ctypes.POINTER(_i), _vp]
_lib.ngc_build_decoding_table.argtypes = [_vp, _i, ctypes.POINTER(_i64)]
_lib.ngc_decoding_row_index.argtypes = [_vp, _i, _vp, ctypes.POINTER(_i64)]
_lib.ngc_get_decoding_row.argtypes = [_vp, _i, _i64, _vp]
_lib.ngc_decode_lookup.argtypes = [_vp, _i, _vp, _vp, _vp]
_lib.ngc_latency_cdf_gc.argtypes = [_i, _i, _dbl, _dbl, _dbl, _dbl, _dbl, _vp, _i, _vp]
_lib.ngc_latency_cdf_ngc.argtypes = _lib.ngc_latency_cdf_gc.argtypes
_lib.ngc_latency_simulate.argtypes = [_vp, _i, _i, _dbl, _dbl, _dbl, _dbl, _dbl, _u64, _i64, _vp, _vp]
_lib.ngc_worker_task_count.argtypes = [_vp, ctypes.POINTER(_i)]
_lib.ngc_worker_schedule.argtypes = [_vp, _i, _vp, ctypes.POINTER(_i)]
_lib.ngc_worker_grads.argtypes = [_vp, _i, _vp, _vp, _vp, _i64, _vp, _vp]
_lib.ngc_worker_encode.argtypes = [_vp, _vp, _vp, _vp]
_lib.ngc_select_from_progress.argtypes = [_vp, _vp, _i, ctypes.POINTER(_i), _vp, _vp,
                                          ctypes.POINTER(_dbl)]
_lib.ngc_sync.argtypes = [_vp]
_lib.ngc_profile_enable.argtypes = [_vp, _i]
_lib.ngc_profile_read.argtypes = [_vp, _vp, _vp]
_lib.ngc_profile_launches.argtypes = [_vp, _i, _vp, _i64, ctypes.POINTER(_i64)]
_lib.ngc_probe_copy.argtypes = [_vp, _vp, _vp, _i64]
_lib.ngc_probe_read.argtypes = [_vp, _vp, _i64]
_lib.ngc_strerror.argtypes = [_i]
_lib.ngc_strerror.restype = ctypes.c_char_p
_lib.ngc_last_error.argtypes = [_vp]
_lib.ngc_last_error.restype = ctypes.c_char_p


class NgcError(RuntimeError):
    def __init__(self, code, detail=""):
        self.code = code
        msg = _lib.ngc_strerror(code).decode()
        super().__init__("libngc error %d (%s)%s" % (code, msg, ": " + detail if detail else ""))


def _check(rc, ctx=None):
    if rc != NGC_OK:
        detail = _lib.ngc_last_error(ctx).decode() if ctx else ""
        raise NgcError(rc, detail)


def _dev(t, need=None, dtype=None):
    """Raw device address of a torch tensor (contiguous, on the GPU).  With `need` the tensor
    must hold at least that many elements, with `dtype` ("float32", "int32", "float64") be of
    that type: the library gets a bare pointer and cannot check either."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device buffers must be contiguous GPU tensors")
    if dtype is not None and str(t.dtype) != "torch." + dtype:
        raise ValueError("device buffer has dtype %s, expected %s" % (t.dtype, dtype))
    if need is not None and t.numel() < need:
        raise ValueError("device buffer holds %d elements, the call needs %d" % (t.numel(), need))
    return ctypes.c_void_p(t.data_ptr())


_shapes = {}   # context address -> shape, so that the checks cost no library call per use


def ngc_get_shape(ctx):
    """-> (n, k, layers, d, mlp_d_in) of the context."""
    key = ctx.value if isinstance(ctx, ctypes.c_void_p) else None
    if key in _shapes:
        return _shapes[key]
    n, k, L, din = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    d = ctypes.c_int64(0)
    _check(_lib.ngc_get_shape(ctx, ctypes.byref(n), ctypes.byref(k), ctypes.byref(L), ctypes.byref(d),
                              ctypes.byref(din)), ctx)
    shape = (n.value, k.value, L.value, d.value, din.value)
    if key is not None:
        _shapes[key] = shape
    return shape


def _data_args(ctx, loss, X, y, theta, rows):
    """Checked pointers of the data arguments shared by the gradient calls."""
    n, k, L, d, din = ngc_get_shape(ctx)
    rows = int(rows)
    mlp = int(loss) == NGC_LOSS_MLP2
    width = din if mlp else d
    if rows < 1:
        raise ValueError("rows_per_part must be positive")
    return (_dev(X, k * rows * max(width, 1), "float32"), _dev(y, k * rows, "int32" if mlp else "float32"),
            _dev(theta, d, "float32"))


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def ngc_strerror(code):
    return _lib.ngc_strerror(int(code)).decode()


def ngc_last_error(ctx):
    return _lib.ngc_last_error(ctx).decode()


def ngc_create(n, k, layers, d, hip_stream=0):
    """-> opaque context handle.  hip_stream: integer hipStream_t (0 = default)."""
    layers = [int(s) for s in layers]
    arr = (ctypes.c_int * max(1, len(layers)))(*layers)
    out = ctypes.c_void_p()
    rc = _lib.ngc_create(ctypes.byref(out), int(n), int(k), len(layers), arr, int(d),
                         ctypes.c_void_p(int(hip_stream)))
    _check(rc)
    return out


def ngc_destroy(ctx):
    _shapes.pop(getattr(ctx, "value", None), None)
    _lib.ngc_destroy(ctx)


def ngc_set_code(ctx, layer, B):
    B, p = _host(B, np.float64)
    n, k = ngc_get_shape(ctx)[:2]
    if B.size != n * k:
        raise ValueError("B must be n x k")
    _check(_lib.ngc_set_code(ctx, int(layer), p), ctx)


def ngc_get_code(ctx, layer, n=None, k=None):
    n, k = ngc_get_shape(ctx)[:2]                      # sizes come from the context
    out = np.empty((n, k), np.float64)
    _check(_lib.ngc_get_code(ctx, int(layer), out.ctypes.data_as(ctypes.c_void_p)), ctx)
    return out


def ngc_build_code(ctx, kind, seed):
    _check(_lib.ngc_build_code(ctx, int(kind), int(seed)), ctx)


def ngc_set_mlp2_shape(ctx, d_in, hidden, classes):
    _shapes.pop(getattr(ctx, "value", None), None)
    _check(_lib.ngc_set_mlp2_shape(ctx, int(d_in), int(hidden), int(classes)), ctx)


def ngc_partition_grads(ctx, loss, X, y, theta, rows_per_part, G):
    n, k, L, d, din = ngc_get_shape(ctx)
    pX, py, pt = _data_args(ctx, loss, X, y, theta, rows_per_part)
    _check(_lib.ngc_partition_grads(ctx, int(loss), pX, py, pt, int(rows_per_part),
                                    _dev(G, k * d, "float32")), ctx)


def ngc_partition_grads_static(ctx, loss, X, y, theta, rows_per_part, G):
    n, k, L, d, din = ngc_get_shape(ctx)
    pX, py, pt = _data_args(ctx, loss, X, y, theta, rows_per_part)
    _check(_lib.ngc_partition_grads_static(ctx, int(loss), pX, py, pt, int(rows_per_part),
                                           _dev(G, k * d, "float32")), ctx)


def ngc_encode(ctx, G, layer, C):
    n, k, L, d, din = ngc_get_shape(ctx)
    _check(_lib.ngc_encode(ctx, _dev(G, k * d, "float32"), int(layer), _dev(C, L * n * d, "float32")), ctx)


def _select(fn, ctx, mask, n):
    mask, pm = _host(mask, np.uint8)
    if n != ngc_get_shape(ctx)[0] or mask.size != n:
        raise ValueError("mask must have n entries")
    a = np.zeros(n, np.float64)
    layer = ctypes.c_int(-1)
    resid = ctypes.c_double(0.0)
    rc = fn(ctx, pm, ctypes.byref(layer), a.ctypes.data_as(ctypes.c_void_p), ctypes.byref(resid))
    _check(rc, ctx)
    return layer.value, a, resid.value


def ngc_select_decode_vec(ctx, mask, n):
    """-> (layer, a [n] fp64, residual)."""
    return _select(_lib.ngc_select_decode_vec, ctx, mask, n)


def ngc_set_decode_guard(ctx, kappa_limit):
    """Guarded layer choice: limit on the estimated amplification of message rounding; 0 = off."""
    _check(_lib.ngc_set_decode_guard(ctx, float(kappa_limit)), ctx)


def ngc_select_decode_vec_first(ctx, mask, n):
    return _select(_lib.ngc_select_decode_vec_first, ctx, mask, n)


def ngc_decode(ctx, layer, a, C, g):
    a, pa = _host(a, np.float64)
    n, k, L, d, din = ngc_get_shape(ctx)
    if a.size != n:
        raise ValueError("the decode vector must have n entries")
    _check(_lib.ngc_decode(ctx, int(layer), pa, _dev(C, L * n * d, "float32"), _dev(g, d, "float32")), ctx)


def ngc_encode_decode(ctx, G, layer, a, M, g):
    a, pa = _host(a, np.float64)
    n, k, L, d, din = ngc_get_shape(ctx)
    if a.size != n:
        raise ValueError("the decode vector must have n entries")
    _check(_lib.ngc_encode_decode(ctx, _dev(G, k * d, "float32"), int(layer), pa, _dev(M, n * d, "float32"),
                                  _dev(g, d, "float32")), ctx)


def ngc_coded_rounds(ctx, G, g_round_stride, masks, M, m_round_stride, g):
    """-> (layers [rounds] int32, a [rounds, n] fp64).  masks: [rounds, n] uint8."""
    masks, pm = _host(masks, np.uint8)
    n, k, L, d, din = ngc_get_shape(ctx)
    if masks.ndim != 2 or masks.shape[1] != n or masks.shape[0] < 1:
        raise ValueError("masks must be [rounds, n]")
    rounds = masks.shape[0]
    gs, ms = int(g_round_stride), int(m_round_stride)
    if gs < 0 or ms < 0:
        raise ValueError("strides must not be negative")
    layers = np.zeros(rounds, np.int32)
    a = np.zeros((rounds, n), np.float64)
    _check(_lib.ngc_coded_rounds(ctx, _dev(G, (rounds - 1) * gs + k * d, "float32"), gs, rounds, pm,
                                 _dev(M, (rounds - 1) * ms + n * d, "float32"), ms,
                                 _dev(g, rounds * d, "float32"), layers.ctypes.data_as(ctypes.c_void_p),
                                 a.ctypes.data_as(ctypes.c_void_p)), ctx)
    return layers, a


def ngc_tail_lds_bytes(ctx, vec_width):
    """-> (bytes with the code tables in LDS, bytes without)."""
    w, wo = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(_lib.ngc_tail_lds_bytes(ctx, int(vec_width), ctypes.byref(w), ctypes.byref(wo)), ctx)
    return w.value, wo.value


def ngc_worker_task_count(ctx):
    t = ctypes.c_int(0)
    _check(_lib.ngc_worker_task_count(ctx, ctypes.byref(t)), ctx)
    return t.value


def ngc_worker_schedule(ctx, worker):
    parts = np.zeros(64, np.int32)      # at most k <= 64 partitions
    cnt = ctypes.c_int(0)
    _check(_lib.ngc_worker_schedule(ctx, int(worker), parts.ctypes.data_as(ctypes.c_void_p),
                                    ctypes.byref(cnt)), ctx)
    return [int(p) for p in parts[:cnt.value]]


def _worker_rows(ctx):
    """Rows of W: n workers x (tasks x partitions per task)."""
    n, k = ngc_get_shape(ctx)[:2]
    return n * ngc_worker_task_count(ctx) * (k // n)


def ngc_worker_grads(ctx, loss, X, y, theta, rows_per_part, progress, W):
    progress, pp = _host(progress, np.int32)
    n, k, L, d, din = ngc_get_shape(ctx)
    if progress.size != n:
        raise ValueError("progress must have n entries")
    pX, py, pt = _data_args(ctx, loss, X, y, theta, rows_per_part)
    _check(_lib.ngc_worker_grads(ctx, int(loss), pX, py, pt, int(rows_per_part), pp,
                                 _dev(W, _worker_rows(ctx) * d, "float32")), ctx)


def ngc_worker_encode(ctx, W, progress, C):
    progress, pp = _host(progress, np.int32)
    n, k, L, d, din = ngc_get_shape(ctx)
    if progress.size != n:
        raise ValueError("progress must have n entries")
    _check(_lib.ngc_worker_encode(ctx, _dev(W, _worker_rows(ctx) * d, "float32"), pp,
                                  _dev(C, L * n * d, "float32")), ctx)


def ngc_select_from_progress(ctx, progress, n, min_layer=0):
    """-> (layer, mask [n] uint8, a [n] fp64, residual)."""
    progress, pp = _host(progress, np.int32)
    if n != ngc_get_shape(ctx)[0] or progress.size != n:
        raise ValueError("progress must have n entries")
    a = np.zeros(n, np.float64)
    mask = np.ones(n, np.uint8)
    layer = ctypes.c_int(-1)
    resid = ctypes.c_double(0.0)
    rc = _lib.ngc_select_from_progress(ctx, pp, int(min_layer), ctypes.byref(layer),
                                       mask.ctypes.data_as(ctypes.c_void_p),
                                       a.ctypes.data_as(ctypes.c_void_p), ctypes.byref(resid))
    _check(rc, ctx)
    return layer.value, mask, a, resid.value


def _latency_cdf(fn, n, s, lam, rho, eps, gamma, pe, t):
    t, pt = _host(np.atleast_1d(t), np.float64)
    out = np.zeros(t.size, np.float64)
    _check(fn(int(n), int(s), float(lam), float(rho), float(eps), float(gamma), float(pe), pt,
              int(t.size), out.ctypes.data_as(ctypes.c_void_p)))
    return out


def ngc_latency_cdf_gc(n, sigma, lam, rho, eps, gamma, pe, t):
    return _latency_cdf(_lib.ngc_latency_cdf_gc, n, sigma, lam, rho, eps, gamma, pe, t)


def ngc_latency_cdf_ngc(n, smax, lam, rho, eps, gamma, pe, t):
    return _latency_cdf(_lib.ngc_latency_cdf_ngc, n, smax, lam, rho, eps, gamma, pe, t)


def ngc_latency_simulate(hip_stream, n, smax, lam, rho, eps, gamma, pe, seed, trials, L, Tngc=None):
    _check(_lib.ngc_latency_simulate(ctypes.c_void_p(int(hip_stream)), int(n), int(smax), float(lam),
                                     float(rho), float(eps), float(gamma), float(pe), int(seed),
                                     int(trials), _dev(L, (int(smax) + 1) * int(trials), "float64"),
                                     _dev(Tngc, int(trials), "float64")))


def ngc_build_decoding_table(ctx, layer):
    rows = ctypes.c_int64(0)
    _check(_lib.ngc_build_decoding_table(ctx, int(layer), ctypes.byref(rows)), ctx)
    return rows.value


def ngc_decoding_row_index(ctx, layer, mask):
    mask, pm = _host(mask, np.uint8)
    if mask.size != ngc_get_shape(ctx)[0]:
        raise ValueError("mask must have n entries")
    row = ctypes.c_int64(-1)
    _check(_lib.ngc_decoding_row_index(ctx, int(layer), pm, ctypes.byref(row)), ctx)
    return row.value


def ngc_get_decoding_row(ctx, layer, row, n=None):
    a = np.zeros(ngc_get_shape(ctx)[0], np.float64)
    _check(_lib.ngc_get_decoding_row(ctx, int(layer), int(row), a.ctypes.data_as(ctypes.c_void_p)), ctx)
    return a


def ngc_decode_lookup(ctx, layer, mask, C, g):
    mask, pm = _host(mask, np.uint8)
    n, k, L, d, din = ngc_get_shape(ctx)
    if mask.size != n:
        raise ValueError("mask must have n entries")
    _check(_lib.ngc_decode_lookup(ctx, int(layer), pm, _dev(C, L * n * d, "float32"), _dev(g, d, "float32")), ctx)


def ngc_iteration(ctx, loss, X, y, theta, rows_per_part, mask, scale, G, C, g, n):
    """-> (layer, a [n] fp64)."""
    mask, pm = _host(mask, np.uint8)
    n_ctx, k, L, d, din = ngc_get_shape(ctx)
    if n != n_ctx or mask.size != n:
        raise ValueError("mask must have n entries")
    a = np.zeros(n, np.float64)
    layer = ctypes.c_int(-1)
    pX, py, pt = _data_args(ctx, loss, X, y, theta, rows_per_part)
    _check(_lib.ngc_iteration(ctx, int(loss), pX, py, pt, int(rows_per_part), pm,
                              float(scale), _dev(G, k * d, "float32"), _dev(C, L * n * d, "float32"),
                              _dev(g, d, "float32"), ctypes.byref(layer),
                              a.ctypes.data_as(ctypes.c_void_p)), ctx)
    return layer.value, a


def ngc_update(ctx, theta, g, scale):
    d = ngc_get_shape(ctx)[3]
    _check(_lib.ngc_update(ctx, _dev(theta, d, "float32"), _dev(g, d, "float32"), float(scale)), ctx)


def ngc_sync(ctx):
    _check(_lib.ngc_sync(ctx), ctx)


def _bytes(t):
    return t.numel() * t.element_size()


def ngc_probe_copy(ctx, src, dst, nbytes):
    if int(nbytes) > min(_bytes(src), _bytes(dst)):
        raise ValueError("nbytes exceeds a buffer")
    _check(_lib.ngc_probe_copy(ctx, _dev(src), _dev(dst), int(nbytes)), ctx)


def ngc_probe_read(ctx, src, nbytes):
    if int(nbytes) > _bytes(src):
        raise ValueError("nbytes exceeds the buffer")
    _check(_lib.ngc_probe_read(ctx, _dev(src), int(nbytes)), ctx)


def ngc_profile_enable(ctx, kernels):
    """kernels: True/-1 = all, False/0 = off, or an iterable of kernel names to time."""
    if kernels is True:
        mask = -1
    elif not kernels:
        mask = 0
    elif isinstance(kernels, int):
        mask = kernels
    else:
        mask = 0
        for name in kernels:
            mask |= 1 << NGC_KERNEL_NAMES.index(name)
    _check(_lib.ngc_profile_enable(ctx, mask), ctx)


def ngc_profile_launches(ctx, name):
    """-> durations [ms] of the recorded launches of one kernel, in launch order."""
    ms = np.zeros(4096, np.float64)
    cnt = ctypes.c_int64(0)
    _check(_lib.ngc_profile_launches(ctx, NGC_KERNEL_NAMES.index(name), ms.ctypes.data_as(ctypes.c_void_p),
                                     ms.size, ctypes.byref(cnt)), ctx)
    return ms[:min(cnt.value, ms.size)].copy()


def ngc_profile_read(ctx):
    """-> {kernel name: (launches, total_ms)}."""
    cnt = np.zeros(NGC_KERNEL_COUNT, np.int64)
    ms = np.zeros(NGC_KERNEL_COUNT, np.float64)
    _check(_lib.ngc_profile_read(ctx, cnt.ctypes.data_as(ctypes.c_void_p),
                                 ms.ctypes.data_as(ctypes.c_void_p)), ctx)
    return {name: (int(cnt[i]), float(ms[i])) for i, name in enumerate(NGC_KERNEL_NAMES)}
