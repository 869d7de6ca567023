"""ctypes binding of libgrawa.so: the same names and arguments as include/grawa.h.

Argument marshalling only -- every step of the update runs in the library's HIP
kernels.  Tensors are torch CUDA tensors used purely as device memory: the binding
passes ``data_ptr()``, the row stride and the current stream's handle.  There is no
CPU path: if the library has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgrawa.so")

OK, ERR_INVALID_ARG, ERR_ALIGNMENT, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP = range(6)
F32, BF16 = 0, 1
NORM_LAYERSUM, NORM_FLAT = 0, 1
NONFINITE_LAYER_SCORE, NONFINITE_MODEL_SCORE = 1, 2
MAX_WORKERS = 1024

_NORM_MODES = {"layersum": NORM_LAYERSUM, "flat": NORM_FLAT, NORM_LAYERSUM: NORM_LAYERSUM, NORM_FLAT: NORM_FLAT}


class GrawaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


_lib = None


def lib():
    """Load libgrawa.so (once).  Raises if it is not built -- there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "%s is missing: build it first (python -m paper_2403_04206_amd.buildlib, "
            "or __graft_entry__.build())" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i64, it, fl, dbl = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_double
    sig = {
        "grawa_status_string": (C.c_char_p, [it]),
        "grawa_plan_create": (it, [C.POINTER(vp), it, i64, it, vp]),
        "grawa_plan_destroy": (it, [vp]),
        "grawa_plan_info": (it, [vp, C.POINTER(i64), C.POINTER(it)]),
        "grawa_grad_norms": (it, [vp, vp, i64, it, vp, vp]),
        "grawa_mgrawa_update": (it, [vp, vp, i64, vp, i64, it, it, fl, vp, vp, vp]),
        "grawa_lgrawa_update": (it, [vp, vp, i64, vp, i64, it, fl, vp, vp, vp]),
        "grawa_center_pull": (it, [vp, vp, i64, vp, it, fl, vp, vp]),
        "grawa_local_sgd": (it, [vp, i64, vp, i64, it, it, i64, fl, vp]),
        "grawa_mgrawa_update_sgd": (it, [vp, vp, i64, vp, i64, it, it, fl, vp, i64, fl, vp, vp, vp]),
        "grawa_lgrawa_update_sgd": (it, [vp, vp, i64, vp, i64, it, fl, vp, i64, fl, vp, vp, vp]),
        "grawa_local_sgd_prox": (it, [vp, i64, vp, i64, it, it, i64, fl, vp, fl, fl, vp]),
        "grawa_local_step_scored": (it, [vp, vp, i64, vp, i64, it, fl, vp, fl, fl, fl, vp]),
        "grawa_local_lgrawa_update": (it, [vp, vp, i64, fl, vp, vp, vp, vp]),
        "grawa_local_mgrawa_update": (it, [vp, vp, i64, fl, vp, vp, vp, vp]),
        "grawa_local_scores_reset": (it, [vp, vp]),
        "grawa_local_nesterov": (it, [vp, i64, vp, i64, it, vp, i64, it, i64, fl, fl, fl, vp]),
        "grawa_easgd_update": (it, [vp, vp, i64, fl, fl, vp, vp]),
        "grawa_lsgd_update": (it, [vp, vp, i64, vp, fl, vp, vp, vp]),
        "grawa_lgrawa_update_static": (it, [it, i64, it, vp, vp, i64, vp, i64, it, fl, vp, vp, vp]),
        "grawa_plan_nonfinite": (it, [vp, C.POINTER(C.c_uint), it, vp]),
        "grawa_plan_profile": (it, [vp, it]),
        "grawa_plan_profile_read": (it, [vp, C.POINTER(it), C.POINTER(dbl), C.POINTER(dbl)]),
        "grawa_plan_profile_read_call": (it, [vp, it, C.POINTER(dbl), C.POINTER(dbl), C.POINTER(dbl)]),
        "grawa_stream_copy": (it, [vp, vp, i64, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().grawa_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise GrawaError(status, where)


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


_REQUIRE_DEVICE = True     # host-only tests of the shape checks below switch this off


def _on_device(t) -> bool:
    return t.is_cuda or not _REQUIRE_DEVICE


def _covers(t, rows: int, cols: int, what: str):
    """The memory behind a [rows, >= cols] view with row stride t.stride(0) must hold the last row too."""
    if rows < 1 or cols < 1:
        raise ValueError("%s: empty" % what)
    need = (rows - 1) * (t.stride(0) if t.dim() == 2 else 0) + cols
    have = t.untyped_storage().nbytes() // t.element_size() - t.storage_offset()
    if need > have:
        raise ValueError("%s: the tensor's storage holds %d elements from its start, the call reads %d" %
                         (what, have, need))


def _params(x: torch.Tensor, K=None, P=None, what="x"):
    """float32 [K, >= P], unit column stride, rows not overlapping; returns (pointer, row stride)."""
    if x.dtype != torch.float32 or x.dim() != 2 or x.stride(1) != 1 or not _on_device(x):
        raise TypeError("%s must be a float32 CUDA tensor [K, P] with unit column stride" % what)
    K = x.shape[0] if K is None else K
    P = x.shape[1] if P is None else P
    if x.shape[0] != K or x.shape[1] < P:
        raise ValueError("%s has shape %r, expected [%d, >= %d]" % (what, tuple(x.shape), K, P))
    if K > 1 and x.stride(0) < P:
        raise ValueError("%s: row stride %d is shorter than the %d columns used" % (what, x.stride(0), P))
    _covers(x, K, P, what)
    return x.data_ptr(), x.stride(0)


def _grads(g: torch.Tensor, K=None, P=None, what="g"):
    """float32 or bfloat16 [K, >= P]; returns (pointer, row stride, dtype code)."""
    if g.dim() != 2 or g.stride(1) != 1 or not _on_device(g):
        raise TypeError("%s must be a CUDA tensor [K, P] with unit column stride" % what)
    if g.dtype == torch.float32:
        dt = F32
    elif g.dtype == torch.bfloat16:
        dt = BF16
    else:
        raise TypeError("%s must be float32 or bfloat16" % what)
    K = g.shape[0] if K is None else K
    P = g.shape[1] if P is None else P
    if g.shape[0] != K or g.shape[1] < P:
        raise ValueError("%s has shape %r, expected [%d, >= %d]" % (what, tuple(g.shape), K, P))
    if K > 1 and g.stride(0) < P:
        raise ValueError("%s: row stride %d is shorter than the %d columns used" % (what, g.stride(0), P))
    _covers(g, K, P, what)
    return g.data_ptr(), g.stride(0), dt


def _vector(t, n: int, what: str, dtype=torch.float32, optional=True):
    """A contiguous 1-D tensor of at least n elements (a center, the losses, the leader index), or None."""
    if t is None:
        if optional:
            return C.c_void_p(0)
        raise TypeError("%s is required" % what)
    if t.dtype != dtype or t.dim() != 1 or t.stride(0) != 1 or not _on_device(t):
        raise TypeError("%s must be a contiguous 1-D %s CUDA tensor" % (what, str(dtype).replace("torch.", "")))
    if t.numel() < n:
        raise ValueError("%s holds %d elements, the call needs %d" % (what, t.numel(), n))
    _covers(t, 1, n, what)
    return C.c_void_p(t.data_ptr())


def _table(t, shape, what: str):
    """A contiguous float32 tensor of exactly `shape` (weights, norms, estimates), or None."""
    if t is None:
        return C.c_void_p(0)
    if t.dtype != torch.float32 or not t.is_contiguous() or not _on_device(t):
        raise TypeError("%s must be a contiguous float32 CUDA tensor" % what)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %r, expected %r" % (what, tuple(t.shape), tuple(shape)))
    return C.c_void_p(t.data_ptr())


class Plan:
    """grawa_plan_t: problem shape, tile map and device workspace (see include/grawa.h)."""

    def __init__(self, K: int, P: int, layer_offsets=None):
        if layer_offsets is None:
            L = 1
            off_p = None
            self._off = None
        else:
            self._off = np.ascontiguousarray(layer_offsets, dtype=np.int64)
            L = self._off.size - 1
            off_p = self._off.ctypes.data_as(C.c_void_p)
        self.K, self.P, self.L = int(K), int(P), int(L)
        self._h = C.c_void_p()
        _check(lib().grawa_plan_create(C.byref(self._h), self.K, self.P, self.L, off_p), "grawa_plan_create")

    # -- lifetime -------------------------------------------------------------------
    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            torch.cuda.synchronize()
            st = lib().grawa_plan_destroy(self._h)
            self._h = C.c_void_p()
            _check(st, "grawa_plan_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    def info(self):
        n, t = C.c_int64(), C.c_int()
        _check(lib().grawa_plan_info(self._h, C.byref(n), C.byref(t)), "grawa_plan_info")
        return {"n_tiles": n.value, "tile_elems": t.value}

    # -- the calls ------------------------------------------------------------------
    # Every tensor's dtype, shape and extent is checked against the plan's (K, P, L) here: the C side
    # sees only pointers and strides, and a short buffer would be a device memory fault.
    def _xg(self, x, g):
        xp, ldx = _params(x, self.K, self.P)
        gp, ldg, dt = _grads(g, self.K, self.P)
        return xp, ldx, gp, ldg, dt

    def grad_norms(self, g, norms_out=None, stream=None):
        gp, ldg, dt = _grads(g, self.K, self.P)
        if norms_out is None:
            norms_out = torch.empty((self.K, self.L), dtype=torch.float32, device=g.device)
        _check(lib().grawa_grad_norms(self._h, gp, ldg, dt, _table(norms_out, (self.K, self.L), "norms_out"),
                                      _stream(stream)), "grawa_grad_norms")
        return norms_out

    def mgrawa_update(self, x, g, lam, mode="layersum", center_out=None, weights_out=None, stream=None):
        xp, ldx, gp, ldg, dt = self._xg(x, g)
        _check(lib().grawa_mgrawa_update(self._h, xp, ldx, gp, ldg, dt, _NORM_MODES[mode], float(lam),
                                         _vector(center_out, self.P, "center_out"),
                                         _table(weights_out, (self.K,), "weights_out"), _stream(stream)),
               "grawa_mgrawa_update")

    def lgrawa_update(self, x, g, lam, center_out=None, weights_out=None, stream=None):
        xp, ldx, gp, ldg, dt = self._xg(x, g)
        _check(lib().grawa_lgrawa_update(self._h, xp, ldx, gp, ldg, dt, float(lam),
                                         _vector(center_out, self.P, "center_out"),
                                         _table(weights_out, (self.K, self.L), "weights_out"), _stream(stream)),
               "grawa_lgrawa_update")

    def mgrawa_update_sgd(self, x, g, lam, g_sgd, lr, mode="layersum", center_out=None, weights_out=None,
                          stream=None):
        xp, ldx, gp, ldg, dt = self._xg(x, g)
        sp, lds, dts = _grads(g_sgd, self.K, self.P, "g_sgd")
        if dts != dt:
            raise TypeError("g and g_sgd must have the same dtype")
        _check(lib().grawa_mgrawa_update_sgd(self._h, xp, ldx, gp, ldg, dt, _NORM_MODES[mode], float(lam), sp, lds,
                                             float(lr), _vector(center_out, self.P, "center_out"),
                                             _table(weights_out, (self.K,), "weights_out"), _stream(stream)),
               "grawa_mgrawa_update_sgd")

    def lgrawa_update_sgd(self, x, g, lam, g_sgd, lr, center_out=None, weights_out=None, stream=None):
        xp, ldx, gp, ldg, dt = self._xg(x, g)
        sp, lds, dts = _grads(g_sgd, self.K, self.P, "g_sgd")
        if dts != dt:
            raise TypeError("g and g_sgd must have the same dtype")
        _check(lib().grawa_lgrawa_update_sgd(self._h, xp, ldx, gp, ldg, dt, float(lam), sp, lds, float(lr),
                                             _vector(center_out, self.P, "center_out"),
                                             _table(weights_out, (self.K, self.L), "weights_out"), _stream(stream)),
               "grawa_lgrawa_update_sgd")

    def center_pull(self, x, weights, lam, center_out=None, stream=None):
        xp, ldx = _params(x, self.K, self.P)
        if weights is None or weights.dim() not in (1, 2):
            raise TypeError("weights must be a contiguous float32 tensor [K] or [K, L]")
        per_layer = 1 if weights.dim() == 2 else 0
        wp = _table(weights, (self.K, self.L) if per_layer else (self.K,), "weights")
        _check(lib().grawa_center_pull(self._h, xp, ldx, wp, per_layer, float(lam),
                                       _vector(center_out, self.P, "center_out"), _stream(stream)),
               "grawa_center_pull")

    # -- Local MGRAWA / LGRAWA (Appendix G) -----------------------------------------
    def local_step_scored(self, x, g, lr, gamma, center=None, mu=0.0, tau=1.0, stream=None):
        xp, ldx, gp, ldg, dt = self._xg(x, g)
        _check(lib().grawa_local_step_scored(self._h, xp, ldx, gp, ldg, dt, float(lr),
                                             _vector(center, self.P, "center"), float(mu), float(tau), float(gamma),
                                             _stream(stream)), "grawa_local_step_scored")

    def local_lgrawa_update(self, x, lam, center_out=None, weights_out=None, est_out=None, stream=None):
        xp, ldx = _params(x, self.K, self.P)
        _check(lib().grawa_local_lgrawa_update(self._h, xp, ldx, float(lam), _vector(center_out, self.P, "center_out"),
                                               _table(weights_out, (self.K, self.L), "weights_out"),
                                               _table(est_out, (self.K, self.L), "est_out"), _stream(stream)),
               "grawa_local_lgrawa_update")

    def local_mgrawa_update(self, x, lam, center_out=None, weights_out=None, est_out=None, stream=None):
        xp, ldx = _params(x, self.K, self.P)
        _check(lib().grawa_local_mgrawa_update(self._h, xp, ldx, float(lam), _vector(center_out, self.P, "center_out"),
                                               _table(weights_out, (self.K,), "weights_out"),
                                               _table(est_out, (self.K, self.L), "est_out"), _stream(stream)),
               "grawa_local_mgrawa_update")

    def local_scores_reset(self, stream=None):
        _check(lib().grawa_local_scores_reset(self._h, _stream(stream)), "grawa_local_scores_reset")

    # -- competing centers (Appendix F) ---------------------------------------------
    def easgd_update(self, x, lam, rho, center, stream=None):
        xp, ldx = _params(x, self.K, self.P)
        _check(lib().grawa_easgd_update(self._h, xp, ldx, float(lam), float(rho),
                                        _vector(center, self.P, "center", optional=False), _stream(stream)),
               "grawa_easgd_update")

    def lsgd_update(self, x, losses, lam, center_out=None, leader_out=None, stream=None):
        xp, ldx = _params(x, self.K, self.P)
        _check(lib().grawa_lsgd_update(self._h, xp, ldx, _vector(losses, self.K, "losses", optional=False), float(lam),
                                       _vector(center_out, self.P, "center_out"),
                                       _vector(leader_out, 1, "leader_out", dtype=torch.int32), _stream(stream)),
               "grawa_lsgd_update")

    def nonfinite(self, clear=True, stream=None):
        """grawa_plan_nonfinite: the NONFINITE_* bits seen since the last clear (waits for the stream)."""
        f = C.c_uint()
        _check(lib().grawa_plan_nonfinite(self._h, C.byref(f), 1 if clear else 0, _stream(stream)),
               "grawa_plan_nonfinite")
        return f.value

    # -- measurement aid ------------------------------------------------------------
    def profile(self, enable: bool):
        _check(lib().grawa_plan_profile(self._h, 1 if enable else 0), "grawa_plan_profile")

    def profile_read(self):
        n, a, b = C.c_int(), C.c_double(), C.c_double()
        _check(lib().grawa_plan_profile_read(self._h, C.byref(n), C.byref(a), C.byref(b)), "grawa_plan_profile_read")
        return {"calls": n.value, "norm_ms": a.value, "pull_ms": b.value}

    def profile_read_call(self, i):
        a, b, c = C.c_double(), C.c_double(), C.c_double()
        _check(lib().grawa_plan_profile_read_call(self._h, int(i), C.byref(a), C.byref(b), C.byref(c)),
               "grawa_plan_profile_read_call")
        return {"norm_ms": a.value, "pull_ms": b.value, "span_ms": c.value}


def _row_shape(x, P):
    K = x.shape[0] if x.dim() == 2 else 0
    return K, (x.shape[1] if P is None else int(P))


def local_sgd(x, g, lr, P=None, stream=None):
    """grawa_local_sgd: x[k] -= lr * g[k] on the first P columns of every row."""
    K, P = _row_shape(x, P)
    xp, ldx = _params(x, K, P)
    gp, ldg, dt = _grads(g, K, P)
    _check(lib().grawa_local_sgd(xp, ldx, gp, ldg, dt, K, P, float(lr), _stream(stream)), "grawa_local_sgd")


def local_sgd_prox(x, g, lr, center, mu, tau, P=None, stream=None):
    """grawa_local_sgd_prox: SGD step then the proximity step toward the stored center."""
    K, P = _row_shape(x, P)
    xp, ldx = _params(x, K, P)
    gp, ldg, dt = _grads(g, K, P)
    _check(lib().grawa_local_sgd_prox(xp, ldx, gp, ldg, dt, K, P, float(lr),
                                      _vector(center, P, "center", optional=False), float(mu), float(tau),
                                      _stream(stream)), "grawa_local_sgd_prox")


def local_nesterov(x, g, buf, lr, momentum, weight_decay=0.0, P=None, stream=None):
    """grawa_local_nesterov: one Nesterov-momentum SGD step with weight decay; buf is updated in place."""
    K, P = _row_shape(x, P)
    xp, ldx = _params(x, K, P)
    bp, ldb = _params(buf, K, P, "buf")
    gp, ldg, dt = _grads(g, K, P)
    _check(lib().grawa_local_nesterov(xp, ldx, gp, ldg, dt, bp, ldb, K, P, float(lr), float(momentum),
                                      float(weight_decay), _stream(stream)), "grawa_local_nesterov")


def lgrawa_update_static(x, g, layer_offsets_dev, lam, center_out=None, weights_out=None, P=None, stream=None):
    """grawa_lgrawa_update_static: the LGRAWA update without a plan and without any allocation;
    layer_offsets_dev is an int64 CUDA tensor [L+1]."""
    K, P = _row_shape(x, P)
    xp, ldx = _params(x, K, P)
    gp, ldg, dt = _grads(g, K, P)
    off = layer_offsets_dev
    if off is None or off.dtype != torch.int64 or off.dim() != 1 or not _on_device(off) or not off.is_contiguous() \
            or off.numel() < 2:
        raise TypeError("layer_offsets_dev must be a contiguous int64 CUDA tensor [L+1]")
    L = off.numel() - 1
    _check(lib().grawa_lgrawa_update_static(K, P, L, _ptr(off), xp, ldx, gp, ldg, dt, float(lam),
                                            _vector(center_out, P, "center_out"),
                                            _table(weights_out, (K, L), "weights_out"), _stream(stream)),
           "grawa_lgrawa_update_static")


def stream_copy(dst, src, stream=None):
    """grawa_stream_copy over two equally sized contiguous tensors."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(lib().grawa_stream_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "grawa_stream_copy")
