"""Python face of the float64 CPU oracle for the GRAWA distributed update.

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  It loads
``libgrawa_oracle.so`` (built from ``grawa_oracle.c`` in this folder with the
host C compiler) and strings its functions together in the order the paper
gives them.  It imports nothing from the GPU package.

Arrays are NumPy: parameters ``x`` are float32 ``[K, ldx]`` (C order), gradients
``g`` are float32 or bfloat16 bit patterns held as uint16, ``[K, ldg]``; layer
offsets are ``L+1`` int64 values with ``off[0] = 0`` and ``off[L] = P``.

Paper passages followed: Sec. 4.3.1 eq. (2) and the center/pull display after
it; Sec. 5.1 eqs. (3)-(4) (MGRAWA); Sec. 5.2 eqs. (5)-(7) (LGRAWA); Algorithms
1 and 2 for the local SGD step, the proximity step and the order of the steps.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "grawa_oracle.c")
_LIB = os.path.join(_HERE, "libgrawa_oracle.so")

F32, BF16 = 0, 1
LAYERSUM, FLAT = 0, 1
_MODES = {"layersum": LAYERSUM, "flat": FLAT, LAYERSUM: LAYERSUM, FLAT: FLAT}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fno-fast-math", "-ffp-contract=off",
             "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib(path: str | None = None):
    """The loaded oracle library (building it first if it is not there)."""
    global _lib
    if path is not None:
        return _bind(C.CDLL(path))
    if _lib is None:
        _lib = _bind(C.CDLL(build()))
    return _lib


def _bind(L):
    i64, dbl, vp, it = C.c_int64, C.c_double, C.c_void_p, C.c_int
    L.oracle_sumsq.argtypes = [vp, it, i64, i64, i64, vp, vp]
    L.oracle_layer_norms.argtypes = [vp, i64, i64, vp]
    L.oracle_model_norms.argtypes = [vp, i64, i64, it, vp]
    L.oracle_weights.argtypes = [vp, i64, i64, vp]
    L.oracle_load_params.argtypes = [vp, i64, i64, i64, i64, vp]
    L.oracle_local_sgd.argtypes = [vp, i64, i64, i64, vp, it, i64, dbl]
    L.oracle_center.argtypes = [vp, i64, i64, i64, vp, i64, vp, vp]
    L.oracle_pull.argtypes = [vp, i64, i64, vp, dbl]
    L.oracle_prox.argtypes = [vp, i64, i64, vp, dbl, dbl]
    L.oracle_norm_momentum.argtypes = [vp, vp, vp, i64, dbl, i64]
    L.oracle_sum_layers.argtypes = [vp, i64, i64, vp]
    L.oracle_nesterov_sgd.argtypes = [vp, vp, i64, i64, i64, vp, it, i64, dbl, dbl, dbl]
    L.oracle_nesterov_sgd.restype = it
    L.oracle_easgd_center.argtypes = [vp, i64, i64, vp, dbl]
    L.oracle_easgd_center.restype = it
    L.oracle_leader.argtypes = [vp, i64]
    L.oracle_leader.restype = i64
    L.oracle_nonfinite.argtypes = [vp, i64]
    L.oracle_nonfinite.restype = it
    for name in ("oracle_norm_momentum", "oracle_sum_layers", "oracle_sumsq", "oracle_layer_norms", "oracle_model_norms", "oracle_weights",
                 "oracle_load_params", "oracle_local_sgd", "oracle_center", "oracle_pull",
                 "oracle_prox"):
        getattr(L, name).restype = it
    return L


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _ok(rc: int, what: str):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (code %d)" % (what, rc))


def _params(x) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype != np.float32 or x.ndim != 2 or not x.flags.c_contiguous:
        raise TypeError("x must be a C-contiguous float32 [K, ldx] array")
    return x


def _grads(g):
    g = np.asarray(g)
    if g.ndim != 2 or not g.flags.c_contiguous:
        raise TypeError("g must be a C-contiguous [K, ldg] array")
    if g.dtype == np.float32:
        return g, F32
    if g.dtype == np.uint16:
        return g, BF16
    raise TypeError("g must be float32 or uint16 (bfloat16 bit patterns)")


def _offsets(off, P=None) -> np.ndarray:
    if off is None:
        off = [0, P]
    off = np.ascontiguousarray(off, dtype=np.int64)
    if off.ndim != 1 or off.size < 2 or off[0] != 0 or np.any(np.diff(off) <= 0):
        raise ValueError("offsets must start at 0 and increase strictly")
    return off


# ----------------------------------------------------------------------------
# the single steps
# ----------------------------------------------------------------------------

def grad_sumsq(g, off, *, _lib=None) -> np.ndarray:
    """S[m, k] = squared Frobenius norm of worker m's gradient in layer k."""
    g, dt = _grads(g)
    off = _offsets(off)
    K, L = g.shape[0], off.size - 1
    S = np.empty((K, L), dtype=np.float64)
    _ok((_lib or lib()).oracle_sumsq(_p(g), dt, K, g.shape[1], L, _p(off), _p(S)), "sumsq")
    return S


def layer_norms(S, *, _lib=None) -> np.ndarray:
    """LGRAWA scores A[m, k], eq. (5)-(6)."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    A = np.empty_like(S)
    _ok((_lib or lib()).oracle_layer_norms(_p(S), S.shape[0], S.shape[1], _p(A)), "layer_norms")
    return A


def model_norms(S, mode="layersum", *, _lib=None) -> np.ndarray:
    """Model-level score A[m]: eq. (3) for 'layersum', eq. (2) for 'flat'."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    A = np.empty(S.shape[0], dtype=np.float64)
    _ok((_lib or lib()).oracle_model_norms(_p(S), S.shape[0], S.shape[1], _MODES[mode], _p(A)),
        "model_norms")
    return A


def weights(A, *, _lib=None) -> np.ndarray:
    """Inverse-norm weights normalised over the worker axis (axis 0)."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    shape = A.shape
    A2 = A.reshape(shape[0], -1)
    B = np.empty_like(A2)
    _ok((_lib or lib()).oracle_weights(_p(A2), A2.shape[0], A2.shape[1], _p(B)), "weights")
    return B.reshape(shape)


def nonfinite(A, *, _lib=None) -> bool:
    """True if any score in A is infinite or NaN."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    rc = (_lib or lib()).oracle_nonfinite(_p(A), A.size)
    if rc < 0:
        raise ValueError("oracle nonfinite rejected its arguments")
    return bool(rc)


def update_chunks(x, beta, off, lam, *, g_sgd=None, lr=0.0, prox_center=None, mu=0.0, tau=1.0,
                  chunk=1 << 20, _lib=None):
    """Yield (i0, i1, x_new[K, n] float64, center[n] float64) over column chunks.

    Per chunk, in the order of Algorithms 1 and 2: optional local SGD step with
    ``g_sgd``, optional proximity step toward ``prox_center``, then center and
    pull with the given weights.  ``beta`` is [K] or [K, L].
    """
    Lb = _lib or lib()
    x = _params(x)
    beta = np.ascontiguousarray(beta, dtype=np.float64)
    K = x.shape[0]
    G = 1 if beta.ndim == 1 else beta.shape[1]
    beta2 = np.ascontiguousarray(beta.reshape(K, G))
    if G > 1:
        off = _offsets(off)
        if off.size - 1 != G:
            raise ValueError("beta has %d columns but there are %d layers" % (G, off.size - 1))
        P = int(off[-1])
    else:
        P = int(off[-1]) if off is not None else x.shape[1]
        off = None
    if g_sgd is not None:
        g_sgd, gdt = _grads(g_sgd)
    if prox_center is not None:
        prox_center = np.ascontiguousarray(prox_center, dtype=np.float64)
    for i0 in range(0, P, chunk):
        i1 = min(P, i0 + chunk)
        n = i1 - i0
        xd = np.empty((K, n), dtype=np.float64)
        _ok(Lb.oracle_load_params(_p(x), K, x.shape[1], i0, i1, _p(xd)), "load_params")
        if g_sgd is not None:
            _ok(Lb.oracle_local_sgd(_p(xd), K, n, i0, _p(g_sgd), gdt, g_sgd.shape[1], float(lr)),
                "local_sgd")
        if prox_center is not None:
            pc = np.ascontiguousarray(prox_center[i0:i1])
            _ok(Lb.oracle_prox(_p(xd), K, n, _p(pc), float(mu), float(tau)), "prox")
        c = np.empty(n, dtype=np.float64)
        _ok(Lb.oracle_center(_p(xd), K, n, i0, _p(beta2), G, _p(off) if off is not None else None,
                             _p(c)), "center")
        _ok(Lb.oracle_pull(_p(xd), K, n, _p(c), float(lam)), "pull")
        yield i0, i1, xd, c


def center_pull(x, beta, off, lam, **kw):
    """Whole-array form of :func:`update_chunks`: returns (x_new, center)."""
    x = _params(x)
    P = int(np.asarray(off)[-1]) if off is not None else x.shape[1]
    xn = np.empty((x.shape[0], P), dtype=np.float64)
    c = np.empty(P, dtype=np.float64)
    for i0, i1, xd, cc in update_chunks(x, beta, off if off is not None else [0, P], lam, **kw):
        xn[:, i0:i1] = xd
        c[i0:i1] = cc
    return xn, c


def local_sgd(x, g, lr, *, P=None, prox_center=None, mu=0.0, tau=1.0, chunk=1 << 20, _lib=None):
    """x_m - lr * g_m for every worker (then the proximity step if asked), float64 [K, P]."""
    Lb = _lib or lib()
    x = _params(x)
    g, gdt = _grads(g)
    K = x.shape[0]
    P = min(x.shape[1], g.shape[1]) if P is None else P
    out = np.empty((K, P), dtype=np.float64)
    for i0 in range(0, P, chunk):
        i1 = min(P, i0 + chunk)
        n = i1 - i0
        xd = np.empty((K, n), dtype=np.float64)
        _ok(Lb.oracle_load_params(_p(x), K, x.shape[1], i0, i1, _p(xd)), "load_params")
        _ok(Lb.oracle_local_sgd(_p(xd), K, n, i0, _p(g), gdt, g.shape[1], float(lr)), "local_sgd")
        if prox_center is not None:
            pc = np.ascontiguousarray(np.asarray(prox_center, dtype=np.float64)[i0:i1])
            _ok(Lb.oracle_prox(_p(xd), K, n, _p(pc), float(mu), float(tau)), "prox")
        out[:, i0:i1] = xd
    return out


# ----------------------------------------------------------------------------
# the distributed phase as a whole
# ----------------------------------------------------------------------------

def mgrawa_weights(g, off, mode="layersum", *, _lib=None):
    """(A[K], beta[K]) of MGRAWA (mode 'layersum', eqs. (3)-(4)) or vanilla GRAWA ('flat', eq. (2))."""
    S = grad_sumsq(g, off, _lib=_lib)
    A = model_norms(S, mode, _lib=_lib)
    return A, weights(A, _lib=_lib)


def lgrawa_weights(g, off, *, _lib=None):
    """(A[K, L], beta[K, L]) of LGRAWA, eqs. (5)-(7)."""
    S = grad_sumsq(g, off, _lib=_lib)
    A = layer_norms(S, _lib=_lib)
    return A, weights(A, _lib=_lib)


def mgrawa_update(x, g, off, lam, mode="layersum", *, g_sgd=None, lr=0.0, _lib=None):
    """One MGRAWA distributed phase.  With ``g_sgd`` the local SGD step is taken
    first (Algorithm 1 order), then center and pull.  Returns a dict with
    x (float64 [K, P]), center, beta, norms."""
    A, beta = mgrawa_weights(g, off, mode, _lib=_lib)
    xn, c = center_pull(x, beta, off, lam, g_sgd=g_sgd, lr=lr, _lib=_lib)
    return {"x": xn, "center": c, "beta": beta, "norms": A}


def lgrawa_update(x, g, off, lam, *, g_sgd=None, lr=0.0, _lib=None):
    """One LGRAWA distributed phase (Algorithm 2 order); same return as mgrawa_update
    with beta and norms of shape [K, L]."""
    A, beta = lgrawa_weights(g, off, _lib=_lib)
    xn, c = center_pull(x, beta, off, lam, g_sgd=g_sgd, lr=lr, _lib=_lib)
    return {"x": xn, "center": c, "beta": beta, "norms": A}


# ----------------------------------------------------------------------------
# Local MGRAWA / LGRAWA (Appendix G): norms from the local optimizer's own gradients
# ----------------------------------------------------------------------------

class LocalScores:
    """The running gradient-norm estimate of Appendix G for K workers x L layers:
    g_mvg (moving average), t (steps since the last communication), g_est."""

    def __init__(self, K, L, gamma, *, _lib=None):
        self.K, self.L, self.gamma = int(K), int(L), float(gamma)
        self.g_mvg = np.zeros((self.K, self.L), dtype=np.float64)
        self.g_est = np.zeros((self.K, self.L), dtype=np.float64)
        self.t = 0
        self._lib = _lib

    def step(self, g, off):
        """One local step: g_cur = per-layer norms of this step's gradients, then the update."""
        g_cur = layer_norms(grad_sumsq(g, off, _lib=self._lib), _lib=self._lib)
        self.t += 1
        _ok((self._lib or lib()).oracle_norm_momentum(_p(self.g_mvg), _p(g_cur), _p(self.g_est),
                                                      self.K * self.L, self.gamma, self.t), "norm_momentum")
        return g_cur

    def weights(self, policy):
        """Weights from the running estimate: 'lgrawa' per layer (eq. (7)), 'mgrawa' from the sum of
        the layer estimates (eq. (3)-(4))."""
        if policy == "lgrawa":
            return weights(self.g_est, _lib=self._lib)
        if policy == "mgrawa":
            A = np.empty(self.K, dtype=np.float64)
            _ok((self._lib or lib()).oracle_sum_layers(_p(self.g_est), self.K, self.L, _p(A)), "sum_layers")
            return weights(A, _lib=self._lib)
        raise ValueError(policy)

    def reset(self):
        """After a communication: g_mvg <- 0, t <- 0."""
        self.g_mvg[:] = 0.0
        self.g_est[:] = 0.0
        self.t = 0


def local_grawa_round(x, grads, off, lr, lam, gamma, policy, *, prox_center=None, mu=0.0, tau=1.0, _lib=None):
    """One round of Appendix G's loop for K workers in lockstep.  For every gradient array in
    `grads` (one per local step): update the running norm estimate, take the SGD step and, if a
    stored center is given, the proximity step.  Then form the center from the estimate by the
    given policy ('lgrawa' or 'mgrawa'), pull, and reset the estimate.
    Returns dict(x=float64 [K, P], center, beta, g_est)."""
    Lb = _lib or lib()
    x = _params(x)
    off = _offsets(off)
    K, P = x.shape[0], int(off[-1])
    sc = LocalScores(K, off.size - 1, gamma, _lib=_lib)
    xd = np.empty((K, P), dtype=np.float64)
    _ok(Lb.oracle_load_params(_p(x), K, x.shape[1], 0, P, _p(xd)), "load_params")
    pc = None if prox_center is None else np.ascontiguousarray(prox_center, dtype=np.float64)
    for g in grads:
        sc.step(g, off)
        garr, gdt = _grads(g)
        _ok(Lb.oracle_local_sgd(_p(xd), K, P, 0, _p(garr), gdt, garr.shape[1], float(lr)), "local_sgd")
        if pc is not None:
            _ok(Lb.oracle_prox(_p(xd), K, P, _p(pc), float(mu), float(tau)), "prox")
    beta = sc.weights(policy)
    est = sc.g_est.copy()
    G = 1 if beta.ndim == 1 else beta.shape[1]
    b2 = np.ascontiguousarray(beta.reshape(K, G))
    c = np.empty(P, dtype=np.float64)
    _ok(Lb.oracle_center(_p(xd), K, P, 0, _p(b2), G, _p(off) if G > 1 else None, _p(c)), "center")
    _ok(Lb.oracle_pull(_p(xd), K, P, _p(c), float(lam)), "pull")
    sc.reset()
    return {"x": xd, "center": c, "beta": beta, "g_est": est}


# ----------------------------------------------------------------------------
# Local optimizer of the experiments and the competing centers
# ----------------------------------------------------------------------------

def nesterov_sgd(x, buf, g, lr, momentum, wd=0.0, *, P=None, _lib=None):
    """One Nesterov-momentum SGD step with weight decay (Appendix B.2.2).  x: float32 [K, ld] or
    float64 [K, P]; buf: float64 [K, P] momentum buffer (zeros at the start).
    Returns (x_new float64 [K, P], buf_new float64 [K, P]); the inputs are not modified."""
    Lb = _lib or lib()
    g, gdt = _grads(g)
    x = np.asarray(x)
    K = x.shape[0]
    P = min(x.shape[1], g.shape[1]) if P is None else P
    xd = np.ascontiguousarray(x[:, :P], dtype=np.float64).copy()
    bd = np.ascontiguousarray(buf, dtype=np.float64).copy()
    if bd.shape != (K, P):
        raise ValueError("buf must be [K, P]")
    _ok(Lb.oracle_nesterov_sgd(_p(xd), _p(bd), K, P, 0, _p(g), gdt, g.shape[1], float(lr), float(momentum),
                               float(wd)), "nesterov_sgd")
    return xd, bd


def easgd_update(x, center, lam, rho, *, P=None, _lib=None):
    """EASGD distributed phase (Appendix F): x_a = mean of the workers, x_C <- (1-rho) x_C + rho x_a,
    then the pull of every worker toward x_C.  Returns (x_new float64 [K, P], center_new [P])."""
    Lb = _lib or lib()
    x = _params(x)
    K = x.shape[0]
    P = x.shape[1] if P is None else P
    xd = np.empty((K, P), dtype=np.float64)
    _ok(Lb.oracle_load_params(_p(x), K, x.shape[1], 0, P, _p(xd)), "load_params")
    c = np.ascontiguousarray(np.asarray(center, dtype=np.float64)[:P]).copy()
    _ok(Lb.oracle_easgd_center(_p(xd), K, P, _p(c), float(rho)), "easgd_center")
    _ok(Lb.oracle_pull(_p(xd), K, P, _p(c), float(lam)), "pull")
    return xd, c


def lsgd_update(x, losses, lam, *, P=None, _lib=None):
    """LSGD distributed phase (Appendix F): the center is the worker with the smallest loss; every
    worker is pulled toward it.  Returns (x_new float64 [K, P], leader index)."""
    Lb = _lib or lib()
    x = _params(x)
    K = x.shape[0]
    P = x.shape[1] if P is None else P
    losses = np.ascontiguousarray(losses, dtype=np.float64)
    if losses.shape != (K,):
        raise ValueError("losses must be [K]")
    lead = int(Lb.oracle_leader(_p(losses), K))
    xd = np.empty((K, P), dtype=np.float64)
    _ok(Lb.oracle_load_params(_p(x), K, x.shape[1], 0, P, _p(xd)), "load_params")
    c = xd[lead].copy()
    _ok(Lb.oracle_pull(_p(xd), K, P, _p(c), float(lam)), "pull")
    return xd, lead
