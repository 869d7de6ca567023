"""Shared helpers of the GPU parity tests: tolerances and the comparison rule.

Tolerance.  The target is 1e-5 relative error for fp32 gradients and 1e-2 for bf16 gradients.
A single output element can be arbitrarily close to zero (x - lr*g cancels, a weighted average
of numbers of both signs cancels), so "relative" needs a scale that does not vanish with it.
Two rules are applied:

  * per element:  |gpu - ref| <= tol * s_i,  s_i = max(|ref_i|, max_k(|x_k,i| + |lr * g_k,i|)),
    the largest magnitude that enters the sums of column i.  This is the scale fp32 rounding
    errors are proportional to: forming x - lr*g, the K-term weighted sum and the pull costs at
    most (K + 3) * 2^-24 * s_i, i.e. 2.1e-6 * s_i for K = 32, so tol = 1e-5 leaves a factor of
    about five and still rejects any wrong weight, index or term (those show up at 1e-3..1).
  * per (worker, layer) for layers of at least 256 elements:  max|gpu - ref| <= tol * max|ref|.

Norm and weight tables are compared entry by entry at the same relative tolerance.  The bf16
gradient values are used as stored by both sides (the reference widens them exactly), so the
bf16 cases are held to the fp32 tolerance as well.
"""
import numpy as np

TOL = {"f32": 1e-5, "bf16": 1e-2}
TIGHT = 1e-5
BLOCK_MIN = 256


def tol_for(grad_dtype: str) -> float:
    return TOL[grad_dtype]


def grads_to_f64(g: np.ndarray) -> np.ndarray:
    """float32 gradients, or bf16 bit patterns (uint16), as float64."""
    if g.dtype == np.uint16:
        return (g.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return g.astype(np.float64)


def operand_scale(x: np.ndarray, g=None, lr: float = 0.0) -> np.ndarray:
    """s_i = max_k(|x_k,i| + |lr * g_k,i|) over the workers, per column."""
    s = np.abs(x.astype(np.float64))
    if g is not None and lr != 0.0:
        s = s + abs(lr) * np.abs(grads_to_f64(g[:, :x.shape[1]]))
    return s.max(axis=0)


F32_DENORM_STEP = 2.0 ** -149      # spacing of float32 at the bottom of its range


def assert_table_close(got, ref, tol, what, atol=0.0):
    """atol: an absolute allowance added to the relative bound.  The library's tables are float32;
    a test that drives entries below the float32 range passes F32_DENORM_STEP (what the output type
    can resolve there) and nothing else ever passes a nonzero value."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, "%s: shape %r vs %r" % (what, got.shape, ref.shape)
    err = np.abs(got - ref)
    bound = tol * np.abs(ref) + atol
    # an entry that is exactly 0 in the reference (weight of a worker ruled out) must be 0
    bad = err > bound
    if np.any(bad):
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: entry %r gpu=%r ref=%r rel=%g > %g" %
                             (what, i, got[i], ref[i], err[i] / max(abs(ref[i]), 1e-300), tol))
    return float(np.max(err / np.maximum(np.abs(ref), 1e-300))) if err.size else 0.0


def assert_params_close(got, ref, offsets, tol, what, scale, col0=0):
    """got, ref: [K, n] or [n] (n columns starting at flat index col0); offsets: layer offsets
    of the flat vector; scale: per-column operand scale [n] (see the module docstring).
    Returns the worst error relative to the scale."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, "%s: shape %r vs %r" % (what, got.shape, ref.shape)
    if got.ndim == 1:
        got, ref = got[None, :], ref[None, :]
    n = got.shape[1]
    scale = np.asarray(scale, dtype=np.float64)
    assert scale.shape == (n,), "%s: scale shape %r, expected (%d,)" % (what, scale.shape, n)
    if not np.all(np.isfinite(got)):
        raise AssertionError("%s: non-finite output" % what)
    err = np.abs(got - ref)
    bound = tol * np.maximum(np.abs(ref), scale[None, :])
    if np.any(err > bound):
        k, i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: worker %d column %d gpu=%r ref=%r err=%g scale=%g (tol %g)" %
                             (what, k, col0 + i, got[k, i], ref[k, i], err[k, i], scale[i], tol))
    worst = float(np.max(err / np.maximum(np.maximum(np.abs(ref), scale[None, :]), 1e-300))) if err.size else 0.0
    # block rule on the big layers
    off = np.asarray(offsets, dtype=np.int64)
    l = int(np.searchsorted(off, col0, side="right") - 1)
    while l < off.size - 1 and off[l] < col0 + n:
        a = max(int(off[l]), col0) - col0
        b = min(int(off[l + 1]), col0 + n) - col0
        if b - a >= BLOCK_MIN:
            blk_ref = np.max(np.abs(ref[:, a:b]), axis=1)
            blk_err = np.max(err[:, a:b], axis=1)
            if np.any(blk_err > tol * blk_ref):
                k = int(np.argmax(blk_err - tol * blk_ref))
                raise AssertionError("%s: layer %d worker %d block-relative error %g > %g" %
                                     (what, l, k, blk_err[k] / max(blk_ref[k], 1e-300), tol))
        l += 1
    return worst
