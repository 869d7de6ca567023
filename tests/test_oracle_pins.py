"""Pins for the float64 oracle: exact rationals, closed forms, invariants, library
cross-checks and brute force.  None of these needs a GPU and none calls the GPU
library.  Each test names the passage of the paper that fixes the expected value.
"""
import json
import math
import os
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import grawa_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def fr_list(v):
    return [Fr(s) for s in v]


def as_float(v):
    return np.array([float(f) for f in v], dtype=np.float64)


def theta_weights(norms):
    """beta_m = Theta / A_m with Theta = prod(A) / sum_i(prod(A)/A_i): Sec. 4.3.1 eq. (2),
    in exact rationals (a different expression from the oracle's (1/A)/sum(1/A))."""
    prod = Fr(1)
    for a in norms:
        prod *= a
    theta = prod / sum(prod / a for a in norms)
    return [theta / a for a in norms]


def exact_update(x, beta_cols, off, lam):
    """Center and pull in exact rationals.  beta_cols[l][m] is the weight of worker m in
    layer l.  Display after eq. (2); eq. (7) for the per-layer center."""
    K, P = len(x), len(x[0])
    layer_of = []
    for l in range(len(off) - 1):
        layer_of += [l] * (off[l + 1] - off[l])
    c = [sum(beta_cols[layer_of[i]][m] * x[m][i] for m in range(K)) for i in range(P)]
    xn = [[(1 - lam) * x[m][i] + lam * c[i] for i in range(P)] for m in range(K)]
    return c, xn


# ----------------------------------------------------------------------------
# hand-worked fixtures
# ----------------------------------------------------------------------------

def test_ex1_two_workers_exact():
    ex = json.load(open(os.path.join(GOLD, "ex1_two_workers.json")))
    lam = Fr(ex["lambda"])
    g = np.array(ex["g"], dtype=np.float32)
    x = np.array(ex["x"], dtype=np.float32)
    off = ex["offsets"]
    # the fixture agrees with the paper's closed form, recomputed here exactly
    assert theta_weights(fr_list(ex["norms"])) == fr_list(ex["beta"])
    c_ex, xn_ex = exact_update([[Fr(int(v)) for v in r] for r in ex["x"]], [fr_list(ex["beta"])], off, lam)
    assert c_ex == fr_list(ex["center"])
    assert xn_ex == [fr_list(r) for r in ex["x_new"]]
    # the oracle agrees with the fixture, in all three weightings (one layer: they coincide)
    for res in (orc.mgrawa_update(x, g, off, float(lam), "layersum"),
                orc.mgrawa_update(x, g, off, float(lam), "flat"),
                orc.lgrawa_update(x, g, off, float(lam))):
        np.testing.assert_allclose(np.ravel(res["norms"]), as_float(fr_list(ex["norms"])), rtol=0, atol=0)
        np.testing.assert_allclose(np.ravel(res["beta"]), as_float(fr_list(ex["beta"])), rtol=1e-15)
        np.testing.assert_allclose(res["center"], as_float(fr_list(ex["center"])), rtol=1e-15)
        np.testing.assert_allclose(res["x"], np.array([as_float(fr_list(r)) for r in ex["x_new"]]), rtol=1e-15)


def test_ex2_three_weightings_exact():
    ex = json.load(open(os.path.join(GOLD, "ex2_three_workers_two_layers.json")))
    lam = Fr(ex["lambda"])
    g = np.array(ex["g"], dtype=np.float32)
    x = np.array(ex["x"], dtype=np.float32)
    xq = [[Fr(int(v)) for v in r] for r in ex["x"]]
    off = ex["offsets"]
    ln = [fr_list(r) for r in ex["layer_norms"]]

    # fixture self-consistency against the definitions, in exact arithmetic
    for m, row in enumerate(ex["g"]):
        for l in range(2):
            assert sum(Fr(v) ** 2 for v in row[off[l]:off[l + 1]]) == ln[m][l] ** 2
    assert [sum(r) for r in ln] == fr_list(ex["mgrawa"]["norms"])                      # eq. (3)
    assert [sum(a * a for a in r) for r in ln] == fr_list(ex["flat"]["sumsq"])        # eq. (2)
    bm = theta_weights(fr_list(ex["mgrawa"]["norms"]))                                # eq. (4)
    assert bm == fr_list(ex["mgrawa"]["beta"])
    c, xn = exact_update(xq, [bm, bm], off, lam)
    assert c == fr_list(ex["mgrawa"]["center"]) and xn[0] == fr_list(ex["mgrawa"]["x_new_worker0"])
    bl = [theta_weights([ln[m][l] for m in range(3)]) for l in range(2)]              # eq. (7)
    assert [[bl[l][m] for l in range(2)] for m in range(3)] == [fr_list(r) for r in ex["lgrawa"]["beta"]]
    cl, xl = exact_update(xq, bl, off, lam)
    assert cl == fr_list(ex["lgrawa"]["center"]) and xl[0] == fr_list(ex["lgrawa"]["x_new_worker0"])

    # oracle against the fixture
    S = orc.grad_sumsq(g, off)
    np.testing.assert_array_equal(orc.layer_norms(S), np.array([as_float(r) for r in ln]))
    r = orc.mgrawa_update(x, g, off, float(lam), "layersum")
    np.testing.assert_array_equal(r["norms"], as_float(fr_list(ex["mgrawa"]["norms"])))
    np.testing.assert_allclose(r["beta"], as_float(bm), rtol=1e-15)
    np.testing.assert_allclose(r["center"], as_float(c), rtol=1e-15)
    np.testing.assert_allclose(r["x"], np.array([as_float(v) for v in xn]), rtol=1e-15)
    r = orc.lgrawa_update(x, g, off, float(lam))
    np.testing.assert_allclose(r["beta"], np.array([as_float(v) for v in zip(*bl)]), rtol=1e-15)
    np.testing.assert_allclose(r["center"], as_float(cl), rtol=1e-15)
    np.testing.assert_allclose(r["x"], np.array([as_float(v) for v in xl]), rtol=1e-15)
    # vanilla GRAWA on the flattened gradient: norms sqrt(194), sqrt(125), sqrt(290)
    r = orc.mgrawa_update(x, g, off, float(lam), "flat")
    want = np.sqrt(as_float(fr_list(ex["flat"]["sumsq"])))
    np.testing.assert_allclose(r["norms"], want, rtol=1e-15)
    inv = 1.0 / want
    np.testing.assert_allclose(r["beta"], inv / inv.sum(), rtol=1e-15)
    # the three weightings are different on this example (triangle inequality remark, Sec. 5)
    assert not np.allclose(r["beta"], as_float(bm), rtol=1e-3)


# ----------------------------------------------------------------------------
# brute force in exact rationals on random tiny problems
# ----------------------------------------------------------------------------

TRIPLES = [(3, 4), (5, 12), (8, 15), (7, 24), (20, 21), (9, 40), (12, 35)]


def _rational_problem(rng, K, sizes):
    """Integer gradients whose every layer norm is an integer: each layer is one scaled
    Pythagorean pair placed at random positions, zeros elsewhere."""
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(off[-1])
    g = np.zeros((K, P), dtype=np.float32)
    norms = [[None] * len(sizes) for _ in range(K)]
    for m in range(K):
        for l, n in enumerate(sizes):
            a, b = TRIPLES[rng.integers(len(TRIPLES))]
            s = int(rng.integers(1, 5))
            sign = rng.choice([-1, 1], size=2)
            if n >= 2:
                pos = rng.choice(n, size=2, replace=False)
                g[m, off[l] + pos[0]] = sign[0] * s * a
                g[m, off[l] + pos[1]] = sign[1] * s * b
                norms[m][l] = Fr(s * math.isqrt(a * a + b * b))
            else:
                g[m, off[l]] = sign[0] * s * a
                norms[m][l] = Fr(s * a)
    x = rng.integers(-20, 21, size=(K, P)).astype(np.float32)
    return off, g, x, norms


@pytest.mark.parametrize("seed", range(6))
def test_bruteforce_rationals(seed):
    rng = np.random.default_rng(1000 + seed)
    K = int(rng.integers(1, 6))
    sizes = [int(v) for v in rng.integers(1, 6, size=int(rng.integers(1, 5)))]
    off, g, x, norms = _rational_problem(rng, K, sizes)
    L = len(sizes)
    lam = Fr(int(rng.integers(0, 11)), 10)
    xq = [[Fr(int(v)) for v in r] for r in x]
    # LGRAWA, eqs. (5)-(7)
    bl = [theta_weights([norms[m][l] for m in range(K)]) for l in range(L)]
    c, xn = exact_update(xq, bl, list(off), lam)
    r = orc.lgrawa_update(x, g, off, float(lam))
    np.testing.assert_allclose(r["norms"], np.array([as_float(v) for v in norms]), rtol=0, atol=0)
    np.testing.assert_allclose(r["beta"], np.array([as_float(v) for v in zip(*bl)]), rtol=4e-16)
    np.testing.assert_allclose(r["center"], as_float(c), rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(r["x"], np.array([as_float(v) for v in xn]), rtol=1e-14, atol=1e-14)
    # MGRAWA, eqs. (3)-(4)
    A = [sum(norms[m]) for m in range(K)]
    bm = theta_weights(A)
    c, xn = exact_update(xq, [bm] * L, list(off), lam)
    r = orc.mgrawa_update(x, g, off, float(lam), "layersum")
    np.testing.assert_array_equal(r["norms"], as_float(A))
    np.testing.assert_allclose(r["beta"], as_float(bm), rtol=4e-16)
    np.testing.assert_allclose(r["center"], as_float(c), rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(r["x"], np.array([as_float(v) for v in xn]), rtol=1e-14, atol=1e-14)
    # weights are a probability vector (App. E uses beta_i in [0,1], sum 1)
    assert sum(bm) == 1 and all(0 < b <= 1 for b in bm)
    assert sum(sum(col) for col in bl) == L          # "sum_k sum_m beta = K" of Sec. 5.2


# ----------------------------------------------------------------------------
# library cross-checks
# ----------------------------------------------------------------------------

def _bf16_bits(a32):
    import torch
    return torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_norms_against_numpy_linalg():
    rng = np.random.default_rng(7)
    sizes = [1, 3, 64, 1000, 257, 2]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    K, P = 5, int(off[-1])
    g = (rng.standard_normal((K, P + 3)) * 10.0 ** rng.uniform(-3, 1, size=(K, 1))).astype(np.float32)
    S = orc.grad_sumsq(g, off)
    A = orc.layer_norms(S)
    for m in range(K):
        for l in range(len(sizes)):
            blk = g[m, off[l]:off[l + 1]].astype(np.float64)
            assert A[m, l] == pytest.approx(np.linalg.norm(blk), rel=1e-14)
            assert S[m, l] == pytest.approx(math.fsum(v * v for v in blk), rel=1e-14)
        assert orc.model_norms(S, "flat")[m] == pytest.approx(np.linalg.norm(g[m, :P].astype(np.float64)), rel=1e-14)
        assert orc.model_norms(S, "layersum")[m] == pytest.approx(
            sum(np.linalg.norm(g[m, off[l]:off[l + 1]].astype(np.float64)) for l in range(len(sizes))), rel=1e-14)
    # the padding columns beyond P (ldg > P) are never read into any norm
    g2 = g.copy()
    g2[:, P:] = 1e30
    np.testing.assert_array_equal(orc.grad_sumsq(g2, off), S)


def test_bf16_widening_every_bit_pattern():
    import torch
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    keep = np.isfinite(ref)
    bits, ref = bits[keep], ref[keep]
    # one layer per element: sqrt of the sum of one square is |value|
    n = bits.size
    off = np.arange(n + 1, dtype=np.int64)
    S = orc.grad_sumsq(bits.reshape(1, n).copy(), off)
    np.testing.assert_array_equal(S[0], ref * ref)
    # and the signed value through the SGD step with eta = -1 from x = 0
    out = orc.local_sgd(np.zeros((1, n), np.float32), bits.reshape(1, n).copy(), -1.0)
    np.testing.assert_array_equal(out[0], ref)


def test_local_sgd_is_axpy():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 777)).astype(np.float32)
    g = rng.standard_normal((3, 800)).astype(np.float32)
    out = orc.local_sgd(x, g, 0.1, P=777)
    np.testing.assert_allclose(out, x.astype(np.float64) + (-0.1) * g[:, :777].astype(np.float64), rtol=1e-15)
    gb = _bf16_bits(g)
    import torch
    gb64 = torch.from_numpy(gb.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    out = orc.local_sgd(x, gb, 0.25, P=777)
    np.testing.assert_allclose(out, x.astype(np.float64) - 0.25 * gb64[:, :777], rtol=1e-15)
    # eta = 0 leaves the parameters unchanged; the step is linear in eta
    np.testing.assert_array_equal(orc.local_sgd(x, g, 0.0, P=777), x.astype(np.float64))
    d1 = orc.local_sgd(x, g, 0.5, P=777) - x
    d2 = orc.local_sgd(x, g, 1.0, P=777) - x
    np.testing.assert_allclose(2 * d1, d2, rtol=1e-12, atol=1e-15)


# ----------------------------------------------------------------------------
# invariants the paper fixes
# ----------------------------------------------------------------------------

def _random_problem(seed, K=4, sizes=(5, 1, 33, 8, 130), ld_pad=0, bf16=False):
    rng = np.random.default_rng(seed)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(off[-1])
    x = (0.05 * rng.standard_normal((K, P + ld_pad))).astype(np.float32)
    s = 10.0 ** rng.uniform(-3, 1, size=(K, len(sizes)))
    g = rng.standard_normal((K, P + ld_pad))
    for l in range(len(sizes)):
        g[:, off[l]:off[l + 1]] *= s[:, l:l + 1]
    g = g.astype(np.float32)
    if bf16:
        g = _bf16_bits(g)
    return off, x, g


@pytest.mark.parametrize("bf16", [False, True])
def test_weight_invariants(bf16):
    off, x, g = _random_problem(11, K=6, bf16=bf16)
    L = off.size - 1
    for mode in ("layersum", "flat"):
        A, b = orc.mgrawa_weights(g, off, mode)
        assert b.shape == (6,) and np.all(b > 0) and np.all(b < 1)
        assert b.sum() == pytest.approx(1.0, abs=1e-15)
        np.testing.assert_allclose(b * A, (b * A)[0], rtol=1e-14)       # beta_m * A_m is the same Theta for all m
        assert np.argmax(b) == np.argmin(A)
    A, b = orc.lgrawa_weights(g, off)
    assert b.shape == (6, L) and np.all(b > 0)
    np.testing.assert_allclose(b.sum(axis=0), 1.0, atol=1e-15)
    assert b.sum() == pytest.approx(L, abs=1e-13)                       # Sec. 5.2
    np.testing.assert_allclose(b * A, np.broadcast_to((b * A)[0], b.shape), rtol=1e-14)


def test_equal_norms_give_plain_average():
    # same gradient magnitudes for every worker (signs and positions differ): beta = 1/K
    off, x, g = _random_problem(5, K=5)
    rng = np.random.default_rng(0)
    base = np.abs(g[0])
    for m in range(g.shape[0]):
        for l in range(off.size - 1):
            seg = base[off[l]:off[l + 1]].copy()
            rng.shuffle(seg)
            g[m, off[l]:off[l + 1]] = seg * rng.choice([-1, 1], size=seg.size)
    P = int(off[-1])
    mean = x[:, :P].astype(np.float64).mean(axis=0)
    for r in (orc.mgrawa_update(x, g, off, 0.3), orc.mgrawa_update(x, g, off, 0.3, "flat"),
              orc.lgrawa_update(x, g, off, 0.3)):
        np.testing.assert_allclose(r["beta"], 0.2, rtol=1e-6)   # shuffled sums differ in the last bits
        np.testing.assert_allclose(r["center"], mean, atol=1e-8)


def test_scale_invariance():
    off, x, g = _random_problem(21, K=4)
    L = off.size - 1
    base_m = orc.mgrawa_update(x, g, off, 0.2)
    base_l = orc.lgrawa_update(x, g, off, 0.2)
    # a common positive factor changes nothing (so sum vs mean over the N samples of G_k is immaterial)
    for cfac in (0.25, 8.0, 1024.0):
        np.testing.assert_allclose(orc.mgrawa_update(x, g * np.float32(cfac), off, 0.2)["x"], base_m["x"], rtol=1e-13)
        np.testing.assert_allclose(orc.lgrawa_update(x, g * np.float32(cfac), off, 0.2)["x"], base_l["x"], rtol=1e-13)
    # LGRAWA is also invariant to a separate factor per layer; MGRAWA is not
    g2 = g.copy()
    for l in range(L):
        g2[:, off[l]:off[l + 1]] *= np.float32(2.0 ** (l - 2))
    np.testing.assert_allclose(orc.lgrawa_update(x, g2, off, 0.2)["x"], base_l["x"], rtol=1e-13)
    assert not np.allclose(orc.mgrawa_update(x, g2, off, 0.2)["beta"], base_m["beta"], rtol=1e-6)


def test_lgrawa_is_blockwise_mgrawa_and_single_layer_cases_coincide():
    off, x, g = _random_problem(33, K=3, ld_pad=5)
    P = int(off[-1])
    full = orc.lgrawa_update(x, g, off, 0.4)
    for l in range(off.size - 1):
        a, b = int(off[l]), int(off[l + 1])
        xs = np.ascontiguousarray(x[:, a:b])
        gs = np.ascontiguousarray(g[:, a:b])
        for mode in ("layersum", "flat"):
            one = orc.mgrawa_update(xs, gs, [0, b - a], 0.4, mode)
            np.testing.assert_allclose(full["x"][:, a:b], one["x"], rtol=1e-15)
            np.testing.assert_allclose(full["beta"][:, l], one["beta"], rtol=1e-15)
    # one layer: LGRAWA == MGRAWA == vanilla GRAWA
    o1 = [0, P]
    a = orc.lgrawa_update(x, g, o1, 0.4)
    b = orc.mgrawa_update(x, g, o1, 0.4, "layersum")
    c = orc.mgrawa_update(x, g, o1, 0.4, "flat")
    np.testing.assert_array_equal(a["x"], b["x"])
    np.testing.assert_array_equal(a["x"], c["x"])
    np.testing.assert_array_equal(np.ravel(a["beta"]), b["beta"])


def test_triangle_inequality_between_the_two_model_norms():
    off, x, g = _random_problem(44, K=5)
    S = orc.grad_sumsq(g, off)
    assert np.all(orc.model_norms(S, "layersum") >= orc.model_norms(S, "flat"))
    # equality iff at most one layer is non-zero
    g1 = np.zeros_like(g)
    g1[:, off[2]:off[3]] = g[:, off[2]:off[3]]
    S1 = orc.grad_sumsq(g1, off)
    np.testing.assert_allclose(orc.model_norms(S1, "layersum"), orc.model_norms(S1, "flat"), rtol=1e-15)


def test_worker_permutation():
    off, x, g = _random_problem(55, K=5)
    perm = np.array([3, 0, 4, 1, 2])
    for fn in (lambda a, b: orc.mgrawa_update(a, b, off, 0.15), lambda a, b: orc.lgrawa_update(a, b, off, 0.15)):
        r0 = fn(x, g)
        r1 = fn(np.ascontiguousarray(x[perm]), np.ascontiguousarray(g[perm]))
        np.testing.assert_allclose(r1["x"], r0["x"][perm], rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(r1["center"], r0["center"], rtol=1e-13, atol=1e-16)
        np.testing.assert_allclose(r1["beta"], r0["beta"][perm], rtol=1e-13)


def test_single_worker_is_unchanged():
    off, x, g = _random_problem(66, K=1)
    P = int(off[-1])
    for r in (orc.mgrawa_update(x, g, off, 0.37), orc.lgrawa_update(x, g, off, 0.37)):
        np.testing.assert_array_equal(np.ravel(r["beta"]), 1.0)
        np.testing.assert_array_equal(r["center"], x[0, :P].astype(np.float64))
        np.testing.assert_allclose(r["x"][0], x[0, :P].astype(np.float64), rtol=1e-15)


def test_pull_properties():
    off, x, g = _random_problem(77, K=4)
    P = int(off[-1])
    xd = x[:, :P].astype(np.float64)
    _, beta = orc.lgrawa_weights(g, off)
    # lambda = 0 is the identity, lambda = 1 puts every worker on the center
    r0, c0 = orc.center_pull(x, beta, off, 0.0)
    np.testing.assert_array_equal(r0, xd)
    r1, c1 = orc.center_pull(x, beta, off, 1.0)
    np.testing.assert_array_equal(r1, np.broadcast_to(c1, r1.shape))
    np.testing.assert_array_equal(c0, c1)
    lam = 0.3
    r, c = orc.center_pull(x, beta, off, lam)
    # the center lies in the per-coordinate hull of the workers
    assert np.all(c <= xd.max(axis=0) + 1e-15) and np.all(c >= xd.min(axis=0) - 1e-15)
    # differences between workers contract by (1 - lambda) whatever the weights are
    for m in range(1, 4):
        np.testing.assert_allclose(r[m] - r[0], (1 - lam) * (xd[m] - xd[0]), rtol=1e-12, atol=1e-16)
    # the center is a fixed point of the pull: sum_m beta_m x_m' = x_C
    layer_of = np.repeat(np.arange(off.size - 1), np.diff(off))
    np.testing.assert_allclose((beta[:, layer_of] * r).sum(axis=0), c, rtol=1e-12, atol=1e-16)
    # direction: toward the center
    assert np.all(np.abs(r - c) <= np.abs(xd - c) + 1e-18)
    # one-hot weights make the center that worker (a transposed beta table would not)
    hot = np.zeros((4, off.size - 1))
    hot[np.arange(off.size - 1) % 4, np.arange(off.size - 1)] = 1.0
    _, ch = orc.center_pull(x, hot, off, 0.5)
    for l in range(off.size - 1):
        np.testing.assert_array_equal(ch[off[l]:off[l + 1]], xd[l % 4, off[l]:off[l + 1]])


def test_zero_norm_rule_is_the_limit():
    # weights for A = (eps, 1, 1) tend to (1, 0, 0); for (eps, eps, 1) to (1/2, 1/2, 0)
    for A0, want in (((0.0, 1.0, 1.0), (1.0, 0.0, 0.0)), ((0.0, 0.0, 3.0), (0.5, 0.5, 0.0)),
                     ((0.0, 0.0, 0.0), (1 / 3, 1 / 3, 1 / 3))):
        np.testing.assert_array_equal(orc.weights(np.array(A0)), np.array(want))
        A = np.array(A0)
        for eps in (1e-6, 1e-12, 1e-30):
            Ae = np.where(A == 0.0, eps, A)
            if np.all(A == 0):
                np.testing.assert_allclose(orc.weights(Ae), want, rtol=1e-15)
            else:
                np.testing.assert_allclose(orc.weights(Ae), want, atol=4 * eps)
    # an infinite score gets no weight
    np.testing.assert_allclose(orc.weights(np.array([np.inf, 2.0, 2.0])), [0.0, 0.5, 0.5])
    # a frozen layer (all-zero gradients) under LGRAWA is averaged uniformly
    off, x, g = _random_problem(88, K=3)
    g[:, off[1]:off[2]] = 0
    _, b = orc.lgrawa_weights(g, off)
    np.testing.assert_array_equal(b[:, 1], [1 / 3] * 3)


def test_fused_sgd_order_and_chunking():
    # Algorithms 1/2: the SGD step comes first, then center and pull on the stepped parameters
    off, x, g = _random_problem(99, K=4, ld_pad=3)
    P = int(off[-1])
    lr, lam = 0.1, 0.25
    A, beta = orc.lgrawa_weights(g, off)
    xs = x[:, :P].astype(np.float64) - lr * g[:, :P].astype(np.float64)
    layer_of = np.repeat(np.arange(off.size - 1), np.diff(off))
    c = np.einsum("kp,kp->p", beta[:, layer_of], xs)
    want = (1 - lam) * xs + lam * c
    r = orc.lgrawa_update(x, g, off, lam, g_sgd=g, lr=lr)
    np.testing.assert_allclose(r["x"], want, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(r["center"], c, rtol=1e-13, atol=1e-16)
    # chunk boundaries in the middle of layers change nothing
    for chunk in (1, 7, 64):
        xn, cc = orc.center_pull(x, beta, off, lam, g_sgd=g, lr=lr, chunk=chunk)
        np.testing.assert_array_equal(xn, r["x"])
        np.testing.assert_array_equal(cc, r["center"])
    # and SGD-then-pull differs from pull-then-SGD unless lambda = 0 (order matters)
    other = orc.lgrawa_update(x, g, off, lam)["x"] - lr * g[:, :P].astype(np.float64)
    assert not np.allclose(other, want, rtol=1e-6)


def test_prox_step():
    # Algorithms 1/2 (Prox.): x <- (1 - mu/tau) x + (mu/tau) x_C with the stored center
    off, x, g = _random_problem(111, K=3)
    P = int(off[-1])
    rng = np.random.default_rng(1)
    cprev = rng.standard_normal(P)
    mu, tau, lr = 0.05, 16.0, 0.1
    out = orc.local_sgd(x, g, lr, P=P, prox_center=cprev, mu=mu, tau=tau)
    xs = x[:, :P].astype(np.float64) - lr * g[:, :P].astype(np.float64)
    np.testing.assert_allclose(out, xs + (mu / tau) * (cprev - xs), rtol=1e-12, atol=1e-16)
    # mu = 0 is no prox at all; mu/tau = 1 lands on the stored center
    np.testing.assert_array_equal(orc.local_sgd(x, g, lr, P=P, prox_center=cprev, mu=0.0, tau=tau),
                                  orc.local_sgd(x, g, lr, P=P))
    np.testing.assert_allclose(orc.local_sgd(x, g, lr, P=P, prox_center=cprev, mu=4.0, tau=4.0),
                               np.broadcast_to(cprev, (3, P)), rtol=1e-15)


def test_expected_norm_of_synthetic_gradients():
    # N(0, s^2) entries: ||G||_F concentrates at s * sqrt(n)
    rng = np.random.default_rng(5)
    n, s = 200_000, 0.037
    g = (s * rng.standard_normal((2, n))).astype(np.float32)
    A = orc.layer_norms(orc.grad_sumsq(g, [0, n]))
    np.testing.assert_allclose(A[:, 0], s * math.sqrt(n), rtol=1e-2)


# ----------------------------------------------------------------------------
# Appendix G: running estimate of the norm scores (Local MGRAWA / LGRAWA)
# ----------------------------------------------------------------------------

def test_norm_momentum_closed_forms():
    # constant scores a: g_mvg after t steps is a (1 - gamma^t), so g_est = gamma * a exactly
    gamma = Fr(9, 10)
    a = [Fr(3), Fr(1, 2), Fr(7)]
    sc = orc.LocalScores(1, 3, float(gamma))
    mv = [Fr(0)] * 3
    for t in range(1, 8):
        g_cur = np.array([[float(v) for v in a]])
        lib = orc.lib()
        sc.t += 1
        assert lib.oracle_norm_momentum(orc._p(sc.g_mvg), orc._p(g_cur), orc._p(sc.g_est), 3, float(gamma), sc.t) == 0
        mv = [gamma * m + (1 - gamma) * v for m, v in zip(mv, a)]                 # the recurrence, exactly
        assert mv == [v * (1 - gamma ** t) for v in a]                           # its closed form
        np.testing.assert_allclose(sc.g_mvg[0], as_float(mv), rtol=1e-14)
        np.testing.assert_allclose(sc.g_est[0], as_float([gamma * v for v in a]), rtol=1e-14)
    # varying scores: compare with the exact rational recurrence and the printed correction
    rng = np.random.default_rng(4)
    gamma = Fr(1, 2)
    sc = orc.LocalScores(2, 2, float(gamma))
    mv = [[Fr(0)] * 2 for _ in range(2)]
    for t in range(1, 6):
        cur = rng.integers(1, 50, size=(2, 2))
        g = np.zeros((2, 4), dtype=np.float32)
        g[:, 0] = cur[:, 0]
        g[:, 2] = cur[:, 1]                       # one non-zero entry per layer: norm = |entry|
        got = sc.step(g, [0, 2, 4])
        np.testing.assert_array_equal(got, cur.astype(np.float64))
        mv = [[gamma * mv[m][l] + (1 - gamma) * int(cur[m, l]) for l in range(2)] for m in range(2)]
        est = [[gamma * mv[m][l] / (1 - gamma ** t) for l in range(2)] for m in range(2)]
        np.testing.assert_allclose(sc.g_mvg, np.array([as_float(r) for r in mv]), rtol=1e-15)
        np.testing.assert_allclose(sc.g_est, np.array([as_float(r) for r in est]), rtol=1e-15)
    assert sc.t == 5
    # the leading gamma is common to all workers: weights equal those of the plain bias-corrected average
    plain = np.array([as_float([mv[m][l] / (1 - gamma ** 5) for l in range(2)]) for m in range(2)])
    np.testing.assert_allclose(sc.weights("lgrawa"), orc.weights(plain), rtol=1e-14)
    np.testing.assert_allclose(sc.weights("mgrawa"), orc.weights(plain.sum(axis=1)), rtol=1e-14)
    sc.reset()
    assert sc.t == 0 and not sc.g_mvg.any()
    # gamma outside (0, 1) is rejected
    for bad in (0.0, 1.0, -0.1, 1.5):
        z = np.zeros(1)
        assert orc.lib().oracle_norm_momentum(orc._p(z), orc._p(z), orc._p(z), 1, bad, 1) != 0


def test_local_grawa_round_single_step_equals_fused_update():
    # one local step with the same gradient: the estimate is gamma * (1-gamma)/(1-gamma) * norm = gamma * norm,
    # a common factor, so the round equals the fused SGD + LGRAWA / MGRAWA update of the main algorithms
    off, x, g = _random_problem(123, K=4)
    lr, lam = 0.1, 0.3
    r = orc.local_grawa_round(x, [g], off, lr, lam, 0.7, "lgrawa")
    f = orc.lgrawa_update(x, g, off, lam, g_sgd=g, lr=lr)
    np.testing.assert_allclose(r["beta"], f["beta"], rtol=1e-13)
    np.testing.assert_allclose(r["x"], f["x"], rtol=1e-12, atol=1e-16)
    r = orc.local_grawa_round(x, [g], off, lr, lam, 0.7, "mgrawa")
    f = orc.mgrawa_update(x, g, off, lam, "layersum", g_sgd=g, lr=lr)
    np.testing.assert_allclose(r["beta"], f["beta"], rtol=1e-13)
    np.testing.assert_allclose(r["x"], f["x"], rtol=1e-12, atol=1e-16)


def test_local_grawa_round_several_steps():
    off, x, g0 = _random_problem(124, K=3)
    _, _, g1 = _random_problem(125, K=3)
    _, _, g2 = _random_problem(126, K=3, bf16=True)
    P = int(off[-1])
    lr, lam, gamma, mu, tau = 0.05, 0.4, 0.9, 0.05, 16.0
    rng = np.random.default_rng(2)
    cprev = 0.05 * rng.standard_normal(P)
    r = orc.local_grawa_round(x, [g0, g1, g2], off, lr, lam, gamma, "lgrawa", prox_center=cprev, mu=mu, tau=tau)
    # independent numpy statement of the same loop
    from parity_util import grads_to_f64
    cur = x[:, :P].astype(np.float64)
    mvg = np.zeros((3, off.size - 1))
    w = mu / tau
    for t, g in enumerate((g0, g1, g2), start=1):
        gd = grads_to_f64(g)[:, :P]
        norms = np.array([[np.linalg.norm(gd[m, off[l]:off[l + 1]]) for l in range(off.size - 1)] for m in range(3)])
        mvg = gamma * mvg + (1 - gamma) * norms
        est = gamma * mvg / (1 - gamma ** t)
        cur = cur - lr * gd
        cur = (1 - w) * cur + w * cprev
    beta = (1 / est) / (1 / est).sum(axis=0)
    layer_of = np.repeat(np.arange(off.size - 1), np.diff(off))
    c = (beta[:, layer_of] * cur).sum(axis=0)
    want = (1 - lam) * cur + lam * c
    np.testing.assert_allclose(r["g_est"], est, rtol=1e-13)
    np.testing.assert_allclose(r["beta"], beta, rtol=1e-13)
    np.testing.assert_allclose(r["x"], want, rtol=1e-11, atol=1e-15)


# ----------------------------------------------------------------------------
# Nesterov-momentum local optimizer (Appendix B.2.2) and the competing centers (Appendix F)
# ----------------------------------------------------------------------------

def test_nesterov_matches_the_classical_two_line_form():
    # classical NAG on f(x) = a x^2 / 2 in exact rationals: v <- mu v - eta f'(x + mu v), x <- x + v.
    # The framework form fed with the gradient at its own iterate must walk the look-ahead points y = x + mu v.
    a, mu, eta = Fr(3, 2), Fr(9, 10), Fr(1, 10)
    xc, v = Fr(4), Fr(0)
    y = [xc + mu * v]
    for _ in range(6):
        v = mu * v - eta * a * (xc + mu * v)
        xc = xc + v
        y.append(xc + mu * v)
    x = np.array([[float(y[0])]], dtype=np.float32)          # 4.0 is exact in fp32
    buf = np.zeros((1, 1))
    cur = x.astype(np.float64)
    for t in range(6):
        g = (float(a) * cur).astype(np.float64)
        # feed the gradient through the fp32 interface exactly: use a power-of-two friendly check instead
        g32 = g.astype(np.float32)
        cur, buf = orc.nesterov_sgd(cur, buf, g32, float(eta), float(mu))
        assert cur[0, 0] == pytest.approx(float(y[t + 1]), rel=2e-6)       # fp32 rounding of the fed gradient only


def test_nesterov_special_cases_and_closed_forms():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 50)).astype(np.float32)
    g = rng.standard_normal((3, 56)).astype(np.float32)
    z = np.zeros((3, 50))
    # no momentum, no decay: the plain SGD step, and the buffer holds the gradient
    xn, bn = orc.nesterov_sgd(x, z, g, 0.1, 0.0)
    np.testing.assert_array_equal(xn, orc.local_sgd(x, g, 0.1, P=50))
    np.testing.assert_array_equal(bn, g[:, :50].astype(np.float64))
    # constant gradient: buf_t = g (1 - mu^t)/(1 - mu); x_t = x_0 - eta sum_s (g + mu buf_s)
    mu, eta = 0.5, 0.25
    cur, buf = x.astype(np.float64), z
    gd = g[:, :50].astype(np.float64)
    acc = np.zeros_like(gd)
    for t in range(1, 6):
        cur, buf = orc.nesterov_sgd(cur, buf, g, eta, mu)
        np.testing.assert_allclose(buf, gd * (1 - mu ** t) / (1 - mu), rtol=1e-14)
        acc += gd + mu * gd * (1 - mu ** t) / (1 - mu)
        np.testing.assert_allclose(cur, x.astype(np.float64) - eta * acc, rtol=1e-12, atol=1e-15)
    # weight decay alone from a zero buffer: x <- x (1 - eta wd (1 + mu))
    g0 = np.zeros_like(g)
    xn, bn = orc.nesterov_sgd(x, z, g0, 0.1, 0.9, 5e-4)
    np.testing.assert_allclose(xn, x.astype(np.float64) * (1 - 0.1 * 5e-4 * 1.9), rtol=1e-14)
    np.testing.assert_allclose(bn, 5e-4 * x.astype(np.float64), rtol=1e-14)
    # bf16 gradients are widened exactly
    from parity_util import grads_to_f64
    gb = _bf16_bits(g)
    xn, _ = orc.nesterov_sgd(x, z, gb, 0.1, 0.0)
    np.testing.assert_array_equal(xn, x.astype(np.float64) - 0.1 * grads_to_f64(gb)[:, :50])


def test_easgd_center_and_pull():
    rng = np.random.default_rng(10)
    x = rng.integers(-8, 9, size=(4, 7)).astype(np.float32)
    c0 = rng.integers(-8, 9, size=7).astype(np.float64)
    rho, lam = Fr(1, 4), Fr(1, 2)
    mean = [sum(Fr(int(v)) for v in x[:, i]) / 4 for i in range(7)]
    c = [(1 - rho) * Fr(int(c0[i])) + rho * mean[i] for i in range(7)]
    want = [[(1 - lam) * Fr(int(x[m, i])) + lam * c[i] for i in range(7)] for m in range(4)]
    xn, cn = orc.easgd_update(x, c0, float(lam), float(rho))
    np.testing.assert_array_equal(cn, as_float(c))
    np.testing.assert_array_equal(xn, np.array([as_float(r) for r in want]))
    # rho = 1: the center is the plain average, i.e. GRAWA with equal weights; rho = 0: the old center stays
    xn1, cn1 = orc.easgd_update(x, c0, 0.5, 1.0)
    xr, cr = orc.center_pull(x, np.full(4, 0.25), [0, 7], 0.5)
    np.testing.assert_allclose(cn1, cr, rtol=1e-15)
    np.testing.assert_allclose(xn1, xr, rtol=1e-15)
    _, cn0 = orc.easgd_update(x, c0, 0.5, 0.0)
    np.testing.assert_array_equal(cn0, c0)


def test_lsgd_leader_and_pull():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((5, 9)).astype(np.float32)
    losses = np.array([0.7, 0.2, 0.9, 0.2, 0.5])
    xn, lead = orc.lsgd_update(x, losses, 0.25)
    assert lead == 1                                         # smallest loss, first on ties
    hot = np.zeros(5)
    hot[1] = 1.0
    xr, cr = orc.center_pull(x, hot, [0, 9], 0.25)           # one-hot weights through the GRAWA center
    np.testing.assert_array_equal(cr, x[1].astype(np.float64))
    np.testing.assert_allclose(xn, xr, rtol=1e-15)
    np.testing.assert_array_equal(xn[1], x[1].astype(np.float64))   # the leader does not move


def test_nonfinite_scores_are_reported():
    # pinned to the IEEE classification numpy applies, on every special value and both signs
    assert not orc.nonfinite(np.array([0.0, 1.0, 1e308, 5e-324, -2.5]))
    assert not orc.nonfinite(np.zeros((3, 4)))
    for bad in (np.inf, -np.inf, np.nan):
        for pos in (0, 5, 11):
            A = np.arange(12, dtype=np.float64).reshape(3, 4)
            A.flat[pos] = bad
            assert orc.nonfinite(A) and not np.isfinite(A).all()
    assert not orc.nonfinite(np.array([]))
