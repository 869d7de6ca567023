"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved).

1. The float64 CPU checker: its C source is compiled, with the sanitizers, into a small driver
   (tests/oracle_sanitizer_driver.c) that calls every checker function on exactly-sized heap buffers;
   the results must equal, bit for bit, those of the ordinary build called through ctypes, on ragged
   layer lists, L = P (every layer one element), K = 1, bf16 gradients, column windows that start and
   end inside layers, and the two worked examples of tests/golden/.
2. The plan's index maps (paper_2403_04206_amd/csrc/grawa_maps.cpp, which has no GPU dependency): built by
   tests/maps_sanitizer_driver.cpp, which also verifies the invariants the kernels rely on, for ragged
   offsets, L = P, a row of 2^31 + 5 columns and offsets the library must refuse.
"""
import ctypes as C
import json
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import grawa_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")

pytestmark = pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="no host compiler")


def compile_(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return cmd[cmd.index("-o") + 1]


@pytest.fixture(scope="module")
def oracle_driver(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "oracle_driver")
    return compile_(["gcc", "-std=c11", "-Wall", "-Wextra", "-fno-fast-math", "-ffp-contract=off"] + SAN +
                    [os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"), os.path.join(ROOT, "oracle", "grawa_oracle.c"),
                     "-o", out, "-lm"])


@pytest.fixture(scope="module")
def maps_driver(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "maps_driver")
    csrc = os.path.join(ROOT, "paper_2403_04206_amd", "csrc")
    return compile_(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN + ["-I", csrc,
                    os.path.join(ROOT, "tests", "maps_sanitizer_driver.cpp"), os.path.join(csrc, "grawa_maps.cpp"), "-o", out])


def p(a):
    return a.ctypes.data_as(C.c_void_p)


def through_ctypes(K, L, off, x, g, dt, loss, cprev, i0, i1, s):
    """The driver's call sequence on the ordinary build of the checker."""
    Lb = orc.lib()
    lam, eta, mu, tau, gamma, mom, wd, rho = s
    n = i1 - i0
    ldx, ldg = x.shape[1], g.shape[1]
    out = []
    S = np.empty((K, L)); A = np.empty((K, L)); Am = np.empty(K); Af = np.empty(K); bl = np.empty((K, L)); bm = np.empty(K)
    assert Lb.oracle_sumsq(p(g), dt, K, ldg, L, p(off), p(S)) == 0
    assert Lb.oracle_layer_norms(p(S), K, L, p(A)) == 0
    assert Lb.oracle_model_norms(p(S), K, L, 0, p(Am)) == 0
    assert Lb.oracle_model_norms(p(S), K, L, 1, p(Af)) == 0
    assert Lb.oracle_weights(p(A), K, L, p(bl)) == 0
    assert Lb.oracle_weights(p(Am), K, 1, p(bm)) == 0
    out += [S, A, Am, Af, bl, bm]
    xd = np.empty((K, n)); c = np.empty(n)
    assert Lb.oracle_load_params(p(x), K, ldx, i0, i1, p(xd)) == 0
    assert Lb.oracle_local_sgd(p(xd), K, n, i0, p(g), dt, ldg, eta) == 0
    assert Lb.oracle_prox(p(xd), K, n, p(cprev), mu, tau) == 0
    assert Lb.oracle_center(p(xd), K, n, i0, p(bl), L, p(off), p(c)) == 0
    assert Lb.oracle_pull(p(xd), K, n, p(c), lam) == 0
    out += [xd.copy(), c.copy()]
    assert Lb.oracle_load_params(p(x), K, ldx, i0, i1, p(xd)) == 0
    assert Lb.oracle_center(p(xd), K, n, i0, p(bm), 1, None, p(c)) == 0
    assert Lb.oracle_pull(p(xd), K, n, p(c), lam) == 0
    out += [xd.copy(), c.copy()]
    mvg = np.zeros((K, L)); est = np.empty((K, L)); sl = np.empty(K)
    assert Lb.oracle_norm_momentum(p(mvg), p(A), p(est), K * L, gamma, 1) == 0
    assert Lb.oracle_norm_momentum(p(mvg), p(A), p(est), K * L, gamma, 2) == 0
    assert Lb.oracle_sum_layers(p(est), K, L, p(sl)) == 0
    out += [mvg, est, sl]
    buf = np.zeros((K, n))
    assert Lb.oracle_load_params(p(x), K, ldx, i0, i1, p(xd)) == 0
    for _ in range(2):
        assert Lb.oracle_nesterov_sgd(p(xd), p(buf), K, n, i0, p(g), dt, ldg, eta, mom, wd) == 0
    out += [xd.copy(), buf]
    assert Lb.oracle_load_params(p(x), K, ldx, i0, i1, p(xd)) == 0
    c2 = cprev.copy()
    assert Lb.oracle_easgd_center(p(xd), K, n, p(c2), rho) == 0
    out += [c2, np.array([float(Lb.oracle_leader(p(loss), K))])]
    return np.concatenate([np.ravel(a) for a in out])


CASES = [
    # K, layer sizes, dtype, ld padding, window (None = whole row)
    (3, [5, 1, 33, 8, 130], "f32", 0, None),
    (4, [1] * 37, "f32", 3, None),                      # L = P: every layer is one element
    (1, [17], "bf16", 0, None),                         # one worker, one layer
    (5, [7, 300, 2, 1, 64, 1000], "bf16", 9, (5, 1201)),  # a window that starts and ends inside layers
    (2, [4096, 4097, 1], "f32", 0, (4095, 8194)),
    (6, [3, 3, 3], "f32", 1, (8, 9)),                   # a single column, the last one
]


@pytest.mark.parametrize("K,sizes,dtype,pad,window", CASES)
def test_checker_under_sanitizers(oracle_driver, tmp_path, K, sizes, dtype, pad, window):
    rng = np.random.default_rng([K, len(sizes), pad])
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P, L = int(off[-1]), len(sizes)
    i0, i1 = window or (0, P)
    x = rng.normal(0, 0.05, size=(K, P + pad)).astype(np.float32)
    gf = (rng.normal(size=(K, P + pad)) * 10.0 ** rng.uniform(-3, 1, size=(K, 1))).astype(np.float32)
    if dtype == "bf16":
        g = (gf.view(np.uint32) >> 16).astype(np.uint16)
        dt = 1
    else:
        g, dt = gf, 0
    loss = rng.uniform(size=K)
    cprev = rng.normal(0, 0.05, size=i1 - i0)
    s = np.array([0.3, 0.1, 0.05, 16.0, 0.9, 0.9, 5e-4, 0.25])
    want = through_ctypes(K, L, off, x, g, dt, loss, cprev, i0, i1, s)
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(np.array([K, L, x.shape[1], g.shape[1], dt, i0, i1], dtype=np.int64).tobytes())
        f.write(s.tobytes())
        for a in (off, x, g, loss, cprev):
            f.write(np.ascontiguousarray(a).tobytes())
    res = subprocess.run([oracle_driver, str(src), str(dst)], capture_output=True, text=True, env=ENV, timeout=120)
    assert res.returncode == 0, "sanitizer report or failure:\n" + res.stderr[-4000:]
    assert res.stderr.strip() == "", res.stderr[-4000:]
    got = np.fromfile(dst, dtype=np.float64)
    assert got.shape == want.shape
    np.testing.assert_array_equal(got, want)


def frac(v):
    from fractions import Fraction
    return float(Fraction(v))


@pytest.mark.parametrize("name", ["ex1_two_workers.json", "ex2_three_workers_two_layers.json"])
def test_worked_examples_under_sanitizers(oracle_driver, tmp_path, name):
    # the hand-worked fixtures: the sanitized build reproduces the stored weights and centers
    ex = json.load(open(os.path.join(ROOT, "tests", "golden", name)))
    x = np.asarray(ex["x"], dtype=np.float32)
    g = np.asarray(ex["g"], dtype=np.float32)
    off = np.asarray(ex["offsets"], dtype=np.int64)
    K, P, L = x.shape[0], x.shape[1], off.size - 1
    s = np.array([frac(ex["lambda"]), 0.0, 0.0, 1.0, 0.5, 0.0, 0.0, 0.5])
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(np.array([K, L, P, P, 0, 0, P], dtype=np.int64).tobytes())
        f.write(s.tobytes())
        for a in (off, x, g, np.zeros(K), np.zeros(P)):
            f.write(np.ascontiguousarray(a).tobytes())
    res = subprocess.run([oracle_driver, str(src), str(dst)], capture_output=True, text=True, env=ENV, timeout=120)
    assert res.returncode == 0 and res.stderr.strip() == "", res.stderr[-4000:]
    got = np.fromfile(dst, dtype=np.float64)
    want = through_ctypes(K, L, off, x, g, 0, np.zeros(K), np.zeros(P), 0, P, s)
    np.testing.assert_array_equal(got, want)
    # layout of the output: S, A [K,L] ; Am, Af [K] ; beta_layer [K,L] ; beta_model [K] ; x, c (per layer) ; x, c (model)
    at = 2 * K * L + 2 * K
    beta_layer = got[at:at + K * L].reshape(K, L)
    beta_model = got[at + K * L:at + K * L + K]
    at += K * L + K
    c_layer = got[at + K * P:at + K * P + P]
    c_model = got[at + 2 * K * P + P:at + 2 * K * P + 2 * P]
    if "beta" in ex:                        # one layer: both weightings coincide
        stored = np.array([frac(v) for v in ex["beta"]])
        np.testing.assert_allclose(beta_model, stored, rtol=1e-15)
        np.testing.assert_allclose(beta_layer[:, 0], stored, rtol=1e-15)
        np.testing.assert_allclose(c_model, [frac(v) for v in ex["center"]], rtol=1e-15)
    else:
        np.testing.assert_allclose(beta_model, [frac(v) for v in ex["mgrawa"]["beta"]], rtol=1e-15)
        np.testing.assert_allclose(beta_layer, [[frac(v) for v in r] for r in ex["lgrawa"]["beta"]], rtol=1e-15)
        np.testing.assert_allclose(c_model, [frac(v) for v in ex["mgrawa"]["center"]], rtol=1e-15)
        np.testing.assert_allclose(c_layer, [frac(v) for v in ex["lgrawa"]["center"]], rtol=1e-15)


def run_maps(maps_driver, tmp_path, P, off, T=0, K=4):
    src = tmp_path / "maps.bin"
    off = np.asarray(off, dtype=np.int64)
    with open(src, "wb") as f:
        f.write(np.array([P, off.size - 1, T, K], dtype=np.int64).tobytes())
        f.write(off.tobytes())
    return subprocess.run([maps_driver, str(src)], capture_output=True, text=True, env=ENV, timeout=300)


@pytest.mark.parametrize("sizes,T,K", [
    ([1, 3, 8193, 2, 5, 8191, 20000, 7, 1, 1, 4096, 33, 16385, 6], 0, 4),      # ragged, unaligned everywhere
    ([1] * 3000, 2048, 2),                                                      # L = P
    ([2048] * 40, 2048, 8),                                                     # every boundary on a tile boundary
    ([255, 1, 256, 257, 1023, 1, 1024, 1025], 4096, 16),                        # around the cell and short-tile lengths
    ([16384, 16385, 16383], 16384, 32),
    ([2 ** 31 - 3, 8, 2 ** 20], 16384, 2),                                      # P = 2^31 + 2^20 + 5, a boundary near 2^31
    ([2 ** 31 + 5], 0, 1),                                                      # one layer of 2^31 + 5 columns
])
def test_index_maps_under_sanitizers(maps_driver, tmp_path, sizes, T, K):
    off = np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))])
    res = run_maps(maps_driver, tmp_path, int(off[-1]), off, T, K)
    assert res.returncode == 0, res.stdout + res.stderr[-4000:]
    assert res.stdout.startswith("ok") and res.stderr.strip() == ""


@pytest.mark.parametrize("P,off", [(10, [0, 5, 9]), (10, [1, 5, 10]), (10, [0, 5, 5, 10]), (10, [0, 7, 5, 10]),
                                   (3, [0, 1, 2, 3, 3])])
def test_index_maps_refuse_bad_offsets(maps_driver, tmp_path, P, off):
    res = run_maps(maps_driver, tmp_path, P, off)
    assert res.returncode == 3 and "invalid offsets" in res.stdout and res.stderr.strip() == ""
