"""The library called from a plain C99 program (tests/c_abi_client.c): no Python, no torch on the
calling side.  The program's printed weights and parameters are compared with the CPU reference run
on the same inputs, which are regenerated here from the program's 32-bit linear congruential generator."""
import os
import subprocess

import numpy as np
import pytest

from oracle import grawa_oracle as orc
from paper_2403_04206_amd import buildlib
from parity_util import TIGHT, assert_params_close, assert_table_close, operand_scale

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "paper_2403_04206_amd", "_build", "c_abi_client")
K, SIZES = 3, [5, 300, 1, 1000]


def lcg_inputs():
    P = sum(SIZES)
    ld = (P + 7) // 8 * 8
    state = 12345
    x = np.empty((K, ld), dtype=np.float32)
    g = np.empty((K, ld), dtype=np.float32)
    for k in range(K):
        for i in range(ld):
            state = (1664525 * state + 1013904223) & 0xFFFFFFFF
            x[k, i] = np.float32(((state >> 8) & 0xFFFF) / 65536.0) - np.float32(0.5)
            state = (1664525 * state + 1013904223) & 0xFFFFFFFF
            g[k, i] = (np.float32(((state >> 8) & 0xFFFF) / 65536.0) - np.float32(0.5)) * np.float32(1 << (2 * k))
    return P, ld, x, g


def test_c_program_matches_the_reference():
    if not os.path.exists(CLIENT):
        buildlib.build_c_client(os.path.join(ROOT, "tests", "c_abi_client.c"), CLIENT)
    print("[case] C client %s" % CLIENT, flush=True)
    res = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    lines = res.stdout.split("\n")
    P, ld, x, g = lcg_inputs()
    assert lines[0] == "P %d ld %d" % (P, ld)
    vals = {"beta_layer": [], "beta_model": [], "x": [], "static_equal": [], "nonfinite": []}
    for ln in lines[1:]:
        if ln:
            name, v = ln.split()
            vals[name].append(float(v))
    assert vals["static_equal"] == [1.0], "the allocation-free call differs from the plan-based one"
    assert vals["nonfinite"] == [0.0]
    off = np.concatenate([[0], np.cumsum(SIZES)])
    # the same three calls through the reference, the state rounded to fp32 between calls as it is stored
    x1 = orc.local_sgd(x, g, 0.125, P=P).astype(np.float32)
    xa = x.copy()
    xa[:, :P] = x1
    r1 = orc.lgrawa_update(xa, g, off, 0.25)
    xb = x.copy()
    xb[:, :P] = r1["x"].astype(np.float32)
    r2 = orc.mgrawa_update(xb, g, off, 0.5, g_sgd=g, lr=0.0625)
    assert_table_close(np.array(vals["beta_layer"]).reshape(K, len(SIZES)), r1["beta"], TIGHT, "per-layer weights")
    assert_table_close(np.array(vals["beta_model"]), r2["beta"], TIGHT, "model-level weights")
    got = np.array(vals["x"]).reshape(K, ld)
    sc = operand_scale(x[:, :P], g[:, :P], 0.125 + 0.0625)
    assert_params_close(got[:, :P], r2["x"], off, 3 * TIGHT, "x after three calls", sc)
    np.testing.assert_array_equal(got[:, P:].astype(np.float32), x[:, P:])      # padding untouched
