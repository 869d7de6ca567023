"""Host-only checks of the C ABI: the library loads, exports every function the public
header declares, and rejects bad arguments before touching the device.  No kernel is
launched here, so these run without a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2403_04206_amd import buildlib, grawa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "grawa.h")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(grawa.LIB_PATH):
        buildlib.build(force=True)
    return grawa.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(grawa_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert len(names) >= 14
    for required in ("grawa_mgrawa_update", "grawa_lgrawa_update", "grawa_local_sgd", "grawa_center_pull",
                     "grawa_grad_norms", "grawa_plan_create", "grawa_plan_destroy", "grawa_mgrawa_update_sgd",
                     "grawa_lgrawa_update_sgd", "grawa_status_string"):
        assert required in names
    for n in names:
        assert hasattr(L, n), "libgrawa.so does not export %s" % n


def test_status_strings(L):
    seen = set()
    for code in range(6):
        s = grawa.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 6
    assert grawa.status_string(99) == "unknown status"


def _create(L, K, P, Ln, off):
    h = C.c_void_p()
    offp = None if off is None else np.ascontiguousarray(off, dtype=np.int64).ctypes.data_as(C.c_void_p)
    st = L.grawa_plan_create(C.byref(h), K, P, Ln, offp)
    return st, h


@pytest.mark.parametrize("K,P,Ln,off", [
    (0, 10, 1, None),                 # no workers
    (2, 0, 1, None),                  # no parameters
    (2, 10, 0, None),                 # no layers
    (2, 10, 2, None),                 # offsets required when L > 1
    (2, 10, 2, [0, 5, 9]),            # last offset is not P
    (2, 10, 2, [1, 5, 10]),           # first offset is not 0
    (2, 10, 3, [0, 5, 5, 10]),        # empty layer
    (2, 10, 3, [0, 7, 5, 10]),        # not increasing
    (2, 3, 4, [0, 1, 2, 3, 3]),       # more layers than parameters
])
def test_plan_create_rejects_bad_shapes(L, K, P, Ln, off):
    st, h = _create(L, K, P, Ln, off)
    assert st == grawa.ERR_INVALID_ARG
    assert not h.value


def test_plan_create_limits(L):
    st, h = _create(L, grawa.MAX_WORKERS + 1, 10, 1, None)
    assert st == grawa.ERR_UNSUPPORTED and not h.value
    assert L.grawa_plan_create(None, 2, 10, 1, None) == grawa.ERR_INVALID_ARG


def test_null_plan_and_null_buffers_are_rejected(L):
    z = C.c_void_p(0)
    assert L.grawa_plan_destroy(z) == grawa.OK
    assert L.grawa_grad_norms(z, z, 16, 0, z, z) == grawa.ERR_INVALID_ARG
    assert L.grawa_mgrawa_update(z, z, 16, z, 16, 0, 0, 0.1, z, z, z) == grawa.ERR_INVALID_ARG
    assert L.grawa_lgrawa_update(z, z, 16, z, 16, 0, 0.1, z, z, z) == grawa.ERR_INVALID_ARG
    assert L.grawa_center_pull(z, z, 16, z, 0, 0.1, z, z) == grawa.ERR_INVALID_ARG
    assert L.grawa_plan_profile(z, 1) == grawa.ERR_INVALID_ARG
    assert L.grawa_plan_info(z, None, None) == grawa.ERR_INVALID_ARG
    assert L.grawa_plan_nonfinite(z, C.byref(C.c_uint()), 0, z) == grawa.ERR_INVALID_ARG


def test_local_sgd_argument_checks(L):
    z = C.c_void_p(0)
    a = C.c_void_p(0x1000)       # never dereferenced: every call below must fail validation first
    odd = C.c_void_p(0x1004)
    f = L.grawa_local_sgd
    assert f(z, 16, a, 16, 0, 2, 16, 0.1, z) == grawa.ERR_INVALID_ARG      # x NULL
    assert f(a, 16, z, 16, 0, 2, 16, 0.1, z) == grawa.ERR_INVALID_ARG      # g NULL
    assert f(a, 16, a, 16, 0, 0, 16, 0.1, z) == grawa.ERR_INVALID_ARG      # K < 1
    assert f(a, 16, a, 16, 0, 2, 0, 0.1, z) == grawa.ERR_INVALID_ARG       # P < 1
    assert f(a, 8, a, 16, 0, 2, 16, 0.1, z) == grawa.ERR_INVALID_ARG       # ldx < P
    assert f(a, 16, a, 8, 0, 2, 16, 0.1, z) == grawa.ERR_INVALID_ARG       # ldg < P
    assert f(odd, 16, a, 16, 0, 2, 16, 0.1, z) == grawa.ERR_ALIGNMENT      # x misaligned
    assert f(a, 16, odd, 16, 0, 2, 16, 0.1, z) == grawa.ERR_ALIGNMENT      # g misaligned
    assert f(a, 18, a, 16, 0, 2, 16, 0.1, z) == grawa.ERR_ALIGNMENT        # ldx*4 not a multiple of 16
    assert f(a, 16, a, 20, 1, 2, 16, 0.1, z) == grawa.ERR_ALIGNMENT        # bf16 ldg*2 not a multiple of 16
    assert f(a, 16, a, 16, 7, 2, 16, 0.1, z) == grawa.ERR_UNSUPPORTED      # unknown dtype
    assert f(a, 16, a, 16, 0, 2, 16, float("nan"), z) == grawa.ERR_INVALID_ARG
    assert f(a, 16, a, 16, 0, 65536, 16, 0.1, z) == grawa.ERR_UNSUPPORTED   # more workers than grid rows
    assert f(a, 16, a, 16, 0, 2, 16, float("inf"), z) == grawa.ERR_INVALID_ARG


def test_stream_copy_argument_checks(L):
    z = C.c_void_p(0)
    a = C.c_void_p(0x1000)
    assert L.grawa_stream_copy(z, a, 64, z) == grawa.ERR_INVALID_ARG
    assert L.grawa_stream_copy(a, a, -16, z) == grawa.ERR_INVALID_ARG
    assert L.grawa_stream_copy(a, a, 40, z) == grawa.ERR_ALIGNMENT
    assert L.grawa_stream_copy(C.c_void_p(0x1008), a, 64, z) == grawa.ERR_ALIGNMENT


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    monkeypatch.setattr(grawa, "_lib", None)
    monkeypatch.setattr(grawa, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="missing"):
        grawa.lib()


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2403_04206_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower(), "%s mentions the oracle" % fn


def test_bench_refuses_more_than_one_gpu():
    # The benchmark measures one GPU's throughput; asking for more must end with a message, not a run.
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_header_is_plain_c99_and_the_c_client_builds(tmp_path):
    # The boundary is a C ABI: the header must compile as C (not only as C++), and a C99 program that
    # uses it must link against the library (running it needs a GPU and is a GPU test).
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hdr = os.path.join(root, "include", "grawa.h")
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    out = buildlib.build_c_client(os.path.join(root, "tests", "c_abi_client.c"), str(tmp_path / "client"))
    assert os.path.exists(out)
