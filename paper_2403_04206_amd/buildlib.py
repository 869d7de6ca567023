"""Build libgrawa.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to build."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libgrawa.so")
BUILD = os.path.join(PKG, "_build")
SOURCES = [os.path.join(CSRC, n) for n in ("grawa_api.cpp", "grawa_maps.cpp", "grawa_norms.hip", "grawa_pull.hip",
                                            "grawa_local.hip", "grawa_static.hip")]
HEADERS = [os.path.join(CSRC, "grawa_internal.h"), os.path.join(CSRC, "grawa_device.h"), os.path.join(CSRC, "grawa_maps.h"),
           os.path.join(ROOT, "include", "grawa.h")]

# Packed fp32 instructions are switched off for all device code (a hipcc flag, not a host one;
# the host pass warns that it does not know the feature, which is harmless).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the GRAWA library needs the ROCm toolchain to build")
    return exe


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library (one object per source, in parallel, then one link); returns its path.
    force=False skips an up-to-date build."""
    if not force and not needs_build():
        return LIB
    os.makedirs(BUILD, exist_ok=True)
    tag = ".tmp.%d" % os.getpid()
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]

    def compile_one(src):
        obj = os.path.join(BUILD, os.path.basename(src) + tag + ".o")
        cmd = [hipcc()] + HIPCC_FLAGS + inc + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        return obj, res

    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as pool:
        results = list(pool.map(compile_one, SOURCES))
    objs = [o for o, _ in results]
    tmp = LIB + tag
    try:
        for _, res in results:
            if res.returncode != 0:
                raise RuntimeError("hipcc failed:\n" + res.stdout)
            if verbose and res.stdout.strip():
                print(res.stdout)
        link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        if verbose:
            print(" ".join(link), flush=True)
        res = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stdout)
        os.replace(tmp, LIB)
    finally:
        for f in objs + [tmp]:
            if os.path.exists(f):
                os.remove(f)
    return LIB


def build_c_client(src: str, out: str) -> str:
    """Compile a plain C99 program that calls the library through include/grawa.h (gcc, linked against
    libgrawa.so and the HIP runtime; the library is found relative to the program's own location)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    os.makedirs(os.path.dirname(out), exist_ok=True)
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), src, "-o", out, "-L", PKG, "-l:libgrawa.so",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.relpath(PKG, os.path.dirname(out)).join(
               ["$ORIGIN/", ""]), "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
