"""Builds the native code of this package in-tree.

* ``libxattn.so``: the product -- HIP kernels and C-ABI entry points, gfx950 only, hipcc.  One object
  per source, compiled in parallel, then linked.
* ``libxattn_hosttest.so``: test infrastructure -- the host-only parts (page pool, beam search,
  partition arithmetic) built with g++ against a stand-in for the virtual-memory driver, with the
  test hooks of ``csrc/host_test``.  It runs without a GPU (and under sanitizers, see
  ``tests/test_host_sanitizers.py``); nothing of it is linked into ``libxattn.so``.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
OBJ_DIR = os.path.join(_HERE, "_build")
LIB_PATH = os.path.join(_HERE, "libxattn.so")
HOSTTEST_LIB_PATH = os.path.join(_HERE, "libxattn_hosttest.so")
SOURCES = ["xattn_kernels.hip", "xattn_mla.hip", "xattn_noalloc.hip", "xattn_api.cpp", "xattn_error.cpp", "xtensor.cpp",
           "vmm_hip.cpp", "xtensor_pool.cpp", "xbeam.cpp"]
HOSTTEST_SOURCES = ["xattn_error.cpp", "xtensor_pool.cpp", "xbeam.cpp", os.path.join("host_test", "vmm_fake.cpp"),
                    os.path.join("host_test", "plan_shim.cpp")]
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               # packed-fp32 VALU forms are switched off for all device code of this library
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument", "-pthread"]
GXX_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-pthread"]


def _dependencies():
    deps = []
    for d in (CSRC, os.path.join(CSRC, "host_test"), INCLUDE):
        deps += [os.path.join(d, f) for f in os.listdir(d) if f.endswith((".h", ".hip", ".cpp"))]
    return deps


def _stale(lib: str) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    return any(os.path.getmtime(f) > t for f in _dependencies())


def is_stale(lib: str = LIB_PATH) -> bool:
    """True when the built library is missing or older than any source or header it is built from."""
    return _stale(lib)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("%s failed:\n%s%s" % (cmd[0], res.stdout, res.stderr))
    if verbose and res.stderr.strip():
        print(res.stderr, flush=True)


def build(force: bool = False, verbose: bool = False) -> str:
    """Compile libxattn.so if it is missing or older than its sources (always when force)."""
    if force or _stale(LIB_PATH):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        os.makedirs(OBJ_DIR, exist_ok=True)
        objs = [os.path.join(OBJ_DIR, s.replace(os.sep, "_") + ".o") for s in SOURCES]

        def compile_one(so):
            _run([hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose)

        with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as pool:
            list(pool.map(compile_one, zip(SOURCES, objs)))
        tmp = LIB_PATH + ".tmp.%d" % os.getpid()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread"] + objs + ["-o", tmp], verbose)
        os.replace(tmp, LIB_PATH)
    return LIB_PATH


def build_hosttest(force: bool = False, verbose: bool = False, extra_flags=(), out: str = HOSTTEST_LIB_PATH) -> str:
    """Compile the host test library (g++, no GPU code)."""
    if force or out != HOSTTEST_LIB_PATH or _stale(out):
        tmp = out + ".tmp.%d" % os.getpid()
        _run([os.environ.get("CXX", "g++")] + GXX_FLAGS + list(extra_flags) + ["-shared"] +
             [os.path.join(CSRC, s) for s in HOSTTEST_SOURCES] + ["-o", tmp], verbose)
        os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_hosttest(force=True, verbose=True))
