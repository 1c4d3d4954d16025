"""The host translation units under sanitizers (CPU only): the page pool with its background thread on
the stand-in driver, the beam-search selection, the partition arithmetic, the CPU oracle and the input
generator are compiled with gcc/g++ into one executable (tests/host/sanitize_main.cpp drives them) --
once with AddressSanitizer + UndefinedBehaviorSanitizer, once with ThreadSanitizer -- and run.

The same two commands by hand, from the repository root:

  g++ -std=c++17 -g -O1 -pthread -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp \\
      tests/host/sanitize_main.cpp paper_2510_14686_amd/csrc/{xattn_error,xtensor_pool,xbeam}.cpp \\
      paper_2510_14686_amd/csrc/host_test/{vmm_fake,plan_shim}.cpp -x c oracle/oracle_attn.c workloads/gen.c \\
      -lm -o /tmp/xattn_host_asan && /tmp/xattn_host_asan
  (the same with -fsanitize=thread and without -fopenmp for ThreadSanitizer)
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_14686_amd", "csrc")
CXX_SOURCES = [os.path.join(ROOT, "tests", "host", "sanitize_main.cpp")] + \
    [os.path.join(CSRC, f) for f in ("xattn_error.cpp", "xtensor_pool.cpp", "xbeam.cpp",
                                     os.path.join("host_test", "vmm_fake.cpp"), os.path.join("host_test", "plan_shim.cpp"))]
C_SOURCES = [os.path.join(ROOT, "oracle", "oracle_attn.c"), os.path.join(ROOT, "workloads", "gen.c")]
FOUND = ("ERROR: AddressSanitizer", "ERROR: LeakSanitizer", "runtime error:", "WARNING: ThreadSanitizer", "CHECK failed")


def _build_and_run(tmp_path, name, flags, env_extra):
    exe = os.path.join(str(tmp_path), name)
    objs = []
    for i, src in enumerate(C_SOURCES):
        obj = os.path.join(str(tmp_path), "%s_c%d.o" % (name, i))
        subprocess.run(["gcc", "-std=c11", "-g", "-O1", "-fno-omit-frame-pointer", "-c", src, "-o", obj] + flags,
                       check=True, capture_output=True, text=True)
        objs.append(obj)
    res = subprocess.run(["g++", "-std=c++17", "-g", "-O1", "-fno-omit-frame-pointer", "-pthread", "-Wall", "-Wextra"] + flags +
                         CXX_SOURCES + objs + ["-lm", "-o", exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", **env_extra)
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    text = run.stdout + run.stderr
    sys.stdout.write(text[-2000:])
    for needle in FOUND:
        assert needle not in text, text[-4000:]
    assert run.returncode == 0, text[-4000:]
    assert "all scenarios ran" in text


def test_address_and_undefined_behaviour_sanitizers(tmp_path):
    _build_and_run(tmp_path, "xattn_host_asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp"],
                   {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1"})


def test_thread_sanitizer(tmp_path):
    # without OpenMP: libgomp is not instrumented and would only add false reports; the threads of
    # interest are the pool's pre-mapping thread and the concurrent callers
    _build_and_run(tmp_path, "xattn_host_tsan", ["-fsanitize=thread"], {"TSAN_OPTIONS": "halt_on_error=0"})
