"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, no GPU: the CPU oracle (every function, on heap
buffers of exactly the documented sizes) and the library's host side (descriptor checks, workspace queries, launch
planning, job-table validation, the layer-removal fixed point).  Device code is not instrumented."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
BUILD = os.path.join(ROOT, "_build", "sanitize")
CSRC = os.path.join(ROOT, "paper_1901_09290_amd", "csrc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _newer(target, sources):
    return os.path.exists(target) and os.path.getmtime(target) >= max(os.path.getmtime(s) for s in sources)


def _run(exe, expect):
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=120)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert expect in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    os.makedirs(BUILD, exist_ok=True)
    exe = os.path.join(BUILD, "oracle_driver")
    srcs = [os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "oracle.c"), os.path.join(ROOT, "oracle", "oracle.h")]
    if not _newer(exe, srcs):
        subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
                        "-I", os.path.join(ROOT, "oracle"), "-o", exe, srcs[0], srcs[1], "-lm"], check=True)
    _run(exe, "oracle sanitize ok")


def test_library_host_side_under_address_and_undefined_behaviour_sanitizers():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    os.makedirs(BUILD, exist_ok=True)
    exe = os.path.join(BUILD, "host_driver")
    lib_srcs = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))]
    srcs = [os.path.join(HERE, "host_driver.cpp"), os.path.join(ROOT, "include", "prunetrain.h")] + lib_srcs
    if not _newer(exe, srcs):
        hip = [s for s in lib_srcs if s.endswith(".hip")]
        # the sanitizers apply to the host pass only (each -fsanitize directly behind -Xarch_host)
        cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
               "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-fno-gpu-sanitize",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", exe, "-x", "hip", srcs[0]] + hip
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-4000:]
    _run(exe, "host sanitize ok")
