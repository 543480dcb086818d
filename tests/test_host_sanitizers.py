"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The HIP sources are compiled once more with the sanitizers on their host pass (the device pass is
untouched) and linked with tests/native/host_sanitize_main.cpp, which drives every entry point
through its validation, the wire-format parser, the alias check, the schedule helpers, the
per-thread launch shape and, where no GPU is present, the launch-shape arithmetic of every kernel
choice (the launch itself is then refused by the runtime).  A sanitizer report aborts the program.
"""
import os
import shutil
import subprocess

import pytest

from paper_2502_12996_amd import build as BUILD

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    exe = tmp_path / "host_sanitize"
    flags = [f for f in BUILD.FLAGS if f not in ("-O3", "-fPIC", "-shared")]
    cmd = [hipcc, *flags, "-O1", "-g",
           # sanitizers for the host pass only: each -fsanitize= directly after -Xarch_host
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", BUILD.CSRC,
           *[os.path.join(BUILD.CSRC, s) for s in BUILD.SOURCES],
           os.path.join(ROOT, "tests", "native", "host_sanitize_main.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True)
    nm = shutil.which("nm")
    if nm:       # the runtimes are really linked in
        syms = subprocess.run([nm, str(exe)], check=True, capture_output=True, text=True).stdout
        assert "__asan_init" in syms and "__ubsan_handle" in syms
    import torch
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="print_stacktrace=1")
    runs = [{}]
    if not torch.cuda.is_available():
        # made-up addresses may reach the launch call only where the runtime has no GPU to launch on
        runs.append({"DILOCO_HOST_CHECK_LAUNCH_PATHS": "1"})
    for extra in runs:
        r = subprocess.run([str(exe)], env=dict(env, **extra), capture_output=True, text=True, timeout=300)
        assert r.returncode == 0, (extra, r.stdout[-2000:], r.stderr[-4000:])
        assert "host checks passed" in r.stdout
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
