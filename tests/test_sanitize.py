"""Sanitizer builds (CPU only): the oracle under AddressSanitizer + UndefinedBehaviorSanitizer, driven by
tests/sanitize_oracle_main.c; and the host side of the HIP library (argument validation, no launches) under
the same sanitizers, driven by the argument checks of tests/test_cabi_host.py in a child process."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe, os.path.join(ROOT, "oracle", "moss_oracle.c"),
           os.path.join(HERE, "sanitize_oracle_main.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "oracle sanitizer run: ok" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def test_library_host_side_under_asan_and_ubsan(tmp_path):
    """Every entry point's argument validation (tests/test_cabi_host.py, which never launches a kernel) against a
    build of the library whose host code carries AddressSanitizer and UndefinedBehaviorSanitizer."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    rt = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("the compiler ships no shared AddressSanitizer runtime")
    from paper_2511_05811_amd import build as hip_build
    lib = str(tmp_path / "libmoss_hip_san.so")
    flags = [f for f in hip_build.FLAGS if f != "-O3"] + ["-O1", "-g"]
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        flags += ["-Xarch_host", f]
    cmd = [hipcc] + flags + ["-shared-libasan", "-I", hip_build.INCLUDE, "-o", lib] + [os.path.join(hip_build.CSRC, s) for s in hip_build.SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    preload = ":".join(x for x in (rt, os.environ.get("LD_PRELOAD", "")) if x)     # the sanitizer runtime has to come first
    env = dict(os.environ, MOSS_HIP_LIBRARY=lib, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_cabi_host.py"), "-q", "-x", "-p", "no:cacheprovider"],
                         capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
