"""The library's HIP-free host code (scheduler, host-core expert FFN with its
thread pool, alpha selection) under the host sanitizers: a native driver is
built twice, with AddressSanitizer + UndefinedBehaviorSanitizer and with
ThreadSanitizer, and must run clean.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_18983_amd", "csrc")
DRIVER = os.path.join(ROOT, "tests", "native", "host_sanitize.cpp")


def _build_and_run(tmp_path, name, flags, env_extra):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = tmp_path / name
    cmd = [gxx, "-O1", "-g", "-std=c++17", "-pthread", "-fno-omit-frame-pointer", *flags,
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, DRIVER, os.path.join(CSRC, "cpu_expert.cpp"),
           "-o", str(exe)]
    subprocess.run(cmd, check=True, cwd=ROOT)
    env = dict(os.environ, **env_extra)
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    return r


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    r = _build_and_run(tmp_path, "host_asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"],
                       {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
                        "UBSAN_OPTIONS": "print_stacktrace=1"})
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host code: ok" in r.stdout and "ERROR" not in r.stderr and "runtime error" not in r.stderr


def test_host_thread_pool_under_thread_sanitizer(tmp_path):
    r = _build_and_run(tmp_path, "host_tsan", ["-fsanitize=thread", "-DSMOE_NO_CLONES"], {"TSAN_OPTIONS": "halt_on_error=1"})
    if r.returncode != 0 and "unexpected memory mapping" in r.stderr:
        pytest.skip("ThreadSanitizer cannot map its shadow memory on this kernel")
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host code: ok" in r.stdout and "WARNING: ThreadSanitizer" not in r.stderr
