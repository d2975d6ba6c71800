"""Sanitizer builds.  The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: its pins, the golden fixtures
and the index file reader are run once more in a child process that loads the sanitized build, where any report ends the
run.  The library's HOST code (argument checks, index-file reader, refusals before the GPU is touched) likewise."""
import os
import pathlib
import subprocess
import sys

import pytest

from oracle import build as B

ROOT = pathlib.Path(__file__).resolve().parent.parent


def test_pins_golden_fixtures_and_file_reader_are_clean_under_asan_and_ubsan():
    runtime = B.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's libasan.so is not installed")
    lib = B.build_sanitized()
    env = dict(os.environ)
    preload = [p for p in env.get("LD_PRELOAD", "").split(":") if p]          # keep whatever is preloaded already
    env["LD_PRELOAD"] = ":".join([runtime] + preload)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:verify_asan_link_order=0"     # (the interpreter itself is not leak-clean)
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["LORANN_ORACLE_LIB"] = str(lib)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           "tests/test_oracle_pins.py", "tests/test_golden.py", "tests/test_index_file.py"]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert " passed" in out


def test_library_host_code_is_clean_under_asan_and_ubsan():
    from paper_2410_18926_amd import build as LB
    try:
        runtime = LB.sanitizer_runtime()
    except Exception:
        pytest.skip("clang is not installed")
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("clang's sanitizer runtime is not installed")
    lib = LB.build_sanitized()
    env = dict(os.environ)
    preload = [p for p in env.get("LD_PRELOAD", "").split(":") if p]          # keep whatever is preloaded already
    env["LD_PRELOAD"] = ":".join([runtime] + preload)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["LORANN_LIB"] = str(lib)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           "tests/test_abi_host.py", "tests/test_index_file.py"]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert " passed" in out
