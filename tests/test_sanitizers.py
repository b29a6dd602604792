"""Sanitizer runs on the CPU (AddressSanitizer + UndefinedBehaviorSanitizer, errors are fatal):
  - the C oracle, built with gcc's sanitizers, under its pin tests;
  - the host code of the C-ABI library (argument validation, launch plans, workspace carving), built with hipcc's
    host-side sanitizers, under the boundary tests (which launch nothing).
Each run is a child process with the sanitizer runtime preloaded; the GPU is not involved."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# leaks: the interpreter's own; link order: the runtime is preloaded into an uninstrumented python
ASAN_OPTIONS = "detect_leaks=0:verify_asan_link_order=0:alloc_dealloc_mismatch=0:abort_on_error=0"


def run_pytest_under(preload, files, extra_env, timeout=600):
    env = dict(os.environ)
    env.update(extra_env)
    env["LD_PRELOAD"] = (preload + " " + env.get("LD_PRELOAD", "")).strip()
    env["ASAN_OPTIONS"] = ASAN_OPTIONS
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files]
    pr = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                        timeout=timeout)
    tail = "\n".join(pr.stdout.splitlines()[-40:])
    assert pr.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in pr.stdout and "runtime error:" not in pr.stdout, tail
    assert " passed" in pr.stdout, tail
    return pr.stdout


def gcc_runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], check=True, stdout=subprocess.PIPE,
                          text=True).stdout.strip()
    if not os.path.isabs(path):
        pytest.skip(f"gcc has no {name}")
    return path


def test_oracle_pins_under_asan_ubsan():
    preload = gcc_runtime("libasan.so") + " " + gcc_runtime("libubsan.so")
    out = run_pytest_under(preload, ["tests/test_oracle_pins.py", "tests/test_oracle_sketch_pins.py",
                                     "tests/test_oracle_backward_pins.py"], {"GKA_ORACLE_SANITIZED": "1"})
    assert "skipped" not in out.splitlines()[-1]


def test_library_host_code_under_asan_ubsan():
    from paper_2511_21016_amd import build
    lib = build.build_host_sanitized()
    run_pytest_under(build.sanitizer_runtime(), ["tests/test_library_abi.py"], {"GKA_LIBRARY": lib})
