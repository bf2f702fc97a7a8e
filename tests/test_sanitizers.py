"""Sanitizer passes over the CPU-side code (no GPU): the oracle's C file under gcc's AddressSanitizer +
UndefinedBehaviorSanitizer, and the library's host logic (argument checks, planning, hooks) under
clang's, each in a child process with the matching runtime preloaded.  What runs inside are the
ordinary tests: the oracle's pins, and the host-only ABI tests."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(env_extra, preload, args):
    env = dict(os.environ)
    env.update(env_extra)
    keep = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = preload + (":" + keep if keep else "")         # the sanitizer runtime has to come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *args], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return tail


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("gcc's libasan is not installed")
    tail = _run({"OWL_ORACLE_SANITIZE": "1"}, libasan, ["tests/test_oracle_pins.py", "tests/test_oracle_steps.py"])
    assert " passed" in tail


def test_host_layer_under_address_and_undefined_behaviour_sanitizers():
    from paper_2510_07535_amd import build as owl_build
    rt = owl_build.asan_runtime()
    if not rt:
        pytest.skip("clang's shared ASan runtime is not installed")
    lib = owl_build.build_host_sanitized()
    tail = _run({"OWL_LIB_PATH": lib}, rt, ["tests/test_abi_host.py"])
    assert " passed" in tail
