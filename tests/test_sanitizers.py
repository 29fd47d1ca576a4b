"""Host-code sanitizer runs (CPU only): the oracle under its pins, and the library's host side
(argument checks, workspace layout, allocation helper) under the ABI tests, both compiled with
AddressSanitizer and UndefinedBehaviorSanitizer.  Each suite runs in a child process with the
matching sanitizer runtime preloaded in front of whatever is preloaded already; a finding makes
the child exit non-zero.  Device code is never sanitized."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(runtime, extra_env, args):
    env = dict(os.environ)
    env.update(extra_env)
    env["LD_PRELOAD"] = runtime + (" " + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *args],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail


def test_oracle_pins_under_asan_ubsan():
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    _run(runtime, {"HEXA_ORACLE_SANITIZE": "1"}, ["tests/test_oracle_pins.py"])


def test_library_host_code_under_asan_ubsan():
    from paper_2411_01288_amd import build as bld
    bld.build_sanitized_library()
    _run(bld.sanitizer_runtime(), {"HEXA_MOE_SANITIZE": "1"},
         ["tests/test_abi_host.py", "-k", "not bench_refuses"])
