"""The host side of the library (argument validation, the token schedule, workspace carving, launch-shape logic)
under AddressSanitizer + UndefinedBehaviorSanitizer: the sources are compiled once more with the sanitizers on the
host code only, and the host-ABI tests - every argument error, the schedules of all five configurations - run
against that build in a child process.  No GPU is involved: every call in those tests returns before a launch."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_abi_under_address_and_ub_sanitizers():
    from paper_2601_13143_amd import build as B
    try:
        rt = B.asan_runtime()
    except FileNotFoundError as e:                      # a toolchain without the shared runtime: nothing to run
        pytest.skip(str(e))
    lib = B.build_asan()
    env = dict(os.environ)
    env.update({"LD_PRELOAD": rt, "FASTAV_LIBRARY": lib,
                "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:abort_on_error=0",
                "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"})
    p = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_host_abi.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    out = p.stdout + p.stderr
    assert p.returncode == 0, out[-4000:]
    assert "passed" in out and "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
