"""The CPU checker and the host side of the C-ABI library under the address and
undefined-behaviour sanitizers (no GPU): the checker's pins and the library's host checks
(plan arithmetic, argument validation, byte queries, placement in a fusion buffer) run in a
child process that has clang's sanitizer runtime preloaded and loads the sanitized builds
of both libraries.  Any report ends the child with a non-zero status."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SUITES = ["tests/test_oracle_pins.py", "tests/test_epilogue_oracle.py", "tests/test_accumulate_oracle.py",
          "tests/test_abi_and_host_logic.py"]


@pytest.mark.timeout(900)
def test_checker_and_host_logic_under_asan_and_ubsan():
    from oracle import build as oracle_build
    from paper_1905_04035_amd import build as hip_build

    try:
        runtime = oracle_build.sanitizer_runtime()
    except (FileNotFoundError, subprocess.CalledProcessError) as e:       # no clang runtime on this host
        pytest.skip(str(e))
    oracle_build.build(force=True, sanitize=True)
    hip_build.build(force=True, sanitize=True)

    env = dict(os.environ)
    env["TS_SANITIZE"] = "1"
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: its allocations at exit are not this code's leaks
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + SUITES
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=850)
    text = res.stdout + res.stderr
    assert res.returncode == 0, text[-4000:]
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    assert " passed" in res.stdout
