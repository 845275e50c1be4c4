"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): its own
test files are run once more in a child process that loads the sanitized build of oracle/dam_oracle.c. Any
out-of-bounds access, use after free, signed overflow or misaligned access in the checker aborts that run."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_suite_under_asan_and_ubsan():
    if os.environ.get("DAM_ORACLE_SANITIZE") == "1":
        pytest.skip("already inside the sanitized run")
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    oracle_build.build(force=True, sanitize=True)
    runtime = oracle_build.asan_runtime()
    assert os.path.isabs(runtime) and os.path.exists(runtime), f"libasan not found: {runtime}"
    env = dict(os.environ)
    env["DAM_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime goes first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    # python itself is not instrumented: its own leaks are not this test's business; the link-order check would
    # refuse a runtime that another preloaded library precedes
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    files = sorted(f for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle_") and f.endswith(".py")
                   and f != "test_oracle_sanitized.py")
    assert files
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] +
                       [os.path.join("tests", f) for f in files], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    # the sanitized library is the one that was loaded
    probe = subprocess.run([sys.executable, "-c", "import oracle; print(oracle.lib()._name)"], cwd=ROOT, env=env,
                           capture_output=True, text=True, timeout=120)
    assert probe.returncode == 0 and "libdam_oracle_asan.so" in probe.stdout, probe.stdout + probe.stderr
