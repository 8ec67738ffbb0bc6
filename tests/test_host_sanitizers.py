"""The host side of the C-ABI library under AddressSanitizer + UndefinedBehaviorSanitizer: the library is
built a second time with the host pass instrumented (device code unchanged) and the CPU boundary tests —
every argument check, the host budget allocator, the tuning setter — run against that build in a child
process with the sanitizer runtime preloaded.  Any report aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_boundary_tests_pass_under_host_asan_ubsan():
    from paper_2509_09754_amd import build
    if not os.path.exists(build.HIPCC):
        pytest.skip("no hipcc in this environment")
    lib = build.build_library(verbose=False, sanitize=True)
    runtime = build.sanitizer_runtime()
    assert os.path.isabs(runtime) and os.path.exists(runtime), runtime
    env = dict(os.environ, LD_PRELOAD=runtime, LAVA_LIBRARY=lib, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_boundary.py"), "-q", "-x",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
