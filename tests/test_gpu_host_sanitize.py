"""The C ABI's argument and life-cycle paths under AddressSanitizer + UndefinedBehaviorSanitizer (host code only:
api.hip and the driver tests/host_sanitize/lifecycle.cpp are instrumented, the GPU code is not).  The driver checks
every status against what include/gelo.h promises; the sanitizers watch the host side of those calls - the context
pool, the batch-id window, the mixing objects' reuse - on a real device."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(os.path.dirname(HERE), "paper_2603_05035_amd", "lifecycle_hostsan")


@pytest.mark.gpu
def test_lifecycle_under_host_sanitizers():
    if not os.path.exists(EXE):
        pytest.skip("host sanitizer target not built (python paper_2603_05035_amd/build.py --sanitize)")
    env = dict(os.environ)
    # the HIP runtime keeps allocations until exit and maps memory where the sanitizer's shadow gap would be
    env["ASAN_OPTIONS"] = "detect_leaks=0:protect_shadow_gap=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([EXE], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-4000:]
    assert "all statuses as promised" in r.stdout
