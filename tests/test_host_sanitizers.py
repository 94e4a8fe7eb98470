"""AddressSanitizer + UBSan over the library's host side: argument validation, ctx / workspace sizing at
the accepted limits, the launch-fact cache's fallbacks and the stage timer's enable / read / disable
cycles, driven by a small C++ program (tests/host/abi_sanitizer_driver.cpp) that needs no GPU."""
import os
import subprocess

import pytest


def test_host_side_is_clean_under_asan_and_ubsan():
    import torch
    if torch.cuda.is_available():
        pytest.skip("host sanitizer build is a CPU-box check")
    from paper_2306_15799_amd import build
    lib, driver = build.build_sanitized()
    env = dict(os.environ)
    # the HIP runtime keeps process-lifetime allocations: leak reports at exit are not this library's
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    try:
        res = subprocess.run([driver], capture_output=True, text=True, env=env, timeout=300)
    finally:
        for f in (lib, driver):          # 20 MB of instrumented code nobody else needs
            if os.path.exists(f):
                os.remove(f)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "all expectations held" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
