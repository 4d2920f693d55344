"""The host side of the library (argument validation, the launch plan, handle bookkeeping) under
AddressSanitizer and UndefinedBehaviorSanitizer: tests/host/abi_driver.cpp drives the C ABI with
NG_INIT_HOST_ONLY handles, so no GPU is needed.  The device code is compiled as usual."""
import os
import shutil
import subprocess

import pytest

from paper_2410_16029_amd import build as ngbuild


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_host_scheduler_is_clean_under_asan_and_ubsan():
    exe = ngbuild.build_host_sanitizer(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = res.stdout + res.stderr
    assert res.returncode == 0, report[-4000:]
    assert "all checks passed" in res.stdout
    for marker in ("AddressSanitizer", "LeakSanitizer", "runtime error:"):
        assert marker not in report, report[-4000:]
