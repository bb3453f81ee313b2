"""AddressSanitizer + UndefinedBehaviorSanitizer over the library's host-only code (the host
optimizer with its AVX-512 and scalar paths and thread slicing, the strategy search).  Host code
only: no GPU code is built or run here."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_01890_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang++"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="ROCm clang++ not found")
def test_host_code_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "driver"
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-pthread", os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), os.path.join(CSRC, "autohete_host.cpp"),
           os.path.join(CSRC, "autohete_strategy.cpp"), "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitizer" in build.stderr.lower() and "cannot find" in build.stderr.lower():
        pytest.skip("sanitizer runtime not installed with this clang")
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0"))
    assert run.returncode == 0, (run.stdout[-1500:], run.stderr[-3000:])
    assert "sanitizer driver: ok" in run.stdout
