"""The library's host side (argument validation, clip tables, run splitting, tile scheduler) under
AddressSanitizer and UndefinedBehaviorSanitizer.  csrc/vfm_api.hip is compiled with both for the
host, linked with stub launchers (tests/host_sanitize/driver.hip) that check every table handed
to them, and driven with hundreds of random clip mixes on both sides of every run boundary.
CPU only: nothing is launched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(shutil.which(HIPCC) is None and not os.path.exists(HIPCC), reason="hipcc not available")
def test_host_paths_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    csrc = os.path.join(ROOT, "paper_2503_12964_amd", "csrc")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Wno-unused-command-line-argument",
           "-Wno-inline-asm", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-I", csrc,
           os.path.join(csrc, "vfm_api.hip"), os.path.join(ROOT, "tests", "host_sanitize", "driver.hip"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    assert res.returncode == 0, err[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:] + run.stderr[-4000:])
    assert run.stdout.strip().startswith("ok:"), run.stdout[-500:]
