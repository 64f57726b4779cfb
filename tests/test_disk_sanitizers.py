"""The file-backed history table's host code (paper_2106_05609_amd/csrc/disk.hip) under the sanitizers:
csrc/disk_check.cpp round-trips tables through index lists, ranges and strides with several I/O threads in both I/O
modes and takes the error paths; built once with the address and undefined-behaviour sanitizers and once with the
thread sanitizer (host side only; no GPU is involved)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2106_05609_amd", "csrc")


@pytest.mark.parametrize("sanitizer", ["address,undefined", "thread"])
def test_disk_table_host_code_under_sanitizers(tmp_path, sanitizer):
    exe = str(tmp_path / "disk_check")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-pthread",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unused-command-line-argument", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
                           "-Xarch_host", "-fsanitize=" + sanitizer,
                           os.path.join(CSRC, "disk.hip"), os.path.join(CSRC, "disk_check.cpp"), "-o", exe],
                          stderr=subprocess.DEVNULL)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1",
               TSAN_OPTIONS="halt_on_error=1")
    res = subprocess.run([exe, str(tmp_path)], env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert " 0 failures" in res.stdout
