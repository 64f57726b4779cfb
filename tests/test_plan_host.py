"""The plan builder's host definition (paper_2106_05609_amd/csrc/plan_host.h) under the address and
undefined-behaviour sanitizers: csrc/plan_check.cpp builds plans for seeded random, edge-case and malformed patterns
and checks every invariant the kernels index by.  Host code only; no GPU is involved."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(os.path.dirname(HERE), "paper_2106_05609_amd", "csrc")


def test_plan_builder_invariants_under_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_check")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-o", exe, os.path.join(CSRC, "plan_check.cpp")])
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1")
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert " 0 failures" in res.stdout
