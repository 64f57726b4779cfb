"""The oracle's C source under the address and undefined-behaviour sanitizers: oracle/sanitize_check.c calls every
function on seeded batch subgraphs with exactly-sized buffers, strides and the degenerate shapes.  CPU only."""
import os
import subprocess

ORACLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")


def test_every_oracle_function_is_clean_under_the_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_check")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-o", exe, os.path.join(ORACLE, "sanitize_check.c"), "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert " 0 failures" in res.stdout
