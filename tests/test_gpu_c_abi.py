"""The C ABI used from a program that knows nothing of Python or PyTorch (tests/c_abi_check.cpp: hipMalloc'ed
pointers, the calls of include/gas.h, the oracle's C functions as the checker), built against the in-tree libraries."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_layer_step_from_plain_c(tmp_path):
    from oracle import build as obuild
    from paper_2106_05609_amd import binding
    obuild.build()
    exe = str(tmp_path / "c_abi_check")
    pkg, orc = os.path.dirname(binding.LIB_PATH), os.path.dirname(obuild.LIB)
    subprocess.check_call(["hipcc", "-O1", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_abi_check.cpp"), "-o", exe,
                           "-L" + pkg, "-lgas", "-L" + orc, "-lgas_oracle",
                           "-Wl,-rpath," + pkg, "-Wl,-rpath," + orc], stderr=subprocess.DEVNULL)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    assert res.stdout.strip().endswith("ok")
