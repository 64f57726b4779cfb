"""The C-ABI library loads and exports every symbol include/gas.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

from paper_2106_05609_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gas.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"GAS_API\s+[\w\s\*]+?\b(gas_\w+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert len(names) >= 12 and "gas_pull" in names and "gas_spmm_t" in names
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in gas.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_version_and_error_string_without_a_gpu():
    assert binding.gas_version() >= 100
    assert isinstance(binding.lib().gas_last_error(), bytes)


def test_argument_errors_are_reported_before_any_launch():
    L = binding.lib()
    st = L.gas_pull(None, ctypes.c_int64(10), ctypes.c_int64(4), None, ctypes.c_int64(0), ctypes.c_int64(3),
                    ctypes.c_int32(4), ctypes.c_int(0), None, ctypes.c_int64(4), None)
    assert st == -1 and b"null" in L.gas_last_error()
    st = L.gas_pull(None, ctypes.c_int64(10), ctypes.c_int64(4), None, ctypes.c_int64(0), ctypes.c_int64(3),
                    ctypes.c_int32(4), ctypes.c_int(7), None, ctypes.c_int64(4), None)
    assert st == -2
    # n == 0 is a no-op even with null pointers
    st = L.gas_push(None, ctypes.c_int64(4), None, ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int32(4),
                    ctypes.c_int(0), None, ctypes.c_int64(10), ctypes.c_int64(4), None)
    assert st == 0
    one = ctypes.c_void_p(16)
    st = L.gas_linear(one, ctypes.c_int64(8), ctypes.c_int64(5), ctypes.c_int32(8), one, ctypes.c_int32(4), None,
                      ctypes.c_int(0), ctypes.c_float(0.5), ctypes.c_float(0.5), ctypes.c_int(0), ctypes.c_void_p(32),
                      ctypes.c_int64(4), None)
    assert st == -1 and b"identity" in L.gas_last_error()
