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


def _signatures():
    text = open(os.path.join(ROOT, "include", "gas.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    sigs = {}
    for m in re.finditer(r"GAS_API\s+gas_status\s+(gas_\w+)\s*\(([^;]*?)\)\s*;", text, flags=re.S):
        params = [re.sub(r"\s+", " ", p).strip() for p in m.group(2).split(",")]
        sigs[m.group(1)] = params
    return sigs


def _args(params, pointer, dtype, size):
    """ctypes arguments for a parameter list: every pointer = `pointer`, every dtype = `dtype`, the first
    int64 count = `size`, other integers 4, floats 1."""
    out, first = [], True
    for p in params:
        name = p.split()[-1].lstrip("*")
        if "*" in p:
            out.append(None if pointer is None else ctypes.c_void_p(pointer))
        elif p.startswith("gas_dtype"):
            out.append(ctypes.c_int(dtype))
        elif p.startswith("float"):
            out.append(ctypes.c_float(1.0))
        elif p.startswith("int64_t"):
            counts = name in ("n", "n_rows", "nnz")
            out.append(ctypes.c_int64(size if counts and first else 4))
            first = first and not counts
        elif p.startswith("int32_t"):
            out.append(ctypes.c_int32(4))
        elif p.startswith("int "):
            out.append(ctypes.c_int(0))
        else:
            raise AssertionError(f"unhandled parameter {p!r}")
    return out


def test_every_entry_point_rejects_bad_arguments_without_launching():
    """Null pointers, an unknown dtype and a negative count: each call returns an error status and leaves a
    message; nothing is launched (there is no GPU here), nothing crashes."""
    L = binding.lib()
    sigs = _signatures()
    assert len(sigs) >= 25
    for name, params in sigs.items():
        fn = getattr(L, name)
        fn.restype = ctypes.c_int
        st = fn(*_args(params, None, 0, 4))
        if name == "gas_disk_close":      # like free(): closing no table is allowed
            assert st == 0
            continue
        assert st < 0, f"{name} accepted null pointers"
        assert len(L.gas_last_error()) > 0, name
        takes_object = any("gas_plan" in p or "gas_disk_table*" in p.replace(" *", "*") for p in params)
        if takes_object:
            continue                      # a non-null dummy plan or table would be dereferenced
        if any(p.startswith("gas_dtype") for p in params):
            st = fn(*_args(params, 4096, 7, 4))
            assert st < 0, f"{name} accepted dtype 7"
        if any(p.split()[-1] in ("n", "n_rows", "nnz") for p in params if p.startswith("int64_t")):
            st = fn(*_args(params, 4096, 0, -1))
            assert st < 0, f"{name} accepted a negative count"


def test_a_zero_count_is_a_no_op():
    """n = 0 (an empty batch, an empty halo) succeeds without touching any pointer; the weight gradient and the
    squared norm are the exceptions, since an empty sum still has to be written (a zero matrix, a zero), and so are
    the backward aggregations, whose output rows (n_out of them) exist without any row of the pattern."""
    L = binding.lib()
    for name, params in _signatures().items():
        if any("gas_plan" in p or "gas_disk_table" in p for p in params):
            continue
        if not any(p.split()[-1] in ("n", "n_rows", "nnz") for p in params if p.startswith("int64_t")):
            continue
        fn = getattr(L, name)
        fn.restype = ctypes.c_int
        st = fn(*_args(params, None, 0, 0))
        assert st == (-1 if name in ("gas_linear_bwd_weight", "gas_linear_bwd_weight_static", "gas_sq_norm",
                                  "gas_pna_aggregate_bwd", "gas_gat_aggregate_bwd") else 0), name
