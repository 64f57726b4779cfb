"""The cache model behind bench/l2_model.py (bench/l2_model.c), on traces small enough to check by hand: LRU
replacement within a set, one cache per XCD, work items advancing in turn, cold insertions.  CPU only."""
import ctypes as C
import os
import subprocess

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _model(tmp_path):
    so = str(tmp_path / "libl2_model.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-shared", "-fPIC", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                           "-o", so, os.path.join(ROOT, "bench", "l2_model.c")])
    lib = C.CDLL(so)
    lib.l2_model.restype = C.c_longlong

    def run(index, items, xcd_start, slots, ways, nconc, step, cold=None):
        index = np.ascontiguousarray(index, dtype=np.int32)
        items = np.ascontiguousarray(items, dtype=np.int32)
        xs = np.ascontiguousarray(xcd_start, dtype=np.int32)
        cold = None if cold is None else np.ascontiguousarray(cold, dtype=np.uint8)
        hits = C.c_longlong(0)
        miss = lib.l2_model(index.ctypes.data_as(C.c_void_p), items.ctypes.data_as(C.c_void_p), xs.ctypes.data_as(C.c_void_p),
                            slots, ways, nconc, step, None if cold is None else cold.ctypes.data_as(C.c_void_p), C.byref(hits))
        return int(miss), int(hits.value)
    return run


def test_lru_and_xcd_separation(tmp_path):
    run = _model(tmp_path)
    one_xcd = [0, 1] + [1] * 7
    # one fully associative set of two rows: 1 2 1 3 2 -> miss miss hit miss(evicts 2) miss
    assert run([1, 2, 1, 3, 2], [[0, 5]], one_xcd, 2, 2, 1, 8) == (4, 1)
    # the same row gathered on two XCDs is fetched twice: each XCD has its own cache
    two = [0, 1, 2] + [2] * 6
    assert run([7, 7, 7, 7], [[0, 2], [2, 4]], two, 2, 2, 1, 8) == (2, 2)
    # two items in flight on one XCD advance in turn, one gather each: 5 6 5 6 in a set of two rows -> two misses only
    assert run([5, 5, 6, 6], [[0, 2], [2, 4]], [0] + [2] * 8, 2, 2, 2, 1) == (2, 2)
    # one after the other instead (one item in flight), same result here; with a one-row cache the order matters
    assert run([5, 5, 6, 6], [[0, 2], [2, 4]], [0] + [2] * 8, 1, 1, 1, 1) == (2, 2)
    assert run([5, 5, 6, 6], [[0, 2], [2, 4]], [0] + [2] * 8, 1, 1, 2, 1) == (4, 0)
    # a streaming scan through more rows than the cache holds evicts a reused row ...
    trace = [9, 9] + list(range(100, 104)) + [9]
    assert run(trace, [[0, len(trace)]], one_xcd, 4, 4, 1, 8) == (6, 1)
    # ... unless the scan's gathers are inserted cold: they replace each other and the reused row stays
    cold = [0, 0] + [1] * 4 + [0]
    assert run(trace, [[0, len(trace)]], one_xcd, 4, 4, 1, 8, cold) == (5, 2)
    # nothing to do
    assert run([1], np.zeros((0, 2)), [0] * 9, 4, 4, 4, 8) == (0, 0)
