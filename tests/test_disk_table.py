"""History tables on disk, host side (no GPU): the file is the table, row after row; gas_disk_write_rows /
gas_disk_read_rows are the Push / Pull of Algorithm 1 on it and must agree bit for bit with the oracle's push and
pull on an array in memory, through index lists, ranges, strides, many pieces and several I/O threads."""
import os

import numpy as np
import pytest
import torch

from oracle import ops as oops
from paper_2106_05609_amd import binding
from paper_2106_05609_amd.binding import DiskTable, GasError


def _np_view(t):
    return t.view(torch.int16).numpy() if t.dtype == torch.bfloat16 else t.numpy()


def _file_rows(path, n_rows, width, dtype):
    raw = np.fromfile(path, dtype=np.int16 if dtype == torch.bfloat16 else np.float32)
    return raw.reshape(n_rows, width)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("calls", [False, True])
@pytest.mark.parametrize("n_rows,width,threads", [(1000, 64, 1), (5000, 100, 4), (40000, 7, 8)])
def test_write_then_read_matches_the_oracle(tmp_path, dtype, n_rows, width, threads, calls):
    rng = np.random.default_rng(n_rows + width)
    path = str(tmp_path / "hist.bin")
    t = DiskTable(path, n_rows, width, dtype, create=True, io_threads=threads, calls=calls)
    table = np.zeros((n_rows, width), dtype=np.int16 if dtype == torch.bfloat16 else np.float32)
    for sweep in range(3):
        # distinct rows: scattered singles plus runs of consecutive rows (a batch made of clusters)
        start = int(rng.integers(0, n_rows // 2))
        run = np.arange(start, start + n_rows // 5)
        singles = rng.choice(np.setdiff1d(np.arange(n_rows), run), size=n_rows // 4, replace=False)
        idx = np.concatenate([singles[: len(singles) // 2], run, singles[len(singles) // 2:]]).astype(np.int32)
        src = torch.randn(len(idx), width).to(dtype)
        t.write_rows(src, idx)
        oops.push(_np_view(src), idx, table)
        # pull with duplicates and in any order
        want_idx = rng.integers(0, n_rows, size=n_rows // 3).astype(np.int32)
        got = torch.empty(len(want_idx), width, dtype=dtype)
        t.read_rows(got, want_idx)
        assert np.array_equal(_np_view(got), oops.pull(table, want_idx))
    # range form, and the file itself
    got = torch.empty(n_rows // 2, width, dtype=dtype)
    t.read_rows(got, base=n_rows // 4)
    assert np.array_equal(_np_view(got), table[n_rows // 4: n_rows // 4 + n_rows // 2])
    t.sync()
    t.close()
    assert os.path.getsize(path) == n_rows * width * (2 if dtype == torch.bfloat16 else 4)
    assert np.array_equal(_file_rows(path, n_rows, width, dtype), table)


def test_rows_never_written_read_as_zeros_and_the_file_persists(tmp_path):
    path = str(tmp_path / "h.bin")
    t = DiskTable(path, 300, 16, torch.float32, create=True)
    src = torch.arange(5 * 16, dtype=torch.float32).reshape(5, 16) + 1
    t.write_rows(src, base=100)
    t.close()
    t = DiskTable(path, 300, 16, torch.float32, create=False)
    got = torch.full((300, 16), -1.0)
    t.read_rows(got)
    want = torch.zeros(300, 16)
    want[100:105] = src
    assert torch.equal(got, want)
    t.close()
    # create=True empties an existing file
    t = DiskTable(path, 300, 16, torch.float32, create=True)
    t.read_rows(got)
    assert torch.equal(got, torch.zeros(300, 16))
    t.close()


def test_strided_host_rows(tmp_path):
    t = DiskTable(str(tmp_path / "h.bin"), 64, 8, torch.float32, create=True, io_threads=3)
    wide = torch.randn(20, 12)
    idx = torch.randperm(64)[:20].to(torch.int32)
    t.write_rows(wide[:, :8], idx)
    back = torch.zeros(20, 12)
    t.read_rows(back[:, :8], idx)
    assert torch.equal(back[:, :8], wide[:, :8]) and torch.count_nonzero(back[:, 8:]) == 0
    t.close()


def test_errors(tmp_path):
    path = str(tmp_path / "h.bin")
    with pytest.raises(GasError) as e:
        DiskTable(str(tmp_path / "missing.bin"), 10, 4, torch.float32, create=False)
    assert e.value.status == -7
    with pytest.raises(GasError) as e:
        DiskTable(str(tmp_path / "no_such_dir" / "h.bin"), 10, 4, torch.float32, create=True)
    assert e.value.status == -7
    t = DiskTable(path, 10, 4, torch.float32, create=True)
    rows = torch.zeros(3, 4)
    for bad in ([0, 10, 1], [-1, 2, 3]):
        with pytest.raises(GasError) as e:
            t.read_rows(rows, torch.tensor(bad, dtype=torch.int32))
        assert e.value.status == -4
        with pytest.raises(GasError) as e:
            t.write_rows(rows, torch.tensor(bad, dtype=torch.int32))
        assert e.value.status == -4
    with pytest.raises(GasError) as e:
        t.read_rows(rows, base=8)
    assert e.value.status == -4
    with pytest.raises(ValueError):
        t.read_rows(torch.zeros(3, 5))
    with pytest.raises(ValueError):
        t.read_rows(rows, torch.tensor([1, 2, 3]))          # int64 indices
    with pytest.raises(GasError):
        t.wait(5)                                            # a ticket that was never issued
    t.wait()                                                 # nothing queued: returns at once
    t.close()
    t.close()                                                # twice is fine
    with pytest.raises(GasError) as e:                       # a table of another shape on the same file
        DiskTable(path, 11, 4, torch.float32, create=False)
    assert e.value.status == -1
    # an empty table and empty transfers
    t = DiskTable(str(tmp_path / "e.bin"), 0, 4, torch.float32, create=True)
    t.read_rows(torch.zeros(0, 4))
    t.write_rows(torch.zeros(0, 4), torch.zeros(0, dtype=torch.int32))
    t.close()


def test_bad_open_arguments():
    L = binding.lib()
    import ctypes as C
    h = C.c_void_p(0)
    for args in ((b"/tmp/x", 4, 4, 0, 4, 0, 0), (b"/tmp/x", -1, 4, 0, 1, 0, 0), (b"/tmp/x", 4, 0, 0, 1, 0, 0), (b"/tmp/x", 4, 4, 9, 1, 0, 0),
                 (b"/tmp/x", 4, 4, 0, 1, 17, 0), (b"/tmp/x", 4, 4, 0, 1, 0, -5)):
        st = L.gas_disk_open(args[0], C.c_int64(args[1]), C.c_int32(args[2]), C.c_int(args[3]), C.c_int32(args[4]),
                             C.c_int32(args[5]), C.c_int64(args[6]), C.byref(h))
        assert st in (-1, -2) and not h.value
