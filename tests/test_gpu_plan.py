"""The plan built by kernels on the device against the host builder that defines it (csrc/plan_host.h, selected with
gas_plan_options.host_builder): the same lists, entry by entry, for batch subgraphs of the benchmark's graph
families, fused source indices, and parameter sets that force many heavy rows, tiny windows and one-entry chunks;
malformed row pointers are rejected on the device without reading an index."""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches
from tests.util import to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gas():
    import paper_2106_05609_amd as g
    g.lib()
    return g


def _batch(cfg_id, scale, n_batches=None):
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    return batches.batch_subgraph(g, bl[0], cfg.self_loops)


def _same_plan(gas, ptr, ind, nnz, n_rows, max_F, options):
    dev_plan = gas.gas_plan_create(ptr, nnz, max_F, n_rows=n_rows, ind=ind, options=options)
    host_plan = gas.gas_plan_create(ptr, nnz, max_F, n_rows=n_rows, ind=ind, options=dict(options or {}, host_builder=1))
    a, b = dev_plan.describe(), host_plan.describe()
    assert a == b, (a, b)
    for x, y, name in zip(dev_plan.lists(), host_plan.lists(), ("group", "heavy", "chunk")):
        assert np.array_equal(x, y), (name, options, int(np.flatnonzero(x != y)[0]) if x.shape == y.shape else (x.shape, y.shape))
    return a


OPTIONS = [None, dict(heavy_threshold=8, chunk=32), dict(heavy_threshold=64, chunk=64, window_rows=32, min_chunk=1),
           dict(heavy_threshold=1, chunk=16, window_rows=1, min_chunk=2), dict(window_rows=-1, heavy_threshold=100),
           dict(xcd_ranges=1), dict(xcd_ranges=2, heavy_threshold=300, window_rows=1 << 20)]


@pytest.mark.parametrize("cfg_id,scale", [(0, 1.0), (1, 0.1), (2, 0.01), (4, 0.0005), (2, 0.05)])
def test_device_plan_equals_host_plan(gas, cfg_id, scale):
    sg = _batch(cfg_id, scale)
    d = lambda t: t.to("cuda")
    ptr, col, n_id = d(sg.rowptr), d(sg.col), d(sg.n_id)
    src = torch.empty_like(col)
    gas.gas_fuse_sources(col, sg.nb, n_id, src)
    nnz_t = int(sg.colptr[sg.nb])
    seen_heavy = 0
    for opt in OPTIONS:
        info = _same_plan(gas, ptr, col, sg.nnz, sg.nb, 256, opt)                       # local column ids
        seen_heavy += info["n_heavy"]
        _same_plan(gas, ptr, src, sg.nnz, sg.nb, 64, opt)                               # fused sources (negative = history row)
        _same_plan(gas, ptr, None, sg.nnz, sg.nb, 256, opt)                             # no indices: no windows, no vote
        _same_plan(gas, d(sg.colptr)[: sg.nb + 1], d(sg.row), nnz_t, sg.nb, 256, opt)   # the CSC copy, in-batch columns
    assert seen_heavy > 0


def test_device_plan_edge_cases(gas):
    z = lambda *a: torch.tensor(a, dtype=torch.int32, device="cuda")
    _same_plan(gas, z(0), None, 0, 0, 8, None)                                           # no rows
    _same_plan(gas, z(0, 0, 0, 0), z(), 0, 3, 8, None)                                   # empty rows only
    # 5000 rows of one entry: groups close at 63 rows and at the 1024-row blocks; 1025 and 2049 rows: block edges
    for n in (5000, 1024, 1025, 2049, 63, 64):
        ptr = torch.arange(n + 1, dtype=torch.int32, device="cuda")
        ind = torch.arange(n, dtype=torch.int32, device="cuda")
        info = _same_plan(gas, ptr, ind, n, n, 8, None)
        assert info["n_groups"] >= -(-n // 63)
    # rows of exactly 64, 65, 512, 513 and 20,000 entries
    for length in (64, 65, 512, 513, 20000):
        ptr = z(0, 0, length, length, 2 * length, 2 * length + 1)
        ind = torch.cat([torch.arange(length, dtype=torch.int32) * 3] * 2 + [torch.tensor([7], dtype=torch.int32)]).cuda()
        info = _same_plan(gas, ptr, ind, 2 * length + 1, 5, 256, None)
        assert (info["n_heavy"] == 2) == (length > 512)


def test_malformed_row_pointers_are_rejected_on_the_device(gas):
    z = lambda *a: torch.tensor(a, dtype=torch.int32, device="cuda")
    ind = torch.zeros(600, dtype=torch.int32, device="cuda")
    for ptr, nnz in ((z(0, 1000, 600), 600), (z(0, 5, 3, 8), 8), (z(1, 5, 8), 8), (z(0, 5, 8), 9), (z(0, -5, 8), 8)):
        for host in (0, 1):
            with pytest.raises(gas.GasError) as e:
                gas.gas_plan_create(ptr, nnz, 16, ind=ind, options=dict(host_builder=host))
            assert e.value.status == -1


def test_both_builders_give_the_same_aggregation_bits(gas):
    from gas_inputs import rng
    sg = _batch(2, 0.02)
    d = lambda t: t.to("cuda")
    x = d(rng.normal_matrix(3, 77, sg.nv, 256))
    out = []
    for host in (0, 1):
        plan = gas.gas_plan_create(d(sg.rowptr), sg.nnz, 256, ind=d(sg.col), options=dict(host_builder=host, heavy_threshold=64))
        zt = torch.full((sg.nb, 256), float("nan"), device="cuda")
        gas.gas_spmm(plan, d(sg.rowptr), d(sg.col), None, x, zt)
        out.append(to_np(zt))
    assert np.array_equal(out[0].view(np.uint8), out[1].view(np.uint8))
