"""History tables on disk, device side: gas_disk_pull / gas_disk_push move the same rows as gas_pull / gas_push on
a table in HBM, bit for bit, in any piece size; a table runs its transfers in the order queued and after the
stream work queued before them; the executor with tables on disk gives the bits of the executor with tables in
HBM and the oracle's values within tolerance."""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches
from oracle import model as omodel
from oracle import ops as oops
from tests.util import to_np, node_rel_err, oracle_model
from tests.test_gpu_gas import _gpu_model, _gpu_batch, TOL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n_rows,width,staging,calls", [(3000, 64, 0, False), (20000, 256, 64 << 10, False),
                                                        (20000, 256, 64 << 10, True), (5000, 100, 1000, False),
                                                        (777, 7, 28, True)])
def test_pull_and_push_match_the_table_in_hbm(tmp_path, dtype, n_rows, width, staging, calls):
    import paper_2106_05609_amd as gas
    g = torch.Generator().manual_seed(n_rows)
    init = torch.randn(n_rows, width, generator=g).to(dtype)
    hbm = init.to("cuda")
    disk = gas.DiskTable(str(tmp_path / "h.bin"), n_rows, width, dtype, create=True, io_threads=4, staging_bytes=staging,
                         calls=calls)
    disk.write_rows(init)
    for trial in range(3):
        # push: distinct rows (a run of consecutive ones among scattered ones), source rows inside a wider tensor
        perm = torch.randperm(n_rows, generator=g)
        start = int(perm[0]) // 2
        run = torch.arange(start, start + n_rows // 4)
        rest = perm[~torch.isin(perm, run)][: n_rows // 3]
        idx = torch.cat([rest[:50], run, rest[50:]]).to(torch.int32)
        wide = torch.randn(len(idx), width + 24, generator=g).to(dtype).to("cuda")
        src = wide[:, 8: 8 + width]
        gas.gas_push(src, idx.to("cuda"), hbm)
        ticket = disk.push(src, idx)
        # pull, queued behind the push: duplicates, any order, into a wider tensor
        pidx = torch.randint(0, n_rows, (n_rows // 2,), generator=g).to(torch.int32)
        a = torch.zeros(len(pidx), width + 8, dtype=dtype, device="cuda")
        b = torch.zeros_like(a)
        gas.gas_pull(hbm, pidx.to("cuda"), a[:, :width])
        t2 = disk.pull(pidx, b[:, :width])
        assert t2 > ticket
        disk.wait(t2)
        assert torch.equal(a, b)
        assert np.array_equal(to_np(b[:, :width]), oops.pull(to_np(hbm), pidx.numpy()))
    # range forms and an empty transfer
    a = torch.empty(n_rows // 2, width, dtype=dtype, device="cuda")
    disk.wait(disk.pull(None, a, base=n_rows // 4))
    assert torch.equal(a, hbm[n_rows // 4: n_rows // 4 + n_rows // 2])
    disk.wait(disk.push(a[:10], None, base=0))
    disk.wait(disk.pull(torch.zeros(0, dtype=torch.int32), a[:0]))
    hbm[:10] = a[:10]
    back = torch.empty(n_rows, width, dtype=dtype)
    disk.read_rows(back)
    assert torch.equal(back, hbm.cpu())
    disk.close()


def test_transfers_wait_for_the_stream_and_keep_their_order(tmp_path):
    """A push reads its source after the kernels queued before it; pushes and pulls of one table run in the order
    queued, so the last value pushed is the one a later pull returns."""
    import paper_2106_05609_amd as gas
    n, width = 8000, 128
    disk = gas.DiskTable(str(tmp_path / "h.bin"), n, width, torch.float32, create=True, staging_bytes=1 << 20)
    idx = torch.randperm(n)[: n // 2].to(torch.int32)
    idx_dev = idx.to("cuda")
    table = torch.zeros(n, width, device="cuda")
    src = torch.zeros(len(idx), width, device="cuda")
    out = [torch.empty_like(src) for _ in range(4)]
    big = torch.randn(4096, 4096, device="cuda")
    tickets = []
    for k in range(4):
        for _ in range(3):
            big = big @ big * 1e-2                    # work in front of the kernel that produces the source
        gas.gas_axpy(src, big[: len(idx), :width], src, alpha=1.0)
        gas.gas_push(src, idx_dev, table)
        keep = src.clone()
        disk.push(keep, idx)
        tickets.append((disk.pull(idx, out[k]), keep))
    for k, (t, keep) in enumerate(tickets):
        disk.wait(t)
        assert torch.equal(out[k], keep), k
    back = torch.empty(n, width)
    disk.read_rows(back)
    assert torch.equal(back, table.cpu())
    disk.close()


def test_errors_are_reported_before_anything_is_queued(tmp_path):
    import paper_2106_05609_amd as gas
    disk = gas.DiskTable(str(tmp_path / "h.bin"), 100, 8, torch.float32, create=True)
    rows = torch.zeros(4, 8, device="cuda")
    with pytest.raises(gas.GasError) as e:
        disk.pull(torch.tensor([1, 2, 100, 3], dtype=torch.int32), rows)
    assert e.value.status == -4
    with pytest.raises(gas.GasError) as e:
        disk.push(rows, None, base=97)
    assert e.value.status == -4
    with pytest.raises(ValueError):
        disk.pull(torch.tensor([1, 2, 3, 4], dtype=torch.int32), rows.cpu())
    disk.wait()
    disk.close()


@pytest.mark.parametrize("cfg_id,scale", [(0, 1.0), (1, 0.1), (4, 0.001), (3, 0.1)])
def test_executor_with_histories_on_disk(tmp_path, cfg_id, scale):
    """Two sweeps over the batches: outputs and tables equal, bit for bit, those of the run with the tables in
    device memory; the first batches are also compared with the oracle."""
    from paper_2106_05609_amd import executor
    import paper_2106_05609_amd as gas
    cfg0 = configs.config(cfg_id, scale)
    if cfg0.op == "gcnii":
        cfg0.widths = cfg0.widths[:6]
    wl = configs.build_workload(cfg0)
    cfg, g = wl.cfg, wl.graph
    init = [h for h in configs.make_histories(cfg, init="normal")]
    hs_cpu = [to_np(h).copy() for h in init]
    hs_dev = [h.to("cuda") for h in init]
    tables = []
    for l, h in enumerate(init):
        t = gas.DiskTable(str(tmp_path / f"hist{l}.bin"), h.shape[0], h.shape[1], h.dtype, create=True,
                          staging_bytes=256 << 10)
        t.write_rows(h)
        tables.append(t)
    om, gm = oracle_model(wl), _gpu_model(wl)
    x_dev, deg_dev = wl.x.to("cuda"), g.deg.to("cuda")
    pipe = executor.DiskPipeline()
    order = list(range(min(4, len(wl.batches)))) * 2
    bgs = {}
    for k, b in enumerate(order):
        if b not in bgs:
            sg = batches.batch_subgraph(g, wl.batches[b], cfg.self_loops)
            bgs[b] = (sg, _gpu_batch(wl, sg, deg_dev))
        sg, bg = bgs[b]
        y_dev = executor.forward_batch(gm, bg, x_dev, hs_dev)
        y_disk = executor.forward_batch_disk(gm, bg, x_dev, tables, pipe)
        assert torch.equal(y_dev, y_disk), (k, b)
        if k < 2:
            y_cpu = omodel.gas_batch_forward(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(g.deg),
                                             to_np(wl.x), hs_cpu)
            assert node_rel_err(to_np(y_disk), y_cpu) <= TOL[cfg.dtype]
    pipe.join()
    torch.cuda.synchronize()
    for a, t in zip(hs_dev, tables):
        back = torch.empty(a.shape, dtype=a.dtype)
        t.read_rows(back)
        assert torch.equal(a.cpu(), back)
        t.close()
