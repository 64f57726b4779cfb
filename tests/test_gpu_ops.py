"""GPU parity of every C-ABI call against the CPU oracle, element by element,
on the same seeded inputs.  Pull, push, the GCN coefficients and index work
are bit-exact; aggregation and transform are within 1e-5 (fp32) or 2e-2 (bf16
storage) of the oracle, measured as max|a-b| / max|b| per output tensor."""
import os

import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, rng
from oracle import ops as oops
from tests.util import to_np, node_rel_err

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


@pytest.fixture(scope="module")
def gas():
    import paper_2106_05609_amd as g
    g.lib()
    return g


def dev(t):
    return t.to("cuda")


# ------------------------------------------------------------------ pull / push
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("F,ld", [(256, 256), (64, 64), (100, 100), (128, 160), (7, 7), (1, 1), (520, 520), (2048, 2048)])
def test_pull_push_bit_exact(gas, dtype, F, ld):
    n_hist, n = 5003, 1237                                  # ragged against every tile size
    table = rng.normal_matrix(1, 300, n_hist, ld, dtype=dtype)
    hist = dev(table)[:, :F]
    idx = rng.randint(1, 301, torch.arange(n), n_hist).to(torch.int32)
    dst_full = torch.full((n, ld), -7.0, dtype=dtype, device="cuda")
    dst = dst_full[:, :F]
    gas.gas_pull(hist, dev(idx), dst)
    want = oops.pull(to_np(table)[:, :F], to_np(idx))
    assert np.array_equal(to_np(dst), want)
    if ld > F:
        assert (dst_full[:, F:] == -7.0).all()              # padding untouched
    # push distinct rows back into a fresh table
    uniq = rng.permutation(1, 302, n_hist)[:n].to(torch.int32)
    src = rng.normal_matrix(1, 303, n, F, dtype=dtype)
    hist2 = dev(table.clone())
    gas.gas_push(dev(src), dev(uniq), hist2[:, :F])
    ref = to_np(table).copy()
    oops.push(to_np(src), to_np(uniq), ref[:, :F])
    assert np.array_equal(to_np(hist2), ref)
    # contiguous-range forms
    dst2 = torch.empty((100, F), dtype=dtype, device="cuda")
    gas.gas_pull(hist, None, dst2, base=4900, n=100)
    assert np.array_equal(to_np(dst2), to_np(table)[4900:5000, :F])
    gas.gas_push(dst2, None, hist2[:, :F], base=3, n=100)
    assert np.array_equal(to_np(hist2)[3:103, :F], to_np(table)[4900:5000, :F])


def test_pull_push_empty_and_errors(gas):
    hist = torch.zeros((10, 8), device="cuda")
    dst = torch.zeros((0, 8), device="cuda")
    gas.gas_pull(hist, torch.zeros(0, dtype=torch.int32, device="cuda"), dst)
    gas.gas_push(dst, torch.zeros(0, dtype=torch.int32, device="cuda"), hist)
    with pytest.raises(gas.GasError):
        gas.gas_pull(hist, None, torch.zeros((4, 8), device="cuda"), base=8, n=4)     # range leaves the table
    assert gas.gas_validate_indices(torch.tensor([0, 9, 3], dtype=torch.int32, device="cuda"), 10)
    assert not gas.gas_validate_indices(torch.tensor([0, 10, 3], dtype=torch.int32, device="cuda"), 10)
    assert not gas.gas_validate_indices(torch.tensor([-1], dtype=torch.int32, device="cuda"), 10)


# ------------------------------------------------------------------ batch subgraphs
def _batch(cfg_id, scale, batch=0, self_loops=None):
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[batch], cfg.self_loops if self_loops is None else self_loops)
    return cfg, g, sg


@pytest.fixture(scope="module")
def graphs_small():
    return {"sbm": _batch(0, 1.0, 1), "powerlaw": _batch(2, 0.01), "gin": _batch(4, 0.0005)}


def test_gcn_norm_bit_exact(gas, graphs_small):
    for name in ("sbm", "powerlaw"):
        cfg, g, sg = graphs_small[name]
        val = torch.empty(sg.nnz, dtype=torch.float32, device="cuda")
        gas.gas_gcn_norm(dev(sg.rowptr), dev(sg.col), dev(sg.n_id), dev(g.deg), val)
        want = oops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id), to_np(g.deg))
        assert np.array_equal(to_np(val), want)
        val_t = torch.empty(sg.nnz, dtype=torch.float32, device="cuda")
        gas.gas_gcn_norm(dev(sg.colptr), dev(sg.row), dev(sg.n_id), dev(g.deg), val_t)
        assert np.array_equal(to_np(val_t), want[to_np(sg.csc_perm)])


def _spmm_case(gas, g, sg, F, dtype, use_val, diag=0.0, s_agg=1.0, res=False, ld_pad=0, out_dtype=None, options=None):
    x = rng.normal_matrix(2, 310, sg.nv, F + ld_pad, dtype=dtype)
    r = rng.normal_matrix(2, 311, sg.nb, F + ld_pad, dtype=dtype) if res else None
    val = oops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id), to_np(g.deg)) if use_val else None
    out_dtype = out_dtype or dtype
    z = torch.full((sg.nb, F + ld_pad), float("nan"), dtype=out_dtype, device="cuda")
    plan = gas.gas_plan_create(dev(sg.rowptr), sg.nnz, F, ind=dev(sg.col), options=options)
    dval = None if val is None else dev(torch.from_numpy(val))
    xd, rd = dev(x), None if r is None else dev(r)
    args = (plan, dev(sg.rowptr), dev(sg.col), dval, xd[:, :F], z[:, :F])
    kw = dict(diag=diag, s_agg=s_agg, r=None if rd is None else rd[:, :F], s_res=0.3 if res else 0.0)
    gas.gas_spmm(*args, **kw)
    want = oops.spmm(to_np(sg.rowptr), to_np(sg.col), val, to_np(x)[:, :F], diag=diag, s_agg=s_agg,
                     r=None if r is None else to_np(r)[:, :F], s_res=0.3 if res else 0.0,
                     out_dt=oops.F32 if out_dtype == torch.float32 else oops.BF16)
    got = to_np(z[:, :F])
    err = node_rel_err(got, want)
    # run-to-run determinism: no atomics, fixed order
    z2 = torch.full_like(z, float("nan"))
    gas.gas_spmm(plan, *args[1:4], xd[:, :F], z2[:, :F], **kw)
    assert np.array_equal(to_np(z2[:, :F]).view(np.uint8), got.view(np.uint8))
    return err


@pytest.mark.parametrize("F", [64, 100, 128, 256, 512, 12, 1024, 7, 1436, 2050])      # the last two: rows above 4096 bytes
def test_spmm_fp32_gcn(gas, graphs_small, F):
    for name in ("sbm", "powerlaw"):
        cfg, g, sg = graphs_small[name]
        assert _spmm_case(gas, g, sg, F, torch.float32, True) <= TOL[torch.float32], (name, F)


@pytest.mark.parametrize("F", [128, 256, 64, 8, 520, 9, 2056])
def test_spmm_bf16_gin(gas, graphs_small, F):
    cfg, g, sg = graphs_small["gin"]
    assert _spmm_case(gas, g, sg, F, torch.bfloat16, False, diag=1.0) <= TOL[torch.bfloat16]
    assert _spmm_case(gas, g, sg, F, torch.bfloat16, False, diag=1.1, out_dtype=torch.float32) <= 1e-5


def test_spmm_epilogues_padding_and_heavy_rows(gas, graphs_small):
    cfg, g, sg = graphs_small["powerlaw"]
    deg = np.diff(to_np(sg.rowptr))
    assert deg.max() > 512 and deg.min() < 32          # both the chunked and the one-wavefront path run
    assert _spmm_case(gas, g, sg, 256, torch.float32, True, s_agg=0.9, res=True, ld_pad=8) <= 1e-5
    assert _spmm_case(gas, g, sg, 64, torch.float32, False, diag=1.25) <= 1e-5
    # tiny thresholds: almost every row is cut into many chunks
    tiny = dict(heavy_threshold=8, chunk=32)
    assert _spmm_case(gas, g, sg, 256, torch.float32, True, s_agg=0.9, res=True, options=tiny) <= 1e-5
    assert _spmm_case(gas, g, sg, 128, torch.bfloat16, True, diag=0.5, options=tiny) <= 2e-2
    assert _spmm_case(gas, g, sg, 20, torch.float32, True, options=tiny) <= 1e-5
    # heavy rows cut at window boundaries (windows of 512, 32 and 2^20 rows, chunks that may shrink to one entry
    # or must hold 16) and processed window by window, each XCD its own range; and no windows at all
    for window, min_chunk in ((512, 1), (32, 16), (1 << 20, 8), (-1, 8)):
        opt = dict(heavy_threshold=64, chunk=64, window_rows=window, min_chunk=min_chunk)
        assert _spmm_case(gas, g, sg, 256, torch.float32, True, s_agg=0.9, res=True, options=opt) <= 1e-5
        assert _spmm_case(gas, g, sg, 256, torch.bfloat16, False, diag=1.0, options=opt) <= 2e-2
        assert _spmm_case(gas, g, sg, 100, torch.float32, True, options=opt) <= 1e-5


def test_spmm_empty_rows_and_empty_matrix(gas):
    ptr = torch.tensor([0, 0, 2, 2, 5], dtype=torch.int32, device="cuda")
    col = torch.tensor([0, 2, 1, 3, 4], dtype=torch.int32, device="cuda")
    x = torch.arange(20, dtype=torch.float32, device="cuda").view(5, 4)
    z = torch.full((4, 4), float("nan"), device="cuda")
    plan = gas.gas_plan_create(ptr, 5, 4)
    gas.gas_spmm(plan, ptr, col, None, x, z)
    want = oops.spmm(to_np(ptr), to_np(col), None, to_np(x))
    assert np.array_equal(to_np(z), want) and (want[0] == 0).all()
    gas.gas_spmm(plan, ptr, col, None, x, z, diag=2.0)
    assert np.array_equal(to_np(z), oops.spmm(to_np(ptr), to_np(col), None, to_np(x), diag=2.0))
    empty = gas.gas_plan_create(torch.zeros(1, dtype=torch.int32, device="cuda"), 0, 4)
    gas.gas_spmm(empty, ptr, col, None, x, z[:0])
    with pytest.raises(gas.GasError):
        gas.gas_plan_create(ptr, 4, 4)                   # nnz does not match ptr


@pytest.mark.parametrize("dtype,F", [(torch.float32, 256), (torch.float32, 100), (torch.bfloat16, 256), (torch.float32, 6),
                                     (torch.float32, 1028)])
def test_spmm_t_parity(gas, graphs_small, dtype, F):
    for name in ("sbm", "powerlaw"):
        cfg, g, sg = graphs_small[name]
        val = oops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id), to_np(g.deg))
        val_t = torch.from_numpy(val[to_np(sg.csc_perm)])
        gz = rng.normal_matrix(3, 320, sg.nb, F, dtype=dtype)
        for n_out in (sg.nb, sg.nv):
            nnz_out = int(sg.colptr[n_out])
            plan = gas.gas_plan_create(dev(sg.colptr[: n_out + 1]), nnz_out, F, n_rows=n_out)
            gx = torch.full((n_out, F), float("nan"), dtype=dtype, device="cuda")
            gas.gas_spmm_t(plan, dev(sg.colptr), dev(sg.row), dev(val_t), dev(gz), gx, diag=0.75)
            want = oops.spmm_t(to_np(sg.rowptr), to_np(sg.col), val, to_np(gz), n_out, diag=0.75)
            assert node_rel_err(to_np(gx), want) <= TOL[dtype], (name, n_out)


# ------------------------------------------------------------------ dense transform
@pytest.mark.parametrize("M,K,N", [(1000, 256, 256), (37, 64, 64), (4097, 100, 256), (513, 128, 64),
                                    (300, 15, 20), (129, 256, 130), (64, 8, 8)])
def test_linear_fp32_parity(gas, M, K, N):
    z = rng.normal_matrix(4, 330, M, K)
    w = rng.glorot_uniform(4, 331, K, N)
    b = rng.normal(4, 332, 0, N)
    for kw in (dict(), dict(relu=True), dict(bias=b, relu=True)):
        y = torch.full((M, N), float("nan"), device="cuda")
        gas.gas_linear(dev(z), dev(w), y, bias=None if "bias" not in kw else dev(b), relu=kw.get("relu", False))
        want = oops.linear(to_np(z), to_np(w), bias=None if "bias" not in kw else to_np(b), relu=kw.get("relu", False))
        assert node_rel_err(to_np(y), want) <= 1e-5, (M, K, N, kw)
    if K == N:
        y = torch.full((M, N), float("nan"), device="cuda")
        gas.gas_linear(dev(z), dev(w), y, c_identity=0.6, c_weight=0.4, relu=True)
        want = oops.linear(to_np(z), to_np(w), c_identity=0.6, c_weight=0.4, relu=True)
        assert node_rel_err(to_np(y), want) <= 1e-5


def test_linear_strided_rows(gas):
    zbuf = rng.normal_matrix(4, 333, 700, 300)
    w = rng.glorot_uniform(4, 334, 256, 64)
    ybuf = torch.full((900, 64), float("nan"), device="cuda")
    gas.gas_linear(dev(zbuf)[:, :256], dev(w), ybuf[:700])
    want = oops.linear(to_np(zbuf)[:, :256], to_np(w))
    assert node_rel_err(to_np(ybuf[:700]), want) <= 1e-5 and torch.isnan(ybuf[700:]).all()


@pytest.mark.parametrize("M,K,N", [(1000, 256, 256), (4097, 128, 256), (300, 64, 64), (129, 256, 128), (257, 72, 200),
                                    (100, 15, 20), (64, 8, 8), (5001, 256, 256), (4500, 64, 200), (4100, 128, 128),
                                    (9000, 40, 24)])
def test_linear_bf16_parity(gas, M, K, N):
    z = rng.normal_matrix(5, 340, M, K, dtype=torch.bfloat16)
    w = rng.glorot_uniform(5, 341, K, N, dtype=torch.bfloat16)
    b = rng.normal(5, 342, 0, N, dtype=torch.bfloat16)
    for kw in (dict(), dict(bias=b, relu=True)):
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        gas.gas_linear(dev(z), dev(w), y, bias=None if "bias" not in kw else dev(b), relu=kw.get("relu", False))
        want = oops.linear(to_np(z), to_np(w), bias=None if "bias" not in kw else to_np(b), relu=kw.get("relu", False))
        assert node_rel_err(to_np(y), want) <= 2e-2, (M, K, N, kw)
    if K == N:
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        gas.gas_linear(dev(z), dev(w), y, c_identity=0.6, c_weight=0.4, relu=True)
        want = oops.linear(to_np(z), to_np(w), c_identity=0.6, c_weight=0.4, relu=True)
        assert node_rel_err(to_np(y), want) <= 2e-2


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,K,H,N", [(1000, 256, 256, 256), (4099, 128, 256, 256), (77, 64, 96, 40), (130, 24, 256, 264),
                                      (50, 10, 17, 6), (6001, 256, 256, 256), (5000, 200, 136, 72)])
def test_mlp2_parity(gas, dtype, M, K, H, N):
    z = rng.normal_matrix(6, 350, M, K, dtype=dtype)
    w1 = rng.glorot_uniform(6, 351, K, H, dtype=dtype)
    w2 = rng.glorot_uniform(6, 352, H, N, dtype=dtype)
    b1 = rng.normal(6, 353, 0, H, dtype=dtype)
    b2 = rng.normal(6, 354, 0, N, dtype=dtype)
    for bias, relu_out in ((False, False), (True, True)):
        y = torch.full((M, N), float("nan"), dtype=dtype, device="cuda")
        gas.gas_mlp2(dev(z), dev(w1), dev(w2), y, b1=dev(b1) if bias else None, b2=dev(b2) if bias else None,
                     relu_out=relu_out)
        want = oops.mlp2(to_np(z), to_np(w1), to_np(w2), b1=to_np(b1) if bias else None,
                         b2=to_np(b2) if bias else None, relu_out=relu_out)
        assert node_rel_err(to_np(y), want) <= TOL[dtype], (dtype, M, K, H, N, bias)
    with pytest.raises(gas.GasError):
        gas.gas_mlp2(dev(z), dev(rng.glorot_uniform(6, 355, K, 300, dtype=dtype)),
                     dev(rng.glorot_uniform(6, 356, 300, N, dtype=dtype)), y)      # hidden width above the limit


@pytest.mark.parametrize("name,dtype,F", [("powerlaw", torch.float32, 256), ("sbm", torch.float32, 100),
                                           ("gin", torch.bfloat16, 256), ("powerlaw", torch.float32, 12),
                                           ("sbm", torch.float32, 1100), ("gin", torch.bfloat16, 2056)])   # rows above 4096 B
def test_spmm_hist_equals_pull_then_spmm(gas, graphs_small, name, dtype, F):
    cfg, g, sg = graphs_small[name]
    use_val = name != "gin"
    nb, nv = sg.nb, sg.nv
    hist = rng.normal_matrix(7, 360, g.n, F, dtype=dtype)
    xb = rng.normal_matrix(7, 361, nb, F, dtype=dtype)
    val = oops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id), to_np(g.deg)) if use_val else None
    dval = None if val is None else dev(torch.from_numpy(val))
    diag = 0.0 if use_val else 1.1
    d_hist, d_xb, d_nid, d_ptr, d_col = dev(hist), dev(xb), dev(sg.n_id), dev(sg.rowptr), dev(sg.col)
    plan = gas.gas_plan_create(d_ptr, sg.nnz, F)
    # unfused: pull the halo rows, then aggregate
    x = torch.empty((nv, F), dtype=dtype, device="cuda")
    x[:nb] = d_xb
    gas.gas_pull(d_hist, d_nid[nb:], x[nb:])
    z_ref = torch.full((nb, F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_spmm(plan, d_ptr, d_col, dval, x, z_ref, diag=diag)
    # fused
    src = torch.empty_like(d_col)
    gas.gas_fuse_sources(d_col, nb, d_nid, src)
    col_np, nid_np = to_np(sg.col), to_np(sg.n_id)
    assert np.array_equal(to_np(src), np.where(col_np < nb, col_np, -1 - nid_np[col_np]))
    z = torch.full((nb, F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_spmm_hist(plan, d_ptr, src, dval, d_xb, d_hist, z, diag=diag)
    assert np.array_equal(to_np(z).view(np.uint8), to_np(z_ref).view(np.uint8))     # same sum, same order
    # and against the oracle's pull + aggregation
    xo = np.concatenate([to_np(xb), oops.pull(to_np(hist), nid_np[nb:])])
    want = oops.spmm(to_np(sg.rowptr), col_np, val, xo, diag=diag)
    assert node_rel_err(to_np(z), want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,K,H,N,push", [(5000, 256, 256, 256, True), (4100, 128, 256, 64, False), (4097, 256, 200, 256, True),
                                          (300, 64, 96, 40, True), (0, 32, 32, 32, False)])
def test_mlp_that_keeps_its_hidden_activation(gas, dtype, M, K, H, N, push):
    """gas_mlp2_keep: the GIN update of a training pass, hidden activation stored (from LDS where the fused kernel
    runs, by two stored linears elsewhere), output pushed; against the oracle's two linears and its push."""
    n_hist = 2 * M + 7
    z = rng.normal_matrix(11, 400, M, K, dtype=dtype)
    w1 = rng.glorot_uniform(11, 401, K, H, dtype=dtype)
    w2 = rng.glorot_uniform(11, 402, H, N, dtype=dtype)
    b1 = rng.normal(11, 403, 0, H, dtype=dtype)
    idx = rng.permutation(11, 404, n_hist)[:M].to(torch.int32)
    table0 = rng.normal_matrix(11, 405, n_hist, N, dtype=dtype)
    y = torch.full((M, N), float("nan"), dtype=dtype, device="cuda")
    h = torch.full((M, H), float("nan"), dtype=dtype, device="cuda")
    table = dev(table0).clone()
    gas.gas_mlp2_keep(dev(z), dev(w1), dev(w2), y, h, idx=dev(idx) if push else None, hist=table if push else None,
                      b1=dev(b1), relu_out=True)
    if M == 0:
        return
    dt = oops.F32 if dtype == torch.float32 else oops.BF16
    want_h = oops.linear(to_np(z), to_np(w1), bias=to_np(b1), relu=True, out_dt=dt)
    assert node_rel_err(to_np(h), want_h) <= TOL[dtype]
    # the second product on the hidden activation the library stored (a unit within rounding of zero may fall on
    # either side of the ReLU in two correct passes)
    want_y = oops.linear(to_np(h), to_np(w2), relu=True, out_dt=dt)
    assert node_rel_err(to_np(y), want_y) <= TOL[dtype]
    want_table = to_np(table0).copy()
    if push:
        oops.push(to_np(y), to_np(idx), want_table)
    assert np.array_equal(to_np(table).view(np.uint8), want_table.view(np.uint8))
    # and the plain fused call gives the same output bits where the same kernel runs
    if dtype == torch.bfloat16 and M >= 4096:
        y2 = torch.empty_like(y)
        gas.gas_mlp2(dev(z), dev(w1), dev(w2), y2, b1=dev(b1), relu_out=True)
        assert torch.equal(y, y2)


@pytest.mark.parametrize("name", ["sbm", "powerlaw"])
def test_spmm_xcd_ranges_give_the_same_bits(gas, graphs_small, name):
    """Handing the light rows to the XCDs in contiguous ranges changes which workgroup does a row, not the sum."""
    cfg, g, sg = graphs_small[name]
    F = 256
    x = dev(rng.normal_matrix(10, 390, sg.nv, F))
    val = dev(torch.from_numpy(oops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id), to_np(g.deg))))
    out = []
    for mode in (2, 1, 0):                             # never, always, decided from the pattern
        plan = gas.gas_plan_create(dev(sg.rowptr), sg.nnz, F, ind=dev(sg.col), options=dict(xcd_ranges=mode))
        z = torch.full((sg.nb, F), float("nan"), device="cuda")
        gas.gas_spmm(plan, dev(sg.rowptr), dev(sg.col), val, x, z)
        out.append(to_np(z))
        gas.gas_plan_destroy(plan)
    assert np.array_equal(out[0].view(np.uint8), out[1].view(np.uint8))
    assert np.array_equal(out[0].view(np.uint8), out[2].view(np.uint8))
    want = oops.spmm(to_np(sg.rowptr), to_np(sg.col), to_np(val), to_np(x))
    assert node_rel_err(out[1], want) <= 1e-5


@pytest.mark.parametrize("name,K,N,variant", [("sbm", 64, 64, "gcnii"), ("sbm", 128, 64, "gcn"), ("powerlaw", 100, 36, "gcn"),
                                               ("powerlaw", 128, 128, "gcnii"), ("gin", 8, 4, "gin"), ("sbm", 64, 64, "plain"),
                                               ("gin", 64, 32, "all_terms")])
def test_layer_in_one_launch_matches_the_oracle(gas, graphs_small, name, K, N, variant):
    """gas_spmm_linear: Eq. (2)'s aggregation with both sources, the transform and the Push in one launch, against
    the oracle's pull + aggregation + transform + push; rows that are not pushed keep their contents."""
    cfg, g, sg = graphs_small[name]
    nb, nv = sg.nb, sg.nv
    ptr_np, col_np, nid_np = to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id)
    hist = rng.normal_matrix(9, 380, g.n, K)
    xb = rng.normal_matrix(9, 381, nb, K)
    w = rng.glorot_uniform(9, 382, K, N)
    bias = rng.normal(9, 383, 0, N) if variant == "gcn" else None
    val = oops.gcn_norm(ptr_np, col_np, nid_np, to_np(g.deg)) if variant != "gin" else None
    kw = dict(diag=1.1) if variant == "gin" else {}
    r = None
    if variant == "gcnii":
        r = rng.normal_matrix(9, 384, nb, K)
        kw.update(s_agg=0.9, s_res=0.1)
    if variant == "all_terms":          # every term of the epilogue at once: the diagonal term is NOT scaled by s_agg
        r = rng.normal_matrix(9, 384, nb, K)
        kw.update(diag=0.75, s_agg=0.6, s_res=0.3)
    lin = dict(c_identity=0.7, c_weight=0.3) if variant == "gcnii" and K == N else {}
    relu = variant != "plain"
    # oracle: pull, aggregate, transform, push
    xo = np.concatenate([to_np(xb), oops.pull(to_np(hist), nid_np[nb:])])
    z = oops.spmm(ptr_np, col_np, val, xo, r=None if r is None else to_np(r), **kw)
    want = oops.linear(z, to_np(w), bias=None if bias is None else to_np(bias), relu=relu, **lin)
    table0 = rng.normal_matrix(9, 385, g.n, N)
    want_table = to_np(table0).copy()
    oops.push(want, nid_np[:nb], want_table)
    # library: one call, halo rows read from the history table in place
    d_ptr, d_col, d_nid = dev(sg.rowptr), dev(sg.col), dev(sg.n_id)
    src = torch.empty_like(d_col)
    gas.gas_fuse_sources(d_col, nb, d_nid, src)
    dval = None if val is None else dev(torch.from_numpy(val))
    y = torch.full((nb, N), float("nan"), device="cuda")
    table = dev(table0).clone()
    gas.gas_spmm_linear(d_ptr, src, dval, dev(xb), dev(w), y, hist=dev(hist), r=None if r is None else dev(r),
                        bias=None if bias is None else dev(bias), relu=relu, push_idx=d_nid[:nb], push_hist=table,
                        **kw, **lin)
    # rows measured against the products summed for them: with N = 4 a ReLU can leave a row whose largest
    # output is a hundredth of its terms
    terms = (np.abs(z.astype(np.float64)) @ np.abs(to_np(w).astype(np.float64))).max(axis=1)
    assert node_rel_err(to_np(y), want, scale=terms) <= 1e-5
    assert np.array_equal(to_np(table)[nid_np[:nb]], to_np(y))
    if variant == "all_terms":
        # the same layer as two calls (gas_spmm_hist, gas_linear) takes the same meaning of diag, s_agg and R
        plan = gas.gas_plan_create(d_ptr, sg.nnz, K, ind=src)
        z2 = torch.full((nb, K), float("nan"), device="cuda")
        gas.gas_spmm_hist(plan, d_ptr, src, dval, dev(xb), dev(hist), z2, r=dev(r), **kw)
        assert node_rel_err(to_np(z2), z) <= 1e-5
        y2 = torch.full((nb, N), float("nan"), device="cuda")
        gas.gas_linear(z2, dev(w), y2, relu=relu)
        assert node_rel_err(to_np(y2), want, scale=terms) <= 1e-5
    keep = np.ones(g.n, dtype=bool)
    keep[nid_np[:nb]] = False
    assert np.array_equal(to_np(table)[keep], want_table[keep])
    # the other form: plain column indices into the whole mini-batch tensor, no history table, no push
    y2 = torch.full((nb, N), float("nan"), device="cuda")
    gas.gas_spmm_linear(d_ptr, d_col, dval, dev(torch.from_numpy(xo)), dev(w), y2, r=None if r is None else dev(r),
                        bias=None if bias is None else dev(bias), relu=relu, **kw, **lin)
    assert np.array_equal(to_np(y2).view(np.uint8), to_np(y).view(np.uint8))       # same sources, same order
    # run to run
    y3 = torch.empty_like(y2)
    gas.gas_spmm_linear(d_ptr, d_col, dval, dev(torch.from_numpy(xo)), dev(w), y3, r=None if r is None else dev(r),
                        bias=None if bias is None else dev(bias), relu=relu, **kw, **lin)
    assert torch.equal(y2, y3)


def test_layer_in_one_launch_limits(gas):
    """Shapes the one-launch layer does not take are refused before anything is launched."""
    ptr = dev(torch.tensor([0, 1, 2], dtype=torch.int32))
    col = dev(torch.tensor([0, 1], dtype=torch.int32))
    for k, n, dtype in [(256, 64, torch.float32), (64, 132, torch.float32), (30, 32, torch.float32),
                        (64, 64, torch.bfloat16)]:
        x = torch.zeros((2, k), dtype=dtype, device="cuda")
        w = torch.zeros((k, n), dtype=dtype, device="cuda")
        y = torch.zeros((2, n), dtype=dtype, device="cuda")
        assert not gas.spmm_linear_supported(x, n)
        with pytest.raises(gas.GasError):
            gas.gas_spmm_linear(ptr, col, None, x, w, y)
    x = torch.zeros((2, 64), device="cuda")
    gas.gas_spmm_linear(ptr[:1], col[:0], None, x[:0], torch.zeros((64, 64), device="cuda"), x[:0].clone())   # empty: no-op


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,K,H,N,ld_hist", [(5000, 256, 256, 256, 256), (4100, 128, 256, 64, 72), (300, 64, 96, 40, 40),
                                             (4097, 256, 256, 256, 260), (0, 32, 32, 32, 32)])
def test_transform_with_fused_push(gas, dtype, M, K, H, N, ld_hist):
    """Algorithm 1's Push taken in the transform's epilogue: same bits as the transform followed by Push, the
    oracle's Push of those rows gives the same table, rows that are not pushed keep their contents."""
    n_hist = 2 * M + 11
    z = dev(rng.normal_matrix(8, 370, M, K, dtype=dtype))
    w1 = dev(rng.glorot_uniform(8, 371, K, H, dtype=dtype))
    w2 = dev(rng.glorot_uniform(8, 372, H, N, dtype=dtype))
    w = dev(rng.glorot_uniform(8, 373, K, N, dtype=dtype))
    b1 = dev(rng.normal(8, 374, 0, H, dtype=dtype))
    b2 = dev(rng.normal(8, 375, 0, N, dtype=dtype))
    idx = dev(rng.permutation(8, 376, n_hist)[:M].to(torch.int32))
    hist0 = rng.normal_matrix(8, 377, n_hist, ld_hist, dtype=dtype)
    for kind in ("linear", "mlp2"):
        y_ref = torch.full((M, N), float("nan"), dtype=dtype, device="cuda")
        y = torch.full((M, N), float("nan"), dtype=dtype, device="cuda")
        hist_ref, hist = dev(hist0.clone()), dev(hist0.clone())
        if kind == "linear":
            gas.gas_linear(z, w, y_ref, bias=b2, relu=True)
            gas.gas_linear_push(z, w, y, idx, hist[:, :N], bias=b2, relu=True)
        else:
            gas.gas_mlp2(z, w1, w2, y_ref, b1=b1, b2=b2, relu_out=True)
            gas.gas_mlp2_push(z, w1, w2, y, idx, hist[:, :N], b1=b1, b2=b2, relu_out=True)
        gas.gas_push(y_ref, idx, hist_ref[:, :N])
        assert np.array_equal(to_np(y).view(np.uint8), to_np(y_ref).view(np.uint8)), kind
        assert np.array_equal(to_np(hist).view(np.uint8), to_np(hist_ref).view(np.uint8)), kind
        want = to_np(hist0.clone())
        if M:
            oops.push(to_np(y), to_np(idx), want[:, :N])
        assert np.array_equal(to_np(hist).view(np.uint8), want.view(np.uint8)), kind
    if M:
        with pytest.raises(gas.GasError):
            gas.gas_linear_push(z, w, y, idx, y, bias=b2)            # the table must not be the output


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("name,F,ld_pad", [("powerlaw", 256, 0), ("gin", 64, 8), ("sbm", 100, 0), ("powerlaw", 7, 0),
                                           ("gin", 520, 0), ("sbm", 8, 0)])
def test_pna_aggregate_parity(gas, graphs_small, dtype, name, F, ld_pad):
    """Scalers x aggregators of PNA (operator appendix) in one pass: every block against the oracle; the
    min and max blocks of a call without the receiving-node term are bit-exact (they select stored values)."""
    cfg, g, sg = graphs_small[name]
    nb, nv = sg.nb, sg.nv
    x = rng.normal_matrix(11, 950, nv, F + ld_pad, dtype=dtype)
    q = rng.normal_matrix(11, 951, nb, F, dtype=dtype)
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    d_ptr, d_col = dev(sg.rowptr), dev(sg.col)
    for add in (None, q):
        out = torch.full((nb, 9 * F + ld_pad), float("nan"), dtype=dtype, device="cuda")
        gas.gas_pna_aggregate(d_ptr, d_col, dev(x)[:, :F], out[:, :9 * F], delta, add=None if add is None else dev(add))
        want = oops.pna_aggregate(to_np(sg.rowptr), to_np(sg.col), to_np(x)[:, :F], delta,
                                  add=None if add is None else to_np(add))
        got = to_np(out[:, :9 * F])
        for j in range(9):
            blk = slice(j * F, (j + 1) * F)
            assert node_rel_err(got[:, blk], want[:, blk]) <= TOL[dtype], (j, node_rel_err(got[:, blk], want[:, blk]))
        if add is None:
            assert np.array_equal(got[:, F:3 * F], want[:, F:3 * F])
    # a row without neighbours gives zeros; an empty problem is fine
    ptr = torch.tensor([0, 0, 2], dtype=torch.int32, device="cuda")
    col = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    out = torch.full((2, 9 * F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_pna_aggregate(ptr, col, dev(x)[:, :F], out, delta)
    assert not to_np(out[0]).any() and not torch.isnan(out.float()).any()
    gas.gas_pna_aggregate(ptr[:1], col[:0], dev(x)[:, :F], out[:0], delta)
    with pytest.raises(gas.GasError):
        gas.gas_pna_aggregate(ptr, col, dev(x)[:, :F], out, 0.0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("name,F,ld_pad", [("powerlaw", 256, 0), ("sbm", 64, 8), ("powerlaw", 100, 0), ("sbm", 7, 0),
                                           ("powerlaw", 520, 0), ("gin", 128, 0), ("sbm", 512, 0), ("powerlaw", 32, 0)])
def test_gat_aggregate_parity(gas, graphs_small, dtype, name, F, ld_pad):
    """GAT's scores, softmax and weighted sum in one pass (operator appendix) against the oracle's three-step form."""
    cfg, g, sg = graphs_small[name]
    nb, nv = sg.nb, sg.nv
    p = rng.normal_matrix(12, 960, nv, F + ld_pad, dtype=dtype)
    a_dst = rng.normal(12, 961, 0, F, dtype=dtype) * 0.3
    a_src = rng.normal(12, 962, 0, F, dtype=dtype) * 0.3
    z = torch.full((nb, F + ld_pad), float("nan"), dtype=dtype, device="cuda")
    gas.gas_gat_aggregate(dev(sg.rowptr), dev(sg.col), dev(p)[:, :F], dev(a_dst), dev(a_src), z[:, :F])
    want = oops.gat_aggregate(to_np(sg.rowptr), to_np(sg.col), to_np(p)[:, :F], to_np(a_dst), to_np(a_src))
    assert node_rel_err(to_np(z[:, :F]), want) <= TOL[dtype], node_rel_err(to_np(z[:, :F]), want)
    # same call again: same bits (entries are folded in index order)
    z2 = torch.full((nb, F + ld_pad), float("nan"), dtype=dtype, device="cuda")
    gas.gas_gat_aggregate(dev(sg.rowptr), dev(sg.col), dev(p)[:, :F], dev(a_dst), dev(a_src), z2[:, :F])
    assert torch.equal(z[:, :F].view(torch.int32 if dtype == torch.float32 else torch.int16),
                       z2[:, :F].view(torch.int32 if dtype == torch.float32 else torch.int16))
    # rows without entries give zeros
    ptr = torch.tensor([0, 0, 2], dtype=torch.int32, device="cuda")
    col = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    out = torch.full((2, F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_gat_aggregate(ptr, col, dev(p)[:, :F], dev(a_dst), dev(a_src), out)
    assert not to_np(out[0]).any() and not torch.isnan(out.float()).any()
    with pytest.raises(gas.GasError):
        gas.gas_gat_aggregate(ptr, col, out, dev(a_dst), dev(a_src), out)


def _pattern_with_long_rows(seed, nv, empty_rows=True):
    """Rows around the length above which a workgroup shares a row (2,048 entries), beside empty ones and rows whose
    lengths sit on either side of what a team of lanes, a wavefront step and a block of 64 entries take."""
    lengths = [0, 1, 3000, 2049, 2048, 5003, 70, 2047, 0, 4096, 9, 2113, 2, 3, 4, 5, 7, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65,
               127, 128, 129, 2050, 2111, 2112]
    if not empty_rows:
        lengths = [n for n in lengths if n > 0]
    gen = np.random.default_rng(seed)
    ptr = np.zeros(len(lengths) + 1, dtype=np.int32)
    ptr[1:] = np.cumsum(lengths)
    col = gen.integers(0, nv, size=int(ptr[-1]), dtype=np.int32)
    return ptr, col


@pytest.mark.parametrize("dtype,F", [(torch.float32, 256), (torch.bfloat16, 256), (torch.bfloat16, 64), (torch.float32, 128),
                                     (torch.float32, 32), (torch.bfloat16, 512)])
def test_pna_and_gat_aggregate_rows_shared_by_a_workgroup(gas, dtype, F):
    """Rows above 2,048 entries are gathered by the eight wavefronts of a workgroup and merged in wavefront order:
    same results as the oracle for every width class (16, 32 and 64 lanes per row), and the same bits twice."""
    nv = 6000
    ptr, col = _pattern_with_long_rows(41, nv)
    nb = ptr.size - 1
    x = rng.normal_matrix(13, 970, nv, F, dtype=dtype)
    q = rng.normal_matrix(13, 971, nb, F, dtype=dtype)
    d_ptr, d_col = dev(torch.from_numpy(ptr)), dev(torch.from_numpy(col))
    out = torch.full((nb, 9 * F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_pna_aggregate(d_ptr, d_col, dev(x), out, 1.3, add=dev(q))
    want = oops.pna_aggregate(ptr, col, to_np(x), 1.3, add=to_np(q))
    got = to_np(out)
    for j in range(9):
        blk = slice(j * F, (j + 1) * F)
        assert node_rel_err(got[:, blk], want[:, blk]) <= TOL[dtype], (j, node_rel_err(got[:, blk], want[:, blk]))
    out2 = torch.full((nb, 9 * F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_pna_aggregate(d_ptr, d_col, dev(x), out2, 1.3)
    assert np.array_equal(to_np(out2)[:, F:3 * F], oops.pna_aggregate(ptr, col, to_np(x), 1.3)[:, F:3 * F])   # min, max: exact
    a_dst = rng.normal(13, 972, 0, F, dtype=dtype) * 0.3
    a_src = rng.normal(13, 973, 0, F, dtype=dtype) * 0.3
    z = [torch.full((nb, F), float("nan"), dtype=dtype, device="cuda") for _ in range(2)]
    for t in z:
        gas.gas_gat_aggregate(d_ptr, d_col, dev(x), dev(a_dst), dev(a_src), t)
    want = oops.gat_aggregate(ptr, col, to_np(x), to_np(a_dst), to_np(a_src))
    assert node_rel_err(to_np(z[0]), want) <= TOL[dtype], node_rel_err(to_np(z[0]), want)
    bits = torch.int32 if dtype == torch.float32 else torch.int16
    assert torch.equal(z[0].view(bits), z[1].view(bits))


def _pna_bwd_row_scale(ptr, col, x, gout, delta, nv, F):
    """Per-row scale of the rounding errors of PNA's backward pass: output row u is a sum of the mean's shares
    c_0[v] / d_v of its entries and of the whole c_1[v, f] / c_2[v, f] of every feature it wins as a row's minimum or
    maximum.  A node with an extreme value wins the same feature in every row that lists it, and those terms (of
    order 10) may cancel to a total of order 0.01; the rounding error is relative to the terms.  Returns, per row,
    the largest over the features of the sum of the terms' magnitudes."""
    x64, g64 = oops.to_f64(x), oops.to_f64(gout)
    mag = np.zeros((nv, F))
    feat = np.arange(F)
    for v in range(ptr.size - 1):
        cols = col[ptr[v]:ptr[v + 1]]
        if cols.size == 0:
            continue
        s = np.log(cols.size + 1.0) / delta
        c = [np.abs(g64[v, j * F:(j + 1) * F] + s * g64[v, (3 + j) * F:(4 + j) * F] + g64[v, (6 + j) * F:(7 + j) * F] / s)
             for j in range(3)]
        np.add.at(mag, cols, c[0] / cols.size)
        xs = x64[cols]
        np.add.at(mag, (cols[xs.argmin(axis=0)], feat), c[1])
        np.add.at(mag, (cols[xs.argmax(axis=0)], feat), c[2])
    return mag.max(axis=1)


@pytest.mark.parametrize("dtype,F", [(torch.float32, 256), (torch.bfloat16, 256), (torch.bfloat16, 64), (torch.float32, 128)])
def test_pna_and_gat_backward_rows_shared_by_a_workgroup(gas, dtype, F):
    """The row passes of the two backward aggregations on rows above 2,048 entries (gathered by the eight wavefronts
    of a workgroup; winners, maxima and sums merged in wavefront order): against the oracle, and the same bits twice."""
    nv = 6000
    ptr, col = _pattern_with_long_rows(43, nv, empty_rows=False)
    nb, nnz = ptr.size - 1, int(ptr[-1])
    order = np.argsort(col, kind="stable")
    rows = np.repeat(np.arange(nb, dtype=np.int32), np.diff(ptr))
    colptr = np.zeros(nv + 1, dtype=np.int32)
    colptr[1:] = np.cumsum(np.bincount(col, minlength=nv))
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda")
    d_ptr, d_col, d_colptr, d_row, d_pos = d(ptr), d(col), d(colptr), d(rows[order]), d(order.astype(np.int32))
    plan_t = gas.gas_plan_create(d_colptr, nnz, F, n_rows=nv, ind=d_row)
    bits = torch.int32 if dtype == torch.float32 else torch.int16
    x = rng.normal_matrix(14, 980, nv, F, dtype=dtype)
    gout = rng.normal_matrix(14, 981, nb, 9 * F, dtype=dtype)
    want_x, want_add = oops.pna_aggregate_bwd(ptr, col, to_np(x), 1.3, to_np(gout), nv)
    res = []
    for _ in range(2):
        gx = torch.full((nv, F), float("nan"), dtype=dtype, device="cuda")
        gadd = torch.full((nb, F), float("nan"), dtype=dtype, device="cuda")
        gas.gas_pna_aggregate_bwd(d_ptr, d_col, d_colptr, d_row, d_pos, x.to("cuda"), gout.to("cuda"), gx, 1.3, gadd=gadd,
                                  plan_t=plan_t)
        res.append(gx)
    terms = _pna_bwd_row_scale(ptr, col, to_np(x), to_np(gout), 1.3, nv, F)
    assert node_rel_err(to_np(res[0]), want_x, scale=terms) <= TOL[dtype], node_rel_err(to_np(res[0]), want_x, scale=terms)
    assert node_rel_err(to_np(gadd), want_add) <= TOL[dtype]
    assert torch.equal(res[0].view(bits), res[1].view(bits))
    p = rng.normal_matrix(14, 982, nv, F, dtype=dtype) * 0.5
    a_dst = rng.normal(14, 983, 0, F, dtype=dtype) * 0.3
    a_src = rng.normal(14, 984, 0, F, dtype=dtype) * 0.3
    gz = rng.normal_matrix(14, 985, nb, F, dtype=dtype)
    want_p, want_d, want_s = oops.gat_aggregate_bwd(ptr, col, to_np(p), to_np(a_dst), to_np(a_src), to_np(gz), nv, 0.2)
    terms = _gat_bwd_row_scale(ptr, col, to_np(p), to_np(a_dst), to_np(a_src), to_np(gz), nb, nv)
    res = []
    for _ in range(2):
        gp = torch.full((nv, F), float("nan"), dtype=dtype, device="cuda")
        gd = torch.full((F,), float("nan"), device="cuda")
        gs = torch.full((F,), float("nan"), device="cuda")
        gas.gas_gat_aggregate_bwd(d_ptr, d_col, d_colptr, d_row, d_pos, p.to("cuda"), a_dst.to("cuda"), a_src.to("cuda"),
                                  gz.to("cuda"), gp, gd, gs, 0.2, plan_t=plan_t)
        res.append(gp)
    assert node_rel_err(to_np(res[0]), want_p, scale=terms) <= TOL[dtype], node_rel_err(to_np(res[0]), want_p, scale=terms)
    scale = max(np.abs(want_d).max(), np.abs(want_s).max())
    assert np.abs(to_np(gd) - want_d).max() <= TOL[dtype] * scale and np.abs(to_np(gs) - want_s).max() <= TOL[dtype] * scale
    assert torch.equal(res[0].view(bits), res[1].view(bits))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_pull_push_with_a_history_table_in_pinned_host_memory(gas, dtype):
    """Histories outside HBM: the row-copy kernel reads and writes a pinned host table through its device-side
    address; same bits as indexing the table on the host."""
    n, F, m = 20000, 256, 7000
    table = rng.normal_matrix(15, 1300, n, F, dtype=dtype).pin_memory()
    ht = gas.HostTable(table)
    idx = rng.permutation(15, 1301, n)[:m].to(torch.int32)
    out = torch.full((m, F), float("nan"), dtype=dtype, device="cuda")
    gas.gas_pull(ht, dev(idx), out)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(out), oops.pull(to_np(table), to_np(idx)))
    fresh = rng.normal_matrix(15, 1302, m, F, dtype=dtype)
    want = to_np(table).copy()
    oops.push(to_np(fresh), to_np(idx), want)
    gas.gas_push(dev(fresh), dev(idx), ht)
    torch.cuda.synchronize()                           # the host reads the table only after the kernel has finished
    assert np.array_equal(to_np(table), want)
    with pytest.raises((gas.GasError, ValueError)):
        gas.HostTable(torch.zeros((4, 4)))              # pageable memory: refused before any kernel sees it


@pytest.mark.parametrize("name,dtype,F", [("sbm", torch.float32, 8), ("powerlaw", torch.float32, 100), ("gin", torch.bfloat16, 128),
                                          ("powerlaw", torch.float32, 7), ("gin", torch.float32, 520),
                                          ("sbm", torch.float32, 256), ("sbm", torch.bfloat16, 512),
                                          ("powerlaw", torch.float32, 256), ("powerlaw", torch.bfloat16, 256)])
def test_pna_aggregate_backward_parity(gas, graphs_small, name, dtype, F):
    """gas_pna_aggregate_bwd against the oracle (itself pinned to float64 autograd): gradient of the gathered rows
    for all columns of the pattern and for the in-batch columns only, gradient of the added term.  The graphs have
    rows of one entry (which then wins every feature: lists longer than a wavefront) and rows above 512 entries
    (items counted and placed in several goes)."""
    cfg, g, sg = graphs_small[name]
    nb, nv = sg.nb, sg.nv
    x = rng.normal_matrix(12, 960, nv, F, dtype=dtype)
    gout = rng.normal_matrix(12, 961, nb, 9 * F, dtype=dtype)
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    d = lambda t: t.to("cuda")
    want_x, want_add = oops.pna_aggregate_bwd(to_np(sg.rowptr), to_np(sg.col), to_np(x), delta, to_np(gout), nv)
    bits = lambda t: t.view(torch.int16 if dtype == torch.bfloat16 else torch.int32)
    for fast in (False, True):
        # fast: with a plan of the CSC copy (rows gathered like the forward call, the mean's share taken by the
        # backward aggregation's kernels, minima and maxima as per-entry item lists); widths it does not take fall
        # back to the plain kernels, which is checked too
        for n_out in (nv, nb):
            plan_t = gas.gas_plan_create(d(sg.colptr)[: n_out + 1], int(sg.colptr[n_out]), F, n_rows=n_out, ind=d(sg.row)) \
                if fast else None
            gx = torch.full((n_out, F), float("nan"), dtype=dtype, device="cuda")
            gadd = torch.full((nb, F), float("nan"), dtype=dtype, device="cuda")
            gas.gas_pna_aggregate_bwd(d(sg.rowptr), d(sg.col), d(sg.colptr)[: n_out + 1], d(sg.row), d(sg.csc_perm).int(),
                                      d(x), d(gout), gx, delta, gadd=gadd, plan_t=plan_t)
            assert node_rel_err(to_np(gx), want_x[:n_out]) <= TOL[dtype], (fast, n_out, node_rel_err(to_np(gx), want_x[:n_out]))
            assert node_rel_err(to_np(gadd), want_add) <= TOL[dtype]
            gx2 = torch.full((n_out, F), float("nan"), dtype=dtype, device="cuda")
            gas.gas_pna_aggregate_bwd(d(sg.rowptr), d(sg.col), d(sg.colptr)[: n_out + 1], d(sg.row), d(sg.csc_perm).int(),
                                      d(x), d(gout), gx2, delta, plan_t=plan_t)
            assert torch.equal(bits(gx2), bits(gx))                                            # fixed order


def _gat_bwd_row_scale(rp, cl, p, a_dst, a_src, gz, nb, nv):
    """Per-row scale of the rounding errors of GAT's backward pass (see test_gat_aggregate_backward_parity): for
    output row u, the sum over its entries of alpha_k ||GZ[v]|| ||P[u]|| max|a_src|, plus for an in-batch row the sum
    over its own row's entries of alpha_k ||GZ[v]|| ||P[col k]|| max|a_dst|."""
    rows = np.repeat(np.arange(nb), np.diff(rp))
    p64 = oops.to_f64(p)
    t = (p64[:nb] @ oops.to_f64(a_dst))[rows] + (p64 @ oops.to_f64(a_src))[cl]
    ex = np.exp(np.where(t > 0, t, 0.2 * t) - np.maximum.reduceat(np.where(t > 0, t, 0.2 * t), rp[:-1])[rows])
    alpha = ex / np.add.reduceat(ex, rp[:-1])[rows]
    assert np.diff(rp).min() > 0                       # no empty rows (reduceat)
    weight = alpha * np.linalg.norm(oops.to_f64(gz), axis=1)[rows] * np.linalg.norm(p64, axis=1)[cl]
    terms = np.bincount(cl, weights=weight, minlength=nv) * np.abs(oops.to_f64(a_src)).max()
    terms[:nb] += np.add.reduceat(weight, rp[:-1]) * np.abs(oops.to_f64(a_dst)).max()
    return terms


@pytest.mark.parametrize("name,dtype,F", [("sbm", torch.float32, 8), ("powerlaw", torch.float32, 100), ("sbm", torch.bfloat16, 128),
                                          ("powerlaw", torch.float32, 7), ("sbm", torch.float32, 520),
                                          ("powerlaw", torch.float32, 256), ("powerlaw", torch.bfloat16, 256),
                                          ("gin", torch.bfloat16, 512)])
def test_gat_aggregate_backward_parity(gas, graphs_small, name, dtype, F):
    """gas_gat_aggregate_bwd against the oracle (pinned to float64 autograd): gradients of P (all rows / in-batch
    rows) and of the two halves of the attention vector."""
    cfg, g, sg = graphs_small[name]
    nb, nv = sg.nb, sg.nv
    p = rng.normal_matrix(12, 970, nv, F, dtype=dtype) * 0.5
    a_dst = rng.normal(12, 971, 0, F, dtype=dtype) * 0.3
    a_src = rng.normal(12, 972, 0, F, dtype=dtype) * 0.3
    gz = rng.normal_matrix(12, 973, nb, F, dtype=dtype)
    d = lambda t: t.to("cuda")
    want_p, want_d, want_s = oops.gat_aggregate_bwd(to_np(sg.rowptr), to_np(sg.col), to_np(p), to_np(a_dst), to_np(a_src),
                                                    to_np(gz), nv, 0.2)
    # Per-row scale of the rounding errors.  The softmax's backward subtracts the row's mean of dalpha from every
    # dalpha_k = GZ[v] . P[col k]; the error of dt_k is relative to the products summed for dalpha_k (at most
    # ||GZ[v]|| ||P[col k]||), not to the difference, and dt_k a_src is a term of output row col k.  So row u is
    # measured against max(its own largest entry, sum over its entries of alpha_k ||GZ[v]|| ||P[u]|| max|a_src|).
    # An in-batch row v also receives (sum_k dt_k) a_dst, a sum over its own row's entries that cancels (it is
    # exactly zero for slope 1): its error is relative to sum_k alpha_k ||GZ[v]|| ||P[col k]|| max|a_dst|.
    terms = _gat_bwd_row_scale(to_np(sg.rowptr), to_np(sg.col), to_np(p), to_np(a_dst), to_np(a_src), to_np(gz), nb, nv)
    for fast in (False, True):
        for n_out in (nv, nb):
            plan_t = gas.gas_plan_create(d(sg.colptr)[: n_out + 1], int(sg.colptr[n_out]), F, n_rows=n_out, ind=d(sg.row)) \
                if fast else None
            gp = torch.full((n_out, F), float("nan"), dtype=dtype, device="cuda")
            gd = torch.full((F,), float("nan"), device="cuda")
            gs = torch.full((F,), float("nan"), device="cuda")
            gas.gas_gat_aggregate_bwd(d(sg.rowptr), d(sg.col), d(sg.colptr), d(sg.row), d(sg.csc_perm).int(), d(p), d(a_dst),
                                      d(a_src), d(gz), gp, gd, gs, 0.2, plan_t=plan_t)
            assert node_rel_err(to_np(gp), want_p[:n_out], scale=terms[:n_out]) <= TOL[dtype], \
                (fast, n_out, node_rel_err(to_np(gp), want_p[:n_out], scale=terms[:n_out]))
            # the two vector gradients are sums over all entries: against the size of the larger of the two
            scale = max(np.abs(want_d).max(), np.abs(want_s).max())
            assert np.abs(to_np(gd) - want_d).max() <= TOL[dtype] * scale and np.abs(to_np(gs) - want_s).max() <= TOL[dtype] * scale
            gp2 = torch.full((n_out, F), float("nan"), dtype=dtype, device="cuda")
            gas.gas_gat_aggregate_bwd(d(sg.rowptr), d(sg.col), d(sg.colptr), d(sg.row), d(sg.csc_perm).int(), d(p), d(a_dst),
                                      d(a_src), d(gz), gp2, gd, gs, 0.2, plan_t=plan_t)
            assert torch.equal(gp.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                               gp2.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))     # fixed order
