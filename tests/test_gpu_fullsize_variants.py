"""PNA's and GAT's aggregations and their backward passes at a benchmark configuration's full size (first batch,
width 256), the way bench/bench_variants.py runs them.  The oracle cannot run whole tensors of this size in seconds:

  - forward calls are checked on sampled output rows, which the oracle computes from those rows' own entries;
  - a backward output row belongs to a COLUMN u of the pattern and depends on every row that has an entry in it and,
    through the softmax or the extremes, on all entries of those rows.  For a sample of columns the oracle therefore
    runs the backward pass of the sub-pattern made of all rows that touch a sampled column, with all their entries,
    and its output rows for the sampled columns are complete and are compared;
  - the fast path (plan of the CSC copy) and the plain kernels are compared with each other on every row.
"""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, rng
from oracle import ops as oops
from tests.util import to_np, node_rel_err

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def _setup(cfg_id):
    import paper_2106_05609_amd as gas
    dev = torch.device("cuda:0")
    cfg = configs.config(cfg_id)
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], True)
    F, dt = 256, cfg.dtype
    plan_t = gas.gas_plan_create(sg.colptr, sg.nnz, F, ind=sg.row)
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    return gas, dev, cfg, g, sg, F, dt, plan_t, delta


def _columns_sample(sg, n_random, n_heavy, seed):
    clen = (sg.colptr[1:] - sg.colptr[:-1]).cpu().numpy()
    r = np.random.default_rng(seed).choice(clen.size, size=n_random, replace=False)
    # long columns (the whole-wavefront paths), but not the longest: the rows that touch a column of 17,000 entries
    # hold millions of entries, minutes of oracle time
    heavy = np.argsort(np.abs(clen - 1000), kind="stable")[:n_heavy]
    empty = np.nonzero(clen == 0)[0][:4]
    return np.unique(np.concatenate([r, heavy, empty, [0, sg.nb - 1, sg.nb, clen.size - 1]]))


def _sub_problem(sg, us):
    """All rows with an entry in one of the columns `us` (plus those columns' own rows, for in-batch columns), with all
    their entries; columns renumbered so that sub-row i is sub-column i.  Returns (rows R, sub_ptr, sub_col, old ids of
    the sub-columns, position of every sampled column among the sub-columns)."""
    colptr, row, rowptr = sg.colptr.cpu().numpy(), sg.row, sg.rowptr.cpu().numpy()
    touching = [row[colptr[u]:colptr[u + 1]].cpu().numpy() for u in us]
    R = np.unique(np.concatenate(touching + [us[us < sg.nb]])).astype(np.int64)
    pos = np.concatenate([np.arange(rowptr[r], rowptr[r + 1]) for r in R]).astype(np.int64)
    sub_ptr = np.zeros(R.size + 1, dtype=np.int32)
    sub_ptr[1:] = np.cumsum(rowptr[R + 1] - rowptr[R])
    ind = sg.col[torch.from_numpy(pos).to(sg.col.device)].cpu().numpy().astype(np.int64)
    others = np.setdiff1d(np.unique(ind), R)
    ids = np.concatenate([R, others])                       # old id of every sub-column; the rows come first
    order = np.argsort(ids)
    sub_col = order[np.searchsorted(ids[order], ind)].astype(np.int32)
    where = order[np.searchsorted(ids[order], us)]          # every sampled column is in ids: a row or a column of R
    assert np.array_equal(ids[where], us)
    return R, sub_ptr, sub_col, ids, where


def _check_pna(cfg_id, gas, dev, cfg, g, sg, F, dt, plan_t, delta):
    nb, nv = sg.nb, sg.nv
    x = rng.normal_matrix(cfg.seed, 1600, nv, F, dev, dt)
    add = rng.normal_matrix(cfg.seed, 1601, nb, F, dev, dt)
    out9 = torch.empty((nb, 9 * F), dtype=dt, device=dev)
    gas.gas_pna_aggregate(sg.rowptr, sg.col, x, out9, delta, add=add)
    # forward: sampled rows from their own entries
    rlen = (sg.rowptr[1:] - sg.rowptr[:-1]).cpu().numpy()
    rs = np.unique(np.concatenate([np.random.default_rng(5).choice(nb, 3000, replace=False), np.argsort(-rlen)[:8],
                                   np.argsort(rlen)[:32]]))
    rp = sg.rowptr.cpu().numpy()
    pos = np.concatenate([np.arange(rp[r], rp[r + 1]) for r in rs]).astype(np.int64)
    sub_ptr = np.zeros(rs.size + 1, dtype=np.int32)
    sub_ptr[1:] = np.cumsum(rp[rs + 1] - rp[rs])
    cols, inv = np.unique(sg.col[torch.from_numpy(pos).to(dev)].cpu().numpy(), return_inverse=True)
    rs_dev = torch.from_numpy(rs).to(dev)
    want = oops.pna_aggregate(sub_ptr, inv.astype(np.int32), to_np(x[torch.from_numpy(cols).to(dev)]), delta,
                              add=to_np(add[rs_dev]))
    assert node_rel_err(to_np(out9[rs_dev]), want) <= TOL[dt]
    # backward: the gradient of every output block, drawn; fast path against the plain kernels on every row
    gout = rng.normal_matrix(cfg.seed, 1602, nb, 9 * F, dev, dt)
    csc_pos = sg.csc_perm.to(torch.int32)
    res = {}
    for name, plan in (("fast", plan_t), ("plain", None)):
        gx = torch.full((nv, F), float("nan"), dtype=dt, device=dev)
        gadd = torch.full((nb, F), float("nan"), dtype=dt, device=dev)
        gas.gas_pna_aggregate_bwd(sg.rowptr, sg.col, sg.colptr, sg.row, csc_pos, x, gout, gx, delta, gadd=gadd, plan_t=plan)
        res[name] = (gx, gadd)
    assert torch.equal(res["fast"][1], res["plain"][1])
    a, b = res["fast"][0].float(), res["plain"][0].float()
    assert not torch.isnan(a).any() and not torch.isnan(b).any()
    scale = torch.maximum(b.abs().amax(dim=1), 1e-3 * b.abs().max())
    worst = float(((a - b).abs().amax(dim=1) / scale).max())
    assert worst <= 2 * TOL[dt], worst                      # two results, each within tol of the exact one
    # backward against the oracle on sampled columns
    us = _columns_sample(sg, 60 if cfg_id == 2 else 400, 2, 7)   # config 2: the touching rows are long
    R, sub_ptr, sub_col, ids, where = _sub_problem(sg, us)
    ids_dev, R_dev = torch.from_numpy(ids).to(dev), torch.from_numpy(R).to(dev)
    want_x, want_add = oops.pna_aggregate_bwd(sub_ptr, sub_col, to_np(x[ids_dev]), delta, to_np(gout[R_dev]), ids.size)
    us_dev = torch.from_numpy(us).to(dev)
    for name in ("fast", "plain"):
        e = node_rel_err(to_np(res[name][0][us_dev]), want_x[where])
        assert e <= TOL[dt], (name, e)
        assert node_rel_err(to_np(res[name][1][R_dev]), want_add) <= TOL[dt]


def _check_gat(cfg_id, gas, dev, cfg, g, sg, F, dt, plan_t, delta):
    nb, nv = sg.nb, sg.nv
    p = rng.normal_matrix(cfg.seed, 1700, nv, F, dev, dt) * 0.5
    a_dst = rng.normal(cfg.seed, 1701, 0, F, dev, dt) * 0.1
    a_src = rng.normal(cfg.seed, 1702, 0, F, dev, dt) * 0.1
    gz = rng.normal_matrix(cfg.seed, 1703, nb, F, dev, dt)
    z = torch.empty((nb, F), dtype=dt, device=dev)
    gas.gas_gat_aggregate(sg.rowptr, sg.col, p, a_dst, a_src, z, 0.2, relu=False)
    csc_pos = sg.csc_perm.to(torch.int32)
    res = {}
    for name, plan in (("fast", plan_t), ("plain", None)):
        gp = torch.full((nv, F), float("nan"), dtype=dt, device=dev)
        gd = torch.full((F,), float("nan"), device=dev)
        gs = torch.full((F,), float("nan"), device=dev)
        gas.gas_gat_aggregate_bwd(sg.rowptr, sg.col, sg.colptr, sg.row, csc_pos, p, a_dst, a_src, gz, gp, gd, gs, 0.2,
                                  plan_t=plan)
        res[name] = (gp, gd, gs)
    # The two vector gradients are sums over all entries, so no sample of the pattern gives them: the two paths are
    # compared with each other (each is compared with the oracle on small graphs).  They are sums of millions of
    # signed terms that cancel to a total far below the sum of their magnitudes, which is what a path's rounding
    # error is relative to: ten times the per-value tolerance on the scale of the larger vector.
    vscale = max(float(res["plain"][1].abs().max()), float(res["plain"][2].abs().max()))
    for k in (1, 2):
        assert float((res["fast"][k] - res["plain"][k]).abs().max()) <= 10 * TOL[dt] * vscale
    # sampled columns against the oracle on the sub-pattern of all rows that touch them (forward rows too)
    us = _columns_sample(sg, 60 if cfg_id == 2 else 400, 2, 9)
    R, sub_ptr, sub_col, ids, where = _sub_problem(sg, us)
    ids_dev, R_dev, us_dev = (torch.from_numpy(t).to(dev) for t in (ids, R, us))
    p_sub, gz_sub = to_np(p[ids_dev]), to_np(gz[R_dev])
    ad, asr = to_np(a_dst), to_np(a_src)
    want_z = oops.gat_aggregate(sub_ptr, sub_col, p_sub, ad, asr, 0.2, relu=False)
    assert node_rel_err(to_np(z[R_dev]), want_z) <= TOL[dt]
    want_p, _, _ = oops.gat_aggregate_bwd(sub_ptr, sub_col, p_sub, ad, asr, gz_sub, ids.size, 0.2)
    # per-row scale of the rounding errors, as in tests/test_gpu_ops.py::test_gat_aggregate_backward_parity
    rows = np.repeat(np.arange(R.size), np.diff(sub_ptr))
    p64, ad64, as64 = oops.to_f64(p_sub), oops.to_f64(ad), oops.to_f64(asr)
    t = (p64[:R.size] @ ad64)[rows] + (p64 @ as64)[sub_col]
    lt = np.where(t > 0, t, 0.2 * t)
    ex = np.exp(lt - np.maximum.reduceat(lt, sub_ptr[:-1])[rows])
    alpha = ex / np.add.reduceat(ex, sub_ptr[:-1])[rows]
    weight = alpha * np.linalg.norm(oops.to_f64(gz_sub), axis=1)[rows] * np.linalg.norm(p64, axis=1)[sub_col]
    terms = np.bincount(sub_col, weights=weight, minlength=ids.size) * np.abs(as64).max()
    terms[:R.size] += np.add.reduceat(weight, sub_ptr[:-1]) * np.abs(ad64).max()
    for name in ("fast", "plain"):
        e = node_rel_err(to_np(res[name][0][us_dev]), want_p[where], scale=terms[where])
        assert e <= TOL[dt], (name, e)


@pytest.mark.parametrize("cfg_id", [2, 4])
def test_pna_and_gat_at_full_size(cfg_id):
    args = _setup(cfg_id)
    _check_pna(cfg_id, *args)
    torch.cuda.empty_cache()
    _check_gat(cfg_id, *args)
