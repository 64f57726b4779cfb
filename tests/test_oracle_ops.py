"""Pins for the oracle's per-operation functions (CPU only).

Each check compares the oracle with something that is not the oracle: a
closed form, a dense numpy product built straight from the edge set, or a
library routine (torch's bf16 cast, numpy matmul).
"""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, graphs, rng
from oracle import ops, model as omodel
from tests.util import to_np, f64


# ---------------------------------------------------------------- bf16 store
def test_bf16_round_matches_torch_cast():
    x = rng.normal(3, 1, 0, 200_000) * 37.0
    want = to_np(x.to(torch.bfloat16))
    got = np.array([ops.round_bf16(float(v)) for v in x[:20_000]], dtype=np.uint16)
    assert np.array_equal(got, want[:20_000])


def test_bf16_round_ties_and_double_rounding():
    one = 0x3F80
    assert ops.round_bf16(1.0) == one
    assert ops.round_bf16(1.0 + 2.0 ** -8) == one                 # tie -> even (down)
    assert ops.round_bf16(1.0 + 3 * 2.0 ** -8) == one + 2         # tie -> even (up)
    # just above a tie: rounding through fp32 first would lose the 2^-30 and tie to even
    assert ops.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == one + 1
    assert ops.round_bf16(-(1.0 + 2.0 ** -8 + 2.0 ** -30)) == 0x8000 | (one + 1)
    assert ops.round_bf16(0.0) == 0
    assert ops.round_bf16(float("inf")) == 0x7F80
    assert ops.round_bf16(3.0e38) == 0x7F62                       # below bf16 max, stays finite


# ---------------------------------------------------------------- pull / push
@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
def test_pull_push_are_row_copies(dtype):
    r = np.random.default_rng(0)
    hist = r.integers(0, 60000, size=(97, 24)).astype(dtype)
    before = hist.copy()
    idx = np.array([5, 96, 0, 5, 33], dtype=np.int32)             # duplicates are fine for pull
    got = ops.pull(hist, idx)
    assert np.array_equal(got, before[idx]) and np.array_equal(hist, before)
    uniq = np.array([7, 0, 96, 41], dtype=np.int32)
    src = r.integers(0, 60000, size=(4, 24)).astype(dtype)
    ops.push(src, uniq, hist)
    assert np.array_equal(hist[uniq], src)
    rest = np.setdiff1d(np.arange(97), uniq)
    assert np.array_equal(hist[rest], before[rest])               # untouched rows unchanged
    assert np.array_equal(ops.pull(hist, uniq), src)              # round trip


def test_pull_push_with_row_stride():
    base = np.arange(10 * 16, dtype=np.float32).reshape(10, 16)
    view = base[:, :12]                                           # ld = 16 > F = 12
    idx = np.array([9, 2], dtype=np.int32)
    assert np.array_equal(ops.pull(view, idx), base[idx, :12])
    ops.push(np.full((2, 12), -1, np.float32), idx, view)
    assert (base[idx, :12] == -1).all() and (base[idx, 12:] >= 0).all()


# ---------------------------------------------------------------- GCN coefficient
def _ring(n, d):
    """d-regular circulant graph (d even): i ~ i +- 1..d/2."""
    rows = []
    for i in range(n):
        rows.append(sorted({(i + s) % n for s in range(-d // 2, d // 2 + 1) if s != 0}))
    ptr = np.cumsum([0] + [len(r) for r in rows]).astype(np.int32)
    return ptr, np.concatenate(rows).astype(np.int32)


def test_gcn_norm_regular_graph_is_one_over_d_plus_1():
    ptr, col = _ring(40, 6)
    deg = np.full(40, 6, np.int32)
    val = ops.gcn_norm(ptr, col, np.arange(40, dtype=np.int32), deg)
    assert np.array_equal(val, np.full(col.size, np.float32(1.0 / 7.0)))


def test_gcn_norm_star_closed_form_and_global_degrees():
    # star with centre 0 and 8 leaves, but the "batch" sees only rows {3, 0} of it:
    # degrees must come from the full graph, not from the rows present
    n_id = np.array([3, 0], dtype=np.int32)
    deg = np.array([8] + [1] * 8, dtype=np.int32)
    ptr = np.array([0, 2, 4], dtype=np.int32)       # row 3: {3, 0}; row 0: {3, 0}
    col = np.array([0, 1, 0, 1], dtype=np.int32)
    val = ops.gcn_norm(ptr, col, n_id, deg)
    want = np.array([1 / 2, 1 / (np.sqrt(2.0) * 3.0), 1 / (np.sqrt(2.0) * 3.0), 1 / 9.0])
    assert np.allclose(val, want, rtol=1e-7)


# ---------------------------------------------------------------- aggregation
def _tiny_batch(op_self_loops=True, seed=0):
    cfg = configs.config(0)
    cfg.seed = seed
    g = configs.build_graph(cfg)
    bl = batches.split(g, 1, seed)
    sg = batches.batch_subgraph(g, bl[1], op_self_loops)
    return g, sg


def _dense_gcn_block(g, n_id, nb):
    """D^-1/2 (A+I) D^-1/2 built densely from the edge list, rows/cols picked by n_id."""
    n = g.n
    a = np.zeros((n, n))
    rp, cl = to_np(g.rowptr), to_np(g.col)
    for v in range(n):
        a[v, cl[rp[v]:rp[v + 1]]] = 1.0
    assert np.array_equal(a, a.T) and np.trace(a) == 0
    dinv = 1.0 / np.sqrt(a.sum(1) + 1.0)
    a_hat = dinv[:, None] * (a + np.eye(n)) * dinv[None, :]
    return a, a_hat[np.ix_(n_id[:nb], n_id)]


def test_spmm_equals_dense_symmetric_normalisation():
    g, sg = _tiny_batch()
    n_id = to_np(sg.n_id)
    _, blk = _dense_gcn_block(g, n_id, sg.nb)
    # every neighbour of a batch node is a column: the dropped columns carry no weight
    x = to_np(rng.normal_matrix(1, 50, sg.nv, 24))
    val = ops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), n_id, to_np(g.deg))
    z = ops.spmm(to_np(sg.rowptr), to_np(sg.col), val, x)
    want = blk @ x.astype(np.float64)
    assert np.abs(z - want).max() <= 2e-7 * np.abs(want).max() + 1e-7
    # and the normalised rows of the full matrix have no weight outside n_id
    a, _ = _dense_gcn_block(g, n_id, sg.nb)
    outside = np.setdiff1d(np.arange(g.n), n_id)
    assert a[np.ix_(n_id[:sg.nb], outside)].sum() == 0


def test_spmm_sum_aggregation_diag_scale_residual():
    g, sg = _tiny_batch(op_self_loops=False)
    rp, cl = to_np(sg.rowptr), to_np(sg.col)
    n_id = to_np(sg.n_id)
    ones = np.ones((sg.nv, 3), np.float32)
    z = ops.spmm(rp, cl, None, ones)
    assert np.array_equal(z[:, 0], to_np(g.deg)[n_id[:sg.nb]].astype(np.float32))   # row sums = degree
    x = to_np(rng.normal_matrix(2, 51, sg.nv, 5))
    r = to_np(rng.normal_matrix(2, 52, sg.nb, 5))
    a01, _ = _dense_gcn_block(g, n_id, sg.nb)
    a_blk = a01[np.ix_(n_id[:sg.nb], n_id)]
    z = ops.spmm(rp, cl, None, x, diag=1.1, s_agg=0.9, r=r, s_res=0.25)
    want = 0.9 * (a_blk @ f64(x)) + 1.1 * f64(x)[:sg.nb] + 0.25 * f64(r)
    assert np.abs(z - want).max() <= 3e-7 * np.abs(want).max()


def test_spmm_empty_rows_give_diag_and_residual_only():
    ptr = np.array([0, 0, 2, 2], dtype=np.int32)
    col = np.array([0, 2], dtype=np.int32)
    x = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]], np.float32)
    z = ops.spmm(ptr, col, None, x)
    assert np.array_equal(z, np.array([[0, 0], [6, 8], [0, 0]], np.float32))
    z = ops.spmm(ptr, col, None, x, diag=2.0)
    assert np.array_equal(z, np.array([[2, 4], [12, 16], [10, 12]], np.float32))


def test_spmm_bf16_storage():
    g, sg = _tiny_batch()
    n_id = to_np(sg.n_id)
    xb = rng.normal_matrix(1, 53, sg.nv, 16, dtype=torch.bfloat16)
    val = ops.gcn_norm(to_np(sg.rowptr), to_np(sg.col), n_id, to_np(g.deg))
    z = ops.spmm(to_np(sg.rowptr), to_np(sg.col), val, to_np(xb))
    assert z.dtype == np.uint16
    # dense matrix holding the same fp32 coefficients, so only the store rounding is under test
    rp, cl = to_np(sg.rowptr), to_np(sg.col)
    blk = np.zeros((sg.nb, sg.nv))
    blk[np.repeat(np.arange(sg.nb), np.diff(rp)), cl] = val.astype(np.float64)
    want = to_np(torch.from_numpy(blk @ f64(xb)).to(torch.bfloat16))   # library cast double -> bf16
    # summation order differs in the last double bit: allow a 1-ulp flip next to a rounding tie
    diff = np.abs(z.astype(np.int32) - want.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 1e-3


def test_spmm_t_is_the_dense_transpose_and_adjoint():
    g, sg = _tiny_batch()
    rp, cl, n_id = to_np(sg.rowptr), to_np(sg.col), to_np(sg.n_id)
    val = ops.gcn_norm(rp, cl, n_id, to_np(g.deg))
    _, blk = _dense_gcn_block(g, n_id, sg.nb)
    gz = to_np(rng.normal_matrix(4, 54, sg.nb, 7))
    gx = ops.spmm_t(rp, cl, val, gz, sg.nv)
    want = blk.T @ f64(gz)
    assert np.abs(gx - want).max() <= 3e-7 * np.abs(want).max()
    gx_b = ops.spmm_t(rp, cl, val, gz, sg.nb)
    assert np.array_equal(gx_b, gx[:sg.nb])
    x = to_np(rng.normal_matrix(4, 55, sg.nv, 7))
    z = ops.spmm(rp, cl, val, x)
    lhs, rhs = (f64(z) * f64(gz)).sum(), (f64(x) * f64(gx)).sum()
    assert abs(lhs - rhs) <= 1e-5 * abs(lhs)
    # sum aggregation with a diagonal term
    g2, sg2 = _tiny_batch(op_self_loops=False)
    rp2, cl2 = to_np(sg2.rowptr), to_np(sg2.col)
    a = omodel.dense_adjacency(to_np(sg2.n_id), rp2, cl2, None, sg2.nb)
    a[:, :sg2.nb] += 1.3 * np.eye(sg2.nb)
    gz2 = to_np(rng.normal_matrix(4, 56, sg2.nb, 3))
    got = ops.spmm_t(rp2, cl2, None, gz2, sg2.nv, diag=1.3)
    assert np.abs(got - a.T @ f64(gz2)).max() <= 3e-7 * np.abs(a.T @ f64(gz2)).max()


def test_csc_copy_is_the_transpose_pattern():
    g, sg = _tiny_batch()
    import scipy.sparse as sp
    nnz = sg.nnz
    m = sp.csr_matrix((np.arange(1, nnz + 1), to_np(sg.col), to_np(sg.rowptr)), shape=(sg.nb, sg.nv))
    t = m.tocsc()
    t.sort_indices()
    assert np.array_equal(t.indptr, to_np(sg.colptr)) and np.array_equal(t.indices, to_np(sg.row))
    assert np.array_equal(t.data - 1, to_np(sg.csc_perm))


# ---------------------------------------------------------------- dense transform
def test_linear_matches_numpy_nonsquare_and_epilogues():
    z = to_np(rng.normal_matrix(5, 60, 37, 12))
    w = to_np(rng.glorot_uniform(5, 61, 12, 20))
    b = to_np(rng.normal(5, 62, 0, 20))
    y = ops.linear(z, w)
    want = f64(z) @ f64(w)
    assert y.shape == (37, 20) and np.abs(y - want).max() <= 2e-7 * np.abs(want).max()
    y = ops.linear(z, w, bias=b, relu=True)
    want = np.maximum(f64(z) @ f64(w) + f64(b), 0.0)
    assert np.abs(y - want).max() <= 2e-7 * np.abs(want).max() and (y >= 0).all() and (y == 0).any()
    ws = to_np(rng.glorot_uniform(5, 63, 12, 12))
    y = ops.linear(z, ws, c_identity=0.7, c_weight=0.3)
    want = f64(z) @ (0.7 * np.eye(12) + 0.3 * f64(ws))             # W <- (1-beta) I + beta W
    assert np.abs(y - want).max() <= 3e-7 * np.abs(want).max()
    assert np.array_equal(ops.linear(z, ws, c_identity=1.0, c_weight=0.0), z)


def test_mlp2_matches_numpy():
    z = to_np(rng.normal_matrix(6, 64, 29, 10))
    w1 = to_np(rng.glorot_uniform(6, 65, 10, 16))
    w2 = to_np(rng.glorot_uniform(6, 66, 16, 6))
    want = np.maximum(f64(z) @ f64(w1), 0.0) @ f64(w2)
    y = ops.mlp2(z, w1, w2)
    assert np.abs(y - want).max() <= 2e-7 * np.abs(want).max()
    y = ops.mlp2(z, w1, w2, relu_out=True)
    assert np.abs(y - np.maximum(want, 0)).max() <= 2e-7 * np.abs(want).max()
    zb = rng.normal_matrix(6, 64, 29, 10, dtype=torch.bfloat16)
    w1b, w2b = (rng.glorot_uniform(6, 65 + i, *s, dtype=torch.bfloat16) for i, s in enumerate([(10, 16), (16, 6)]))
    yb = ops.mlp2(to_np(zb), to_np(w1b), to_np(w2b))
    wantb = torch.from_numpy(np.maximum(f64(zb) @ f64(w1b), 0.0) @ f64(w2b)).to(torch.bfloat16)
    assert np.array_equal(yb, to_np(wantb))
