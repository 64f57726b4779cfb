"""Pins for the oracle's GAT aggregation (CPU only): dense brute force with torch's own softmax and leaky_relu in
float64, the zero attention vector (uniform weights: the mean over N(v) and v), invariance to a shift of the
receiving node's score, weights that sum to one, and the limit of a dominating neighbour."""
import numpy as np
import torch

from gas_inputs import rng
from oracle import ops
from tests.util import to_np, f64
from tests.test_oracle_gas import _workload, _sub


def _case(f=9, op="gcn"):
    wl = _workload(op, n=240, layers=2, f=8)       # gcn: the pattern carries the self-loops
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    p = to_np(rng.normal_matrix(51, 1000, sg.nv, f))
    a_dst = to_np(rng.normal(51, 1001, 0, f))
    a_src = to_np(rng.normal(51, 1002, 0, f))
    return sg, rp, cl, p, a_dst, a_src


def test_matches_dense_softmax_in_float64():
    sg, rp, cl, p, a_dst, a_src = _case()
    z = ops.gat_aggregate(rp, cl, p, a_dst, a_src, 0.2)
    pp = torch.from_numpy(f64(p))
    s_dst = pp[:sg.nb] @ torch.from_numpy(f64(a_dst))
    s_src = pp @ torch.from_numpy(f64(a_src))
    e = torch.nn.functional.leaky_relu(s_dst[:, None] + s_src[None, :], 0.2)
    mask = torch.zeros((sg.nb, sg.nv), dtype=torch.bool)
    for v in range(sg.nb):
        mask[v, cl[rp[v]:rp[v + 1]]] = True
    assert mask[torch.arange(sg.nb), torch.arange(sg.nb)].all()            # v itself is among the entries
    alpha = torch.softmax(e.masked_fill(~mask, float("-inf")), dim=1)
    want = (alpha @ pp).numpy()
    assert np.abs(z - want).max() <= 1e-6 * np.abs(want).max()
    assert torch.allclose(alpha.sum(dim=1), torch.ones(sg.nb, dtype=torch.float64))


def test_zero_attention_vector_is_the_mean_and_shift_invariance():
    sg, rp, cl, p, a_dst, a_src = _case()
    zero = np.zeros_like(a_dst)
    z = ops.gat_aggregate(rp, cl, p, zero, zero)
    for v in (0, 5, sg.nb - 1):
        want = f64(p)[cl[rp[v]:rp[v + 1]]].mean(axis=0)
        assert np.abs(z[v] - want).max() <= 1e-6
    # with slope 1 the activation is the identity and the receiving node's score cancels in the softmax
    z1 = ops.gat_aggregate(rp, cl, p, a_dst, a_src, 1.0)
    z2 = ops.gat_aggregate(rp, cl, p, 3.0 * a_dst, a_src, 1.0)
    assert np.abs(z1 - z2).max() <= 2e-6 * np.abs(z1).max()
    # with the usual slope it does not cancel
    z3 = ops.gat_aggregate(rp, cl, p, a_dst, a_src, 0.2)
    z4 = ops.gat_aggregate(rp, cl, p, 3.0 * a_dst, a_src, 0.2)
    assert np.abs(z3 - z4).max() > 1e-3


def test_dominating_neighbour_and_empty_row():
    # 3 source rows; row 0 lists all of them, row 1 is empty; a_src makes source 2 win by a wide margin
    rp = np.array([0, 3, 3], dtype=np.int32)
    cl = np.array([0, 1, 2], dtype=np.int32)
    p = np.array([[1.0, 0.0], [0.0, 1.0], [50.0, 7.0]], np.float32)
    z = ops.gat_aggregate(rp, cl, p, np.zeros(2, np.float32), np.array([2.0, 0.0], np.float32))
    assert np.allclose(z[0], [50.0, 7.0], rtol=1e-6) and not z[1].any()
    # very large scores neither overflow nor lose the answer
    z = ops.gat_aggregate(rp, cl, p * 100, np.zeros(2, np.float32), np.array([2.0, 0.0], np.float32))
    assert np.isfinite(z).all() and np.allclose(z[0], [5000.0, 700.0], rtol=1e-6)


def test_gat_model_whole_graph_equals_dense_layers():
    """Two layers on a batch that is the whole graph against the same model written densely with torch in float64."""
    from oracle import model as omodel
    wl = _workload("gcn", n=200, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, torch.cat(wl.batches))
    f = [10, 7, 5]
    x = to_np(rng.normal_matrix(52, 1010, g.n, f[0]))
    ws = [(to_np(rng.glorot_uniform(52, 1011 + 3 * l, f[l], f[l + 1])), to_np(rng.normal(52, 1012 + 3 * l, 0, f[l + 1])),
           to_np(rng.normal(52, 1013 + 3 * l, 0, f[l + 1]))) for l in range(2)]
    hist = [np.zeros((g.n, f[1]), np.float32)]
    y = omodel.gat_batch_forward(ws, n_id, rp, cl, sg.nb, x, hist)
    mask = torch.zeros((g.n, g.n), dtype=torch.bool)
    for v in range(sg.nb):
        mask[n_id[v], n_id[cl[rp[v]:rp[v + 1]]]] = True
    h = torch.from_numpy(f64(x))
    for l, (w, a_dst, a_src) in enumerate(ws):
        p = h @ torch.from_numpy(f64(w))
        e = torch.nn.functional.leaky_relu((p @ torch.from_numpy(f64(a_dst)))[:, None] + (p @ torch.from_numpy(f64(a_src)))[None, :], 0.2)
        h = torch.softmax(e.masked_fill(~mask, float("-inf")), dim=1) @ p
        if l == 0:
            h = torch.relu(h)
    want = h.numpy()[n_id[:sg.nb]]
    assert np.abs(y - want).max() <= 5e-6 * np.abs(want).max()
    # the history now holds layer 1 of every node: a proper batch reproduces its rows from it
    sg1, n_id1, rp1, cl1 = _sub(wl, wl.batches[0])
    y1 = omodel.gat_batch_forward(ws, n_id1, rp1, cl1, sg1.nb, x, [hist[0].copy()], do_push=False)
    assert np.abs(y1 - h.numpy()[n_id1[:sg1.nb]]).max() <= 5e-6 * np.abs(want).max()


def test_multi_head_model_equals_dense_heads_in_float64():
    """Four heads: every block of columns is an attention head of its own.  Written densely with torch in float64 as
    one batched softmax over a [heads, n, n] score tensor (not as the oracle's loop over column slices)."""
    from oracle import model as omodel
    wl = _workload("gcn", n=160, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, torch.cat(wl.batches))
    H, f = 4, [10, 12, 8]
    x = to_np(rng.normal_matrix(53, 1020, g.n, f[0]))
    ws = [(to_np(rng.glorot_uniform(53, 1021 + 3 * l, f[l], f[l + 1])), to_np(rng.normal(53, 1022 + 3 * l, 0, f[l + 1])),
           to_np(rng.normal(53, 1023 + 3 * l, 0, f[l + 1]))) for l in range(2)]
    y = omodel.gat_batch_forward(ws, n_id, rp, cl, sg.nb, x, [np.zeros((g.n, f[1]), np.float32)], heads=H)
    mask = torch.zeros((g.n, g.n), dtype=torch.bool)
    for v in range(sg.nb):
        mask[n_id[v], n_id[cl[rp[v]:rp[v + 1]]]] = True
    h = torch.from_numpy(f64(x))
    for l, (w, a_dst, a_src) in enumerate(ws):
        p = (h @ torch.from_numpy(f64(w))).view(g.n, H, -1).permute(1, 0, 2)                 # [H, n, f/H]
        ad = torch.from_numpy(f64(a_dst)).view(H, 1, -1)
        asr = torch.from_numpy(f64(a_src)).view(H, 1, -1)
        e = torch.nn.functional.leaky_relu((p * ad).sum(-1)[:, :, None] + (p * asr).sum(-1)[:, None, :], 0.2)
        alpha = torch.softmax(e.masked_fill(~mask[None], float("-inf")), dim=2)             # [H, n, n]
        h = torch.bmm(alpha, p).permute(1, 0, 2).reshape(g.n, -1)
        if l == 0:
            h = torch.relu(h)
    want = h.numpy()[n_id[:sg.nb]]
    assert np.abs(y - want).max() <= 5e-6 * np.abs(want).max()
    # and the heads really differ from one head over all columns
    y1 = omodel.gat_batch_forward(ws, n_id, rp, cl, sg.nb, x, [np.zeros((g.n, f[1]), np.float32)], heads=1)
    assert np.abs(y1 - y).max() > 1e-3 * np.abs(want).max()


def test_backward_matches_float64_autograd():
    """oracle_gat_aggregate_bwd (gradients of P, a_dst, a_src) against torch autograd on the dense float64
    re-statement of the aggregation; all rows of P and the in-batch rows only; negative slope 0.2 and 1."""
    sg, rp, cl, p, a_dst, a_src = _case(f=7)
    gz = to_np(rng.normal_matrix(51, 1003, sg.nb, 7))
    mask = torch.zeros((sg.nb, sg.nv), dtype=torch.bool)
    for v in range(sg.nb):
        mask[v, cl[rp[v]:rp[v + 1]]] = True
    for slope in (0.2, 1.0):
        pp = torch.from_numpy(f64(p)).requires_grad_()
        ad = torch.from_numpy(f64(a_dst)).requires_grad_()
        asr = torch.from_numpy(f64(a_src)).requires_grad_()
        e = torch.nn.functional.leaky_relu((pp[:sg.nb] @ ad)[:, None] + (pp @ asr)[None, :], slope)
        z = torch.softmax(e.masked_fill(~mask, float("-inf")), dim=1) @ pp
        (z * torch.from_numpy(f64(gz))).sum().backward()
        gp, gd, gs = ops.gat_aggregate_bwd(rp, cl, p, a_dst, a_src, gz, sg.nv, slope)
        scale = np.abs(asr.grad.numpy()).max()
        for got, want in ((gp, pp.grad.numpy()), (gd, ad.grad.numpy()), (gs, asr.grad.numpy())):
            # with slope 1 the receiving node's score shifts a whole row: a_dst's gradient is zero up to rounding
            assert np.abs(got - want).max() <= 2e-6 * max(np.abs(want).max(), 1e-6 * scale), slope
        if slope == 1.0:
            assert np.abs(gd).max() <= 1e-9 * scale
        gp_b, gd_b, gs_b = ops.gat_aggregate_bwd(rp, cl, p, a_dst, a_src, gz, sg.nb, slope)
        assert np.array_equal(gp_b, gp[:sg.nb]) and np.array_equal(gd_b, gd) and np.array_equal(gs_b, gs)
    assert np.abs(pp.grad.numpy()[sg.nb:]).max() > 0
