"""Pins for the oracle's PNA aggregation (CPU only): mean against the row-normalised dense adjacency product,
min and max against numpy's masked reductions over the dense adjacency, the degree scalers against their closed
form on a regular graph (all equal to one) and on a star, the receiving-node term commuting with all three
aggregators, and a node without neighbours."""
import numpy as np

from gas_inputs import rng
from oracle import ops
from tests.util import to_np, f64
from tests.test_oracle_gas import _workload, _sub


def _dense(rp, cl, nb, nv):
    a = np.zeros((nb, nv), dtype=bool)
    for v in range(nb):
        a[v, cl[rp[v]:rp[v + 1]]] = True
    return a


def test_aggregators_match_dense_brute_force():
    wl = _workload("gin", n=300, layers=2, f=8)                # no self-loops: N(v) only
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[2])
    f = 7
    x = to_np(rng.normal_matrix(41, 900, sg.nv, f))
    q = to_np(rng.normal_matrix(41, 901, sg.nb, f))
    deg = to_np(g.deg).astype(np.float64)
    delta = float(np.log(deg + 1.0).mean())
    out = ops.pna_aggregate(rp, cl, x, delta, add=q)
    a = _dense(rp, cl, sg.nb, sg.nv)
    d = a.sum(axis=1)
    assert np.array_equal(d, deg[n_id[:sg.nb]])                # every neighbour of an in-batch node is in G_b
    has = d > 0
    xx = f64(x)
    mean = np.where(has[:, None], (a.astype(np.float64) @ xx) / np.maximum(d, 1)[:, None] + f64(q), 0.0)
    big = np.where(a[:, :, None], xx[None, :, :], np.inf)
    mn = np.where(has[:, None], big.min(axis=1) + f64(q), 0.0)
    mx = np.where(has[:, None], np.where(a[:, :, None], xx[None, :, :], -np.inf).max(axis=1) + f64(q), 0.0)
    s = np.log(d + 1.0) / delta
    blocks = [mean, mn, mx]
    for j in range(3):
        assert np.abs(out[:, j * f:(j + 1) * f] - blocks[j]).max() <= 1e-6 * np.abs(blocks[j]).max(), j
        want = s[:, None] * blocks[j]
        assert np.abs(out[:, (3 + j) * f:(4 + j) * f] - want).max() <= 1e-6 * np.abs(want).max(), j
        want = np.where(has[:, None], blocks[j] / np.where(has, s, 1.0)[:, None], 0.0)
        assert np.abs(out[:, (6 + j) * f:(7 + j) * f] - want).max() <= 1e-6 * np.abs(want).max(), j
    # min <= mean <= max wherever there is a neighbour
    assert (out[has, f:2 * f] <= out[has, :f] + 1e-6).all() and (out[has, :f] <= out[has, 2 * f:3 * f] + 1e-6).all()


def test_scalers_closed_forms_and_isolated_node():
    # a ring: every degree is 2, delta = log 3, so s = 1 and the three scaler blocks coincide
    n, f = 12, 5
    rp = np.arange(0, 2 * n + 1, 2, dtype=np.int32)
    cl = np.stack([(np.arange(n) - 1) % n, (np.arange(n) + 1) % n], axis=1).astype(np.int32)
    cl.sort(axis=1)
    x = to_np(rng.normal_matrix(42, 910, n, f))
    out = ops.pna_aggregate(rp, cl.ravel(), x, float(np.log(3.0)))
    assert np.array_equal(out[:, :3 * f], out[:, 3 * f:6 * f]) and np.array_equal(out[:, :3 * f], out[:, 6 * f:])
    left, right = f64(x)[(np.arange(n) - 1) % n], f64(x)[(np.arange(n) + 1) % n]
    assert np.abs(out[:, :f] - (left + right) / 2).max() <= 1e-7
    assert np.array_equal(out[:, f:2 * f], np.minimum(left, right).astype(np.float32))
    assert np.array_equal(out[:, 2 * f:3 * f], np.maximum(left, right).astype(np.float32))
    # a star with 4 leaves plus an isolated node: centre sees all leaves, a leaf sees only the centre
    rp = np.array([0, 4, 5, 6, 7, 8, 8], dtype=np.int32)
    cl = np.array([1, 2, 3, 4, 0, 0, 0, 0], dtype=np.int32)
    x = np.array([[10.0], [1.0], [2.0], [3.0], [6.0], [99.0]], np.float32)
    delta = 0.7
    out = ops.pna_aggregate(rp, cl, x, delta)
    s_c, s_l = np.log(5.0) / delta, np.log(2.0) / delta
    want_c = [3.0, 1.0, 6.0, 3.0 * s_c, 1.0 * s_c, 6.0 * s_c, 3.0 / s_c, 1.0 / s_c, 6.0 / s_c]
    assert np.allclose(out[0], want_c, rtol=1e-6)
    assert np.allclose(out[1], [10.0] * 3 + [10.0 * s_l] * 3 + [10.0 / s_l] * 3, rtol=1e-6)
    assert not out[5].any()                                     # no neighbour, no message


def test_bf16_storage_rounds_once():
    import torch
    wl = _workload("gin", n=200, layers=2, f=8)
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    f = 8
    xb = rng.normal_matrix(43, 920, sg.nv, f, dtype=torch.bfloat16)
    out = ops.pna_aggregate(rp, cl, to_np(xb), 1.3)
    ref = ops.pna_aggregate(rp, cl, to_np(xb.float()), 1.3)    # same inputs, fp32 storage
    # min and max of bf16 values are bf16 values: exact; the others are within half a bf16 ulp of the fp32 result
    assert np.array_equal(f64(out[:, f:3 * f]), f64(ref[:, f:3 * f]))
    err = np.abs(f64(out) - f64(ref))
    assert (err <= 2.0 ** -8 * np.abs(f64(ref)) + 1e-30).all()


def test_layer_equals_the_formula_written_out_per_message():
    """The operator appendix's formula evaluated literally: every message W1 [h_v, h_w] built on its own, then
    aggregated, scaled, concatenated and multiplied by W2, in float64."""
    from oracle import model as omodel
    wl = _workload("gin", n=160, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    f, f1, f_out = 6, 5, 4
    x = to_np(rng.normal_matrix(44, 930, sg.nv, f))
    w1 = to_np(rng.glorot_uniform(44, 931, 2 * f, f1))
    w2 = to_np(rng.glorot_uniform(44, 932, f + 9 * f1, f_out))
    delta = float(np.log(to_np(g.deg).astype(np.float64) + 1.0).mean())
    y = omodel.pna_layer(x, sg.nb, rp, cl, w1, w2, delta, relu=True)
    xx, ww1, ww2 = f64(x), f64(w1), f64(w2)
    want = np.zeros((sg.nb, f_out))
    for v in range(sg.nb):
        nbrs = cl[rp[v]:rp[v + 1]]
        if len(nbrs):
            msgs = np.stack([np.concatenate([xx[v], xx[w]]) @ ww1 for w in nbrs])
            aggs = np.concatenate([msgs.mean(axis=0), msgs.min(axis=0), msgs.max(axis=0)])
            s = np.log(len(nbrs) + 1.0) / delta
            big = np.concatenate([aggs, s * aggs, aggs / s])
        else:
            big = np.zeros(9 * f1)
        want[v] = np.maximum(np.concatenate([xx[v], big]) @ ww2, 0.0)
    assert np.abs(f64(y) - want).max() <= 3e-6 * np.abs(want).max()
    assert (want > 0).any()


def test_pna_whole_graph_batch_needs_no_history():
    from oracle import model as omodel
    import torch
    wl = _workload("gin", n=160, layers=2, f=8)
    g = wl.graph
    f, f1 = 6, 5
    x = to_np(rng.normal_matrix(45, 940, g.n, f))
    ws = [(to_np(rng.glorot_uniform(45, 941 + 2 * l, 2 * f, f1)), to_np(rng.glorot_uniform(45, 942 + 2 * l, f + 9 * f1, f)))
          for l in range(3)]
    delta = float(np.log(to_np(g.deg).astype(np.float64) + 1.0).mean())
    sg, n_id, rp, cl = _sub(wl, torch.cat(wl.batches))
    junk = [to_np(rng.normal_matrix(45, 950 + l, g.n, f)) for l in range(2)]
    zero = [np.zeros((g.n, f), np.float32) for _ in range(2)]
    a = omodel.pna_batch_forward(ws, delta, n_id, rp, cl, sg.nb, x, junk)
    b = omodel.pna_batch_forward(ws, delta, n_id, rp, cl, sg.nb, x, zero)
    assert np.array_equal(a, b)                                  # no halo: histories are written, never read
    # a proper batch with the whole-graph run's own histories reproduces its rows
    sg1, n_id1, rp1, cl1 = _sub(wl, wl.batches[0])
    assert sg1.nh > 0
    y1 = omodel.pna_batch_forward(ws, delta, n_id1, rp1, cl1, sg1.nb, x, [h.copy() for h in zero], do_push=False)
    order = np.argsort(n_id[:sg.nb])
    full_rows = a[order][n_id1[:sg1.nb]]
    assert np.abs(y1 - full_rows).max() <= 5e-6 * np.abs(full_rows).max()


def test_backward_matches_float64_autograd_and_the_first_extreme_takes_the_gradient():
    """oracle_pna_aggregate_bwd against torch autograd on a dense re-statement of the nine blocks (masked mean,
    amin, amax; continuous data, so no ties), for all columns and for the in-batch columns only; then a tie:
    the first entry of the row that attains the extreme receives its gradient."""
    import torch
    wl = _workload("gin", n=300, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[2])
    f = 6
    x = to_np(rng.normal_matrix(42, 910, sg.nv, f))
    q = to_np(rng.normal_matrix(42, 911, sg.nb, f))
    gout = to_np(rng.normal_matrix(42, 912, sg.nb, 9 * f))
    delta = float(np.log(to_np(g.deg).astype(np.float64) + 1.0).mean())
    a = torch.from_numpy(_dense(rp, cl, sg.nb, sg.nv))
    d = a.sum(dim=1).double()
    has = d > 0
    xt = torch.from_numpy(f64(x)).requires_grad_()
    qt = torch.from_numpy(f64(q)).requires_grad_()
    mean = (a.double() @ xt) / d.clamp(min=1)[:, None]
    mn = torch.where(a[:, :, None], xt[None], torch.tensor(float("inf"), dtype=torch.float64)).amin(dim=1)
    mx = torch.where(a[:, :, None], xt[None], torch.tensor(float("-inf"), dtype=torch.float64)).amax(dim=1)
    s = (torch.log(d + 1.0) / delta)[:, None]
    agg = [torch.where(has[:, None], t + qt, torch.zeros_like(qt)) for t in (mean, mn, mx)]
    out = torch.cat(agg + [torch.where(has[:, None], s * t, torch.zeros_like(t)) for t in agg] +
                    [torch.where(has[:, None], t / s.clamp(min=1e-30), torch.zeros_like(t)) for t in agg], dim=1)
    fwd = ops.pna_aggregate(rp, cl, x, delta, add=q)
    assert np.abs(fwd - out.detach().numpy()).max() <= 1e-6 * np.abs(fwd).max()       # the same function
    (out * torch.from_numpy(f64(gout))).sum().backward()
    gx, gadd = ops.pna_aggregate_bwd(rp, cl, x, delta, gout, sg.nv)
    want_x, want_q = xt.grad.numpy(), qt.grad.numpy()
    assert np.abs(gx - want_x).max() <= 1e-6 * np.abs(want_x).max()
    assert np.abs(gadd - want_q).max() <= 1e-6 * np.abs(want_q).max()
    assert np.abs(want_x[sg.nb:]).max() > 0                                           # halo columns do get gradient
    gx_b, none = ops.pna_aggregate_bwd(rp, cl, x, delta, gout, sg.nb, want_add=False)
    assert none is None and np.array_equal(gx_b, gx[:sg.nb])
    # a tie: two neighbours with the same value in feature 0; the first in stored order takes min and max gradient
    rp2 = np.array([0, 3], dtype=np.int32)
    cl2 = np.array([2, 0, 1], dtype=np.int32)
    x2 = np.array([[5.0], [7.0], [5.0]], dtype=np.float32)                            # entries: x[2]=5, x[0]=5, x[1]=7
    g2 = np.zeros((1, 9), dtype=np.float32)
    g2[0, 1] = 1.0                                                                    # gradient on the min block only
    gx2, _ = ops.pna_aggregate_bwd(rp2, cl2, x2, 1.0, g2, 3)
    assert gx2[:, 0].tolist() == [0.0, 0.0, 1.0]                                      # column 2 is the first entry with 5
