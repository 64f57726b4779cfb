"""Pins for the oracle's APPNP model (CPU only).  The propagation has a closed form its iteration converges to,
alpha (I - (1 - alpha) A_hat)^-1 h0 with A_hat built densely from the edge list, and the usual invariants of
the mini-batch execution hold: a batch that is the whole graph reproduces the full-batch model, exact histories
give exact outputs, alpha = 1 returns the graph-agnostic prediction."""
import numpy as np
import torch

from gas_inputs import rng, configs
from oracle import ops, model as omodel
from tests.util import to_np, f64
from tests.test_oracle_gas import _workload, _sub, _close


def _setup(n=256, f_in=11, f_hid=9, f_out=5, seed=3):
    wl = _workload("gcn", n=n, layers=2, f=8, seed=seed)
    g = wl.graph
    x = to_np(rng.normal_matrix(31, 800, g.n, f_in))
    w1 = to_np(rng.glorot_uniform(31, 801, f_in, f_hid))
    w2 = to_np(rng.glorot_uniform(31, 802, f_hid, f_out))
    return wl, g, x, w1, w2


def _dense_a_hat(g):
    rp, cl = to_np(g.rowptr), to_np(g.col)
    a = np.zeros((g.n, g.n))
    for v in range(g.n):
        a[v, cl[rp[v]:rp[v + 1]]] = 1.0
    a += np.eye(g.n)
    d = a.sum(axis=1)                      # deg + 1
    return a / np.sqrt(np.outer(d, d))


def test_propagation_converges_to_personalised_pagerank():
    wl, g, x, w1, w2 = _setup()
    alpha = 0.2
    whole = torch.cat(wl.batches)
    sg, n_id, rp, cl = _sub(wl, whole)
    hist = [np.zeros((g.n, w2.shape[1]), np.float32) for _ in range(79)]
    y = omodel.appnp_batch_forward(w1, w2, alpha, 80, n_id, rp, cl, sg.nb, to_np(g.deg), x, hist)
    h0 = np.maximum(f64(x) @ f64(w1), 0.0) @ f64(w2)
    want = alpha * np.linalg.solve(np.eye(g.n) - (1.0 - alpha) * _dense_a_hat(g), h0)
    got = np.empty_like(want)
    got[n_id[:sg.nb]] = f64(y)
    assert np.abs(got - want).max() <= 2e-6 * np.abs(want).max()     # (1 - alpha)^80 is far below fp32 rounding
    # one step, brute force
    y1 = omodel.appnp_batch_forward(w1, w2, alpha, 1, n_id, rp, cl, sg.nb, to_np(g.deg), x, [])
    want1 = alpha * h0 + (1.0 - alpha) * _dense_a_hat(g) @ h0
    got1 = np.empty_like(want1)
    got1[n_id[:sg.nb]] = f64(y1)
    assert np.abs(got1 - want1).max() <= 1e-6 * np.abs(want1).max()


def test_alpha_one_returns_the_graph_agnostic_prediction():
    wl, g, x, w1, w2 = _setup()
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    hist = [to_np(rng.normal_matrix(31, 810 + i, g.n, w2.shape[1])) for i in range(2)]
    y = omodel.appnp_batch_forward(w1, w2, 1.0, 3, n_id, rp, cl, sg.nb, to_np(g.deg), x, hist)
    h0 = ops.mlp2(x[n_id[:sg.nb]], w1, w2)
    assert np.array_equal(y, h0)


def test_whole_graph_batch_and_exact_histories_match_the_full_batch_model():
    wl, g, x, w1, w2 = _setup()
    alpha, K = 0.1, 4
    rowptr, col = to_np(g.rowptr).astype(np.int32), to_np(g.col)
    full = omodel.appnp_full_batch(w1, w2, alpha, K, rowptr, col, x)
    # a closed form for the full-batch model itself: h^(K) = sum_{j<K} alpha ((1-alpha) A)^j h0 + ((1-alpha) A)^K h0
    a = (1.0 - alpha) * _dense_a_hat(g)
    h0 = np.maximum(f64(x) @ f64(w1), 0.0) @ f64(w2)
    want, p = np.zeros_like(h0), np.eye(g.n)
    for _ in range(K):
        want += alpha * p @ h0
        p = p @ a
    want += p @ h0
    assert np.abs(full[-1] - want).max() <= 1e-12 * np.abs(want).max()
    # junk histories: only the first step is exact, and the last one is not
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    assert sg.nh > 0
    junk = [to_np(rng.normal_matrix(31, 820 + i, g.n, w2.shape[1])) for i in range(K - 1)]
    y_junk = omodel.appnp_batch_forward(w1, w2, alpha, K, n_id, rp, cl, sg.nb, to_np(g.deg), x, junk, do_push=False)
    assert not _close(y_junk, full[-1][n_id[:sg.nb]], 1e-3)
    # exact histories give exact outputs, for every batch
    for b in wl.batches:
        sg, n_id, rp, cl = _sub(wl, b)
        hist = [full[l].astype(np.float32) for l in range(K - 1)]
        y = omodel.appnp_batch_forward(w1, w2, alpha, K, n_id, rp, cl, sg.nb, to_np(g.deg), x, hist, do_push=False)
        assert _close(y, full[-1][n_id[:sg.nb]], 5e-6)
