"""Pins for the oracle's mini-batch executor (CPU only).

The paper prints no worked numbers for this path, so the executor is pinned
by the facts it states: outputs are exact when a batch has no out-of-batch
neighbours (Section 3, minimising inter-connectivity); layer 1 is always
exact (proof of Theorem 1); exact histories give exact outputs (Eq. 2, line 3
equals line 1); with fixed weights the estimates become exact after a fixed
number of sweeps (Section 2, advantage 4); the error under a perturbed
history obeys Lemma 1; Push and Pull of one layer touch disjoint rows
(Algorithm 1).  The exact model is an independent float64 scipy/numpy
implementation.
"""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, rng
from oracle import ops, model as omodel
from tests.util import to_np, f64, oracle_model


def _workload(op, n=384, n_blocks=4, layers=3, f=12, seed=1):
    cfg = configs.config(0)
    cfg.op, cfg.n, cfg.n_blocks, cfg.seed = op, n, n_blocks, seed
    cfg.graph = dict(kind="sbm_bernoulli", p_in=0.05, p_out=0.01)
    cfg.self_loops = op != "gin"
    if op == "gcnii":
        cfg.widths, cfg.alpha = [f + 3] + [f] * (layers + 1), 0.1
    elif op == "gin":
        cfg.widths, cfg.gin_hidden, cfg.gin_eps = [f + 3] + [f] * layers, f + 5, 0.1
    else:
        cfg.widths = [f + 3] + [f + 1] * (layers - 1) + [f - 2]
    return configs.build_workload(cfg)


def _sub(wl, batch):
    sg = batches.batch_subgraph(wl.graph, batch, wl.cfg.self_loops)
    return sg, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)


def _hist(wl, fill=None):
    hs = [to_np(h).copy() for h in configs.make_histories(wl.cfg, init="zeros")]
    if fill is not None:
        for h, e in zip(hs, fill):
            h[...] = e.astype(np.float32)
    return hs


def _close(a, b, tol=2e-6):
    a, b = f64(a), f64(b)
    return np.abs(a - b).max() <= tol * max(np.abs(b).max(), 1e-30)


OPS = ["gcn", "gin", "gcnii"]


@pytest.mark.parametrize("op", OPS)
def test_inputs_subgraph_matches_plain_construction(op):
    wl = _workload(op)
    g = wl.graph
    for b in wl.batches[:2]:
        sg, n_id, rp, cl = _sub(wl, b)
        n_id2, rp2, cl2 = omodel.batch_subgraph(to_np(g.rowptr), to_np(g.col), b.tolist(), wl.cfg.self_loops)
        assert np.array_equal(n_id, n_id2) and np.array_equal(rp, rp2) and np.array_equal(cl, cl2)
        assert sg.nb == len(b) and sg.nv == len(n_id)


@pytest.mark.parametrize("op", OPS)
def test_whole_graph_batch_equals_full_batch(op):
    wl = _workload(op)
    g, m = wl.graph, oracle_model(wl)
    sg, n_id, rp, cl = _sub(wl, torch.arange(g.n))
    assert sg.nh == 0
    hs = _hist(wl)
    y, layers = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), hs, return_layers=True)
    exact = omodel.full_batch_forward(m, to_np(g.rowptr), to_np(g.col), to_np(wl.x))
    assert len(exact) == m.n_layers == len(layers)
    for got, want in zip(layers, exact):
        assert _close(got, want)
    # and the pushes filled the histories with the exact embeddings
    for h, want in zip(hs, exact[:-1]):
        assert _close(h, want)


@pytest.mark.parametrize("op", OPS)
def test_layer1_is_exact_whatever_the_history_holds(op):
    wl = _workload(op)
    g, m = wl.graph, oracle_model(wl)
    exact = omodel.full_batch_forward(m, to_np(g.rowptr), to_np(g.col), to_np(wl.x))
    junk = [to_np(rng.normal_matrix(9, 70 + i, g.n, h.shape[1])) * 100 for i, h in enumerate(_hist(wl))]
    b = wl.batches[2]
    sg, n_id, rp, cl = _sub(wl, b)
    assert sg.nh > 0
    _, layers = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), junk, return_layers=True)
    assert _close(layers[0][:sg.nb], exact[0][n_id[:sg.nb]])
    # deeper layers do depend on the junk
    assert not _close(layers[1][:sg.nb], exact[1][n_id[:sg.nb]], tol=1e-2)


@pytest.mark.parametrize("op", OPS)
def test_exact_histories_give_exact_outputs(op):
    wl = _workload(op)
    g, m = wl.graph, oracle_model(wl)
    exact = omodel.full_batch_forward(m, to_np(g.rowptr), to_np(g.col), to_np(wl.x))
    hs = _hist(wl, fill=exact[:-1])
    for b in wl.batches:
        sg, n_id, rp, cl = _sub(wl, b)
        y = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), hs)
        assert _close(y, exact[-1][n_id[:sg.nb]], tol=5e-6)


@pytest.mark.parametrize("op", OPS)
def test_fixed_weights_sweeps_converge_to_full_batch(op):
    wl = _workload(op)
    g, m = wl.graph, oracle_model(wl)
    exact = omodel.full_batch_forward(m, to_np(g.rowptr), to_np(g.col), to_np(wl.x))
    hs = _hist(wl)                                            # zeros
    L = m.n_layers
    for sweep in range(1, L + 1):
        outs = {}
        for b in wl.batches:
            sg, n_id, rp, cl = _sub(wl, b)
            outs[tuple(n_id[:sg.nb])] = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), hs)
        # after sweep k the histories of layers <= k are exact
        for l in range(min(sweep, L - 1)):
            assert _close(hs[l], exact[l], tol=5e-6)
        if sweep < L - 1:
            assert not _close(hs[L - 2], exact[L - 2], tol=1e-3)
    for ids, y in outs.items():
        assert _close(y, exact[-1][list(ids)], tol=5e-6)


def test_lemma1_bound_under_perturbed_history():
    # 2-layer GIN (sum aggregation): exact inputs (delta = 0), history rows off by at most eps
    wl = _workload("gin", layers=2)
    g, m = wl.graph, oracle_model(wl)
    exact = omodel.full_batch_forward(m, to_np(g.rowptr), to_np(g.col), to_np(wl.x))
    eps = 0.05
    noise = f64(rng.normal_matrix(11, 80, g.n, exact[0].shape[1]))
    noise *= eps / np.linalg.norm(noise, axis=1, keepdims=True)
    hs = _hist(wl, fill=[exact[0] + noise])
    w1, w2 = m.weights[1]
    k2 = np.linalg.norm(f64(w1), 2) * np.linalg.norm(f64(w2), 2)   # ReLU is 1-Lipschitz
    deg = to_np(g.deg)
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    y = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, deg, to_np(wl.x), hs, do_push=False)
    err = np.linalg.norm(f64(y) - exact[1][n_id[:sg.nb]], axis=1)
    # only out-of-batch neighbours carry the perturbation; |N(v)| bounds their number
    bound = eps * 1.0 * k2 * deg[n_id[:sg.nb]] + 1e-5
    assert (err <= bound).all()
    assert err.max() > 1e-3                                        # the perturbation is visible
    # a node whose neighbours are all in the batch is exact
    n_out = np.array([(cl[rp[v]:rp[v + 1]] >= sg.nb).sum() for v in range(sg.nb)])
    assert (n_out == 0).any() and err[n_out == 0].max() < 1e-5


def test_history_row_reaches_exactly_its_in_batch_neighbours():
    wl = _workload("gcn", layers=2)
    g, m = wl.graph, oracle_model(wl)
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    base = [to_np(rng.normal_matrix(12, 81, g.n, wl.cfg.widths[1]))]
    y0 = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), [base[0].copy()], do_push=False)
    halo_local = sg.nb + 3
    h = base[0].copy()
    h[n_id[halo_local]] += 1.0
    y1 = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), [h], do_push=False)
    changed = np.nonzero(np.abs(y1 - y0).max(axis=1) > 0)[0]
    nbrs = np.array([v for v in range(sg.nb) if halo_local in cl[rp[v]:rp[v + 1]]])
    assert np.array_equal(changed, nbrs) and len(nbrs) > 0
    # an in-batch node's stale history row is never read: its fresh value is used instead
    h = base[0].copy()
    h[n_id[0]] += 1.0
    y2 = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), [h], do_push=False)
    assert np.array_equal(y2, y0)


def test_push_and_pull_touch_disjoint_rows():
    wl = _workload("gcn", layers=2)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    assert len(set(n_id[:sg.nb]) & set(n_id[sg.nb:])) == 0 and len(set(n_id)) == len(n_id)
    hist = to_np(rng.normal_matrix(13, 82, g.n, 8))
    y = to_np(rng.normal_matrix(13, 83, sg.nb, 8))
    a = hist.copy()
    ops.push(y, n_id[:sg.nb], a)
    pulled_after = ops.pull(a, n_id[sg.nb:])
    b = hist.copy()
    pulled_before = ops.pull(b, n_id[sg.nb:])
    ops.push(y, n_id[:sg.nb], b)
    assert np.array_equal(pulled_after, pulled_before) and np.array_equal(a, b)


def test_gcnii_beta_schedule_and_identity_limit():
    betas = omodel.gcnii_betas(4)
    assert np.allclose(betas, [np.log(1.5), np.log(1.25), np.log(0.5 / 3 + 1), np.log(1.125)])
    assert all(0 < b < 1 for b in betas) and betas == sorted(betas, reverse=True)
    # alpha = 1 makes every layer ignore the graph and the layer below: h^(l) = h0 ((1-b_l) I + b_l W_l)
    wl = _workload("gcnii", layers=2)
    g, m = wl.graph, oracle_model(wl)
    m.alpha = 1.0
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    y = omodel.gas_batch_forward(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), _hist(wl))
    h0 = np.maximum(f64(wl.x)[n_id[:sg.nb]] @ f64(wl.w_in), 0)
    h = h0 @ ((1 - betas[1]) * np.eye(h0.shape[1]) + betas[1] * f64(m.weights[1]))
    assert _close(y, h, tol=5e-6)
