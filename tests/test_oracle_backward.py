"""Pins for the oracle's backward pass (CPU only): every gradient is compared
with torch's autograd on a float64 re-statement of the same mini-batch model
(dense aggregation matrix built from the edge list, histories as constants),
and the per-call functions with closed forms."""
import numpy as np
import pytest
import torch

from gas_inputs import rng
from oracle import ops, model as omodel
from tests.util import to_np, f64, oracle_model
from tests.test_oracle_gas import _workload, _sub


def test_relu_and_linear_backward_calls_match_numpy():
    gy = to_np(rng.normal_matrix(8, 500, 33, 10))
    y = np.maximum(to_np(rng.normal_matrix(8, 501, 33, 10)), 0)
    assert np.array_equal(ops.relu_bwd(gy, y), np.where(y > 0, gy, 0).astype(np.float32))
    gp = to_np(rng.normal_matrix(8, 502, 33, 14))
    w = to_np(rng.glorot_uniform(8, 503, 10, 14))
    z = to_np(rng.normal_matrix(8, 504, 33, 10))
    gz = ops.linear_bwd_input(gp, w)
    want = f64(gp) @ f64(w).T
    assert gz.shape == (33, 10) and np.abs(gz - want).max() <= 2e-7 * np.abs(want).max()
    dw = ops.linear_bwd_weight(z, gp, c_weight=0.5)
    want = 0.5 * f64(z).T @ f64(gp)
    assert dw.shape == (10, 14) and np.abs(dw - want).max() <= 2e-7 * np.abs(want).max()
    ws = to_np(rng.glorot_uniform(8, 505, 14, 14))
    mask = np.maximum(to_np(rng.normal_matrix(8, 506, 33, 14)), 0)
    gz = ops.linear_bwd_input(gp, ws, c_identity=0.7, c_weight=0.3, mask=mask)
    want = np.where(mask > 0, 0.7 * f64(gp) + 0.3 * f64(gp) @ f64(ws).T, 0.0)
    assert np.abs(gz - want).max() <= 3e-7 * np.abs(want).max()


def _torch_replica(wl, m, sg, n_id, rp, cl, hist, grad_out):
    """float64 autograd model of one mini-batch with historical embeddings as constants."""
    g = wl.graph
    t = lambda a: torch.from_numpy(f64(a))
    nb, nv = sg.nb, sg.nv
    deg = to_np(g.deg).astype(np.float64)
    a = np.zeros((nb, nv))
    for v in range(nb):
        for k in range(rp[v], rp[v + 1]):
            w = cl[k]
            a[v, w] = 1.0 if m.op == "gin" else 1.0 / np.sqrt((deg[n_id[v]] + 1.0) * (deg[n_id[w]] + 1.0))
    a = torch.from_numpy(a)
    params = {}
    eps = [torch.tensor(float(m.gin_eps), dtype=torch.float64, requires_grad=True) for _ in m.weights]   # one per layer
    if m.op == "gin":
        ws = [(t(w1).requires_grad_(), t(w2).requires_grad_()) for w1, w2 in m.weights]
    else:
        ws = [t(w).requires_grad_() for w in m.weights]
    x0 = t(to_np(wl.x))[torch.from_numpy(n_id.astype(np.int64))]
    x = x0
    h0 = None
    if m.op == "gcnii":
        params["w_in"] = t(m.w_in).requires_grad_()
        h0 = torch.relu(x0 @ params["w_in"])
        x = h0
    L = m.n_layers
    for l in range(1, L + 1):
        if m.op == "gcn":
            y = (a @ x) @ ws[l - 1]
        elif m.op == "gin":
            z = (1.0 + eps[l - 1]) * x[:nb] + a @ x
            y = torch.relu(z @ ws[l - 1][0]) @ ws[l - 1][1]
        else:
            z = (1.0 - m.alpha) * (a @ x) + m.alpha * h0[:nb]
            b = m.betas[l - 1]
            y = (1.0 - b) * z + b * (z @ ws[l - 1])
        if l < L:
            y = torch.relu(y)
            halo = t(hist[l - 1])[torch.from_numpy(n_id[nb:].astype(np.int64))]      # constants: no gradient
            x = torch.cat([y, halo])
    (y * t(grad_out)).sum().backward()
    grads = {}
    for l in range(L):
        grads[l] = (ws[l][0].grad.numpy(), ws[l][1].grad.numpy()) if m.op == "gin" else ws[l].grad.numpy()
    if m.op == "gcnii":
        grads["w_in"] = params["w_in"].grad.numpy()
    if m.op == "gin":
        grads["eps"] = np.array([float(e.grad) for e in eps])
    return y.detach().numpy(), grads


@pytest.mark.parametrize("op", ["gcn", "gin", "gcnii"])
def test_batch_backward_matches_autograd(op):
    wl = _workload(op, layers=3)
    g, m = wl.graph, oracle_model(wl)
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    assert sg.nh > 0
    hist = [to_np(rng.normal_matrix(14, 510 + i, g.n, wl.cfg.widths[i + (2 if op == "gcnii" else 1)])) for i in range(2)]
    f_out = m.weights[-1][1].shape[1] if op == "gin" else m.weights[-1].shape[1]
    grad_out = to_np(rng.normal_matrix(14, 520, sg.nb, f_out))
    y, grads = omodel.gas_batch_train(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), [h.copy() for h in hist],
                                      grad_out, do_push=False)
    y_t, grads_t = _torch_replica(wl, m, sg, n_id, rp, cl, hist, grad_out)
    assert np.abs(y - y_t).max() <= 5e-6 * np.abs(y_t).max()

    def close(a, b):
        return np.abs(f64(a) - b).max() <= 2e-5 * np.abs(b).max()
    for l in range(m.n_layers):
        if op == "gin":
            assert close(grads[l][0], grads_t[l][0]) and close(grads[l][1], grads_t[l][1]), l
        else:
            assert close(grads[l], grads_t[l]), l
    if op == "gcnii":
        assert close(grads["w_in"], grads_t["w_in"])
    if op == "gin":
        # the gradient of every layer's eps (the self term's weight is 1 + eps)
        assert grads["eps"].shape == (m.n_layers,) and np.abs(grads_t["eps"]).min() > 0
        assert np.abs(grads["eps"] - grads_t["eps"]).max() <= 2e-5 * np.abs(grads_t["eps"]).max()
    # the gradients of the lower layers are not all zero: the backward really reached them
    first = grads[0][0] if op == "gin" else grads[0]
    assert np.abs(first).max() > 1e-4
