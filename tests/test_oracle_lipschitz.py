"""Pins for the pieces of the paper's Eq. (3) in the oracle (CPU only): the perturbed input and the row distance
against numpy, the drawn perturbations inside their ball, and the regulariser of a linear layer, whose difference
f(x + eps) - f(x) = A_hat eps W is known in closed form."""
import numpy as np
import torch

from gas_inputs import rng
from oracle import ops, model as omodel
from tests.util import to_np, f64, oracle_model
from tests.test_oracle_gas import _workload, _sub


def test_axpy_and_row_distance_match_numpy():
    x = to_np(rng.normal_matrix(61, 1100, 40, 9))
    e = to_np(rng.normal_matrix(61, 1101, 40, 9))
    y = ops.axpy(x, e, 0.25)
    assert np.array_equal(y, (f64(x) + 0.25 * f64(e)).astype(np.float32))
    d, total = ops.row_distance(x, y)
    want = np.linalg.norm(f64(x) - f64(y), axis=1)
    assert np.abs(d - want).max() <= 1e-7 * want.max() and abs(total - want.sum()) <= 1e-12 * want.sum()
    assert ops.row_distance(x, x)[1] == 0.0
    # 3-4-5
    d, _ = ops.row_distance(np.array([[0.0, 0.0]], np.float32), np.array([[3.0, 4.0]], np.float32))
    assert d[0] == 5.0
    xb = rng.normal_matrix(61, 1102, 16, 8, dtype=torch.bfloat16)
    eb = rng.normal_matrix(61, 1103, 16, 8, dtype=torch.bfloat16)
    yb = ops.axpy(to_np(xb), to_np(eb), 0.5)
    assert np.array_equal(yb, to_np((xb.double() + 0.5 * eb.double()).to(torch.bfloat16)))


def test_perturbations_lie_in_the_ball():
    e = rng.ball_matrix(62, 1110, 5000, 6, 0.3)
    r = e.double().norm(dim=1)
    assert float(r.max()) <= 0.3 * (1 + 1e-6)
    # uniform in the ball: P(r <= 0.3 * 2^(-1/6)) = 1/2, and the mean of every coordinate is 0
    assert abs(float((r <= 0.3 * 2 ** (-1 / 6)).double().mean()) - 0.5) < 0.03
    assert float(e.double().mean(dim=0).abs().max()) < 0.01


def test_regulariser_of_a_linear_layer_has_a_closed_form():
    wl = _workload("gcn", n=200, layers=2, f=8)
    g, m = wl.graph, oracle_model(wl)
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    val = ops.gcn_norm(rp, cl, n_id, to_np(g.deg))
    f_in = m.weights[-1].shape[0]
    x = to_np(rng.normal_matrix(63, 1120, sg.nv, f_in))
    eps = to_np(rng.ball_matrix(63, 1121, sg.nv, f_in, 0.1))
    got = omodel.lipschitz_reg(m, m.n_layers, x, eps, rp, cl, val, sg.nb)      # the last layer has no ReLU: linear
    a = omodel.dense_adjacency(n_id, rp, cl, val, sg.nb)
    diff = a @ f64(eps) @ f64(m.weights[-1])
    want = np.linalg.norm(diff, axis=1).mean()
    assert abs(got - want) <= 2e-4 * want          # the two outputs are rounded to fp32 before they are subtracted
    assert omodel.lipschitz_reg(m, m.n_layers, x, np.zeros_like(eps), rp, cl, val, sg.nb) == 0.0
    # a non-linear layer: bounded by the linear map's norm times the perturbation (ReLU is 1-Lipschitz)
    got1 = omodel.lipschitz_reg(m, 1, to_np(rng.normal_matrix(63, 1122, sg.nv, m.weights[0].shape[0])),
                                to_np(rng.ball_matrix(63, 1123, sg.nv, m.weights[0].shape[0], 0.1)), rp, cl, val, sg.nb)
    bound = 0.1 * np.linalg.norm(a, 2) * np.linalg.norm(f64(m.weights[0]), 2) * np.sqrt(sg.nv) / sg.nb * np.sqrt(sg.nb)
    assert 0.0 < got1 <= bound


def test_row_distance_gradient_matches_autograd_and_its_closed_forms():
    a = to_np(rng.normal_matrix(64, 1130, 30, 7))
    b = to_np(rng.normal_matrix(64, 1131, 30, 7))
    b[3] = a[3]                                              # equal rows: zero gradient
    ta = torch.from_numpy(f64(a)).requires_grad_()
    (0.25 * (ta - torch.from_numpy(f64(b))).norm(dim=1).sum()).backward()
    g = ops.row_distance_bwd(a, b, 0.25)
    want = ta.grad.numpy()
    want[3] = 0.0
    assert np.abs(f64(g) - want).max() <= 1e-7
    assert not g[3].any()
    # every non-zero row of the gradient has norm `scale`
    n = np.linalg.norm(f64(g), axis=1)
    assert np.abs(np.delete(n, 3) - 0.25).max() <= 1e-6
    # 3-4-5
    g = ops.row_distance_bwd(np.array([[3.0, 4.0]], np.float32), np.array([[0.0, 0.0]], np.float32), 1.0)
    assert np.abs(g - np.array([[0.6, 0.8]], np.float32)).max() <= 1e-7


import pytest


@pytest.mark.parametrize("op,layer", [("gcn", 1), ("gcn", 2), ("gin", 1), ("gcnii", 2)])
def test_regulariser_gradient_matches_autograd(op, layer):
    """Eq. (3) differentiated with respect to the layer's weights (input held fixed) against float64 autograd of
    the same expression written with a dense adjacency."""
    wl = _workload(op, n=160, layers=2, f=8)
    g, m = wl.graph, oracle_model(wl)
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    val = ops.gcn_norm(rp, cl, n_id, to_np(g.deg)) if op != "gin" else None
    f_in = (m.weights[layer - 1][0] if op == "gin" else m.weights[layer - 1]).shape[0]
    x = to_np(rng.normal_matrix(65, 1140, sg.nv, f_in))
    eps = to_np(rng.ball_matrix(65, 1141, sg.nv, f_in, 0.2))
    h0 = to_np(torch.relu(rng.normal_matrix(65, 1142, sg.nv, f_in))) if op == "gcnii" else None
    loss, dw = omodel.lipschitz_reg_grad(m, layer, x, eps, rp, cl, val, sg.nb, h0)
    # (GIN: the gradient needs the hidden activation stored, the plain evaluation keeps it unrounded)
    assert abs(loss - omodel.lipschitz_reg(m, layer, x, eps, rp, cl, val, sg.nb, h0)) <= 1e-6 * loss
    # autograd replica
    a = torch.from_numpy(omodel.dense_adjacency(n_id, rp, cl, val if val is not None else np.ones(len(cl), np.float32), sg.nb))
    last = layer == m.n_layers
    ws = [torch.from_numpy(f64(w)).requires_grad_() for w in (m.weights[layer - 1] if op == "gin" else [m.weights[layer - 1]])]

    def f(xx):
        xx = torch.from_numpy(f64(xx))
        if op == "gcn":
            y = (a @ xx) @ ws[0]
        elif op == "gin":
            z = a @ xx + (1.0 + m.gin_eps) * xx[:sg.nb]
            y = torch.relu(z @ ws[0]) @ ws[1]
        else:
            b = m.betas[layer - 1]
            z = (1.0 - m.alpha) * (a @ xx) + m.alpha * torch.from_numpy(f64(h0))[:sg.nb]
            y = (1.0 - b) * z + b * (z @ ws[0])
        return y if last else torch.relu(y)
    l_t = (f(x) - f((f64(x) + f64(eps)).astype(np.float32))).norm(dim=1).mean()    # x + eps is stored in fp32
    l_t.backward()
    assert abs(loss - float(l_t.detach())) <= 1e-5 * float(l_t.detach())
    got = dw if op == "gin" else (dw,)
    for gg, w in zip(got, ws):
        want = w.grad.numpy()
        assert np.abs(f64(gg) - want).max() <= 2e-5 * np.abs(want).max(), np.abs(f64(gg) - want).max() / np.abs(want).max()


def test_training_step_with_the_regulariser_adds_its_gradient():
    """loss + lambda * sum_l Eq. (3): the step's weights differ from the plain step's by -lr * lambda * the
    regulariser's gradient at the kept activations, layer by layer."""
    wl = _workload("gcn", n=160, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[0])
    labels = (np.arange(g.n) % 4).astype(np.int32)
    widths = wl.cfg.widths                                   # [f + 3, f + 1, f - 2]
    hist0 = [to_np(rng.normal_matrix(66, 1150, g.n, widths[1]))]
    eps = [to_np(rng.ball_matrix(66, 1151 + l, sg.nv, widths[l], 0.2)) for l in range(2)]
    lr, lam = 0.3, 0.7
    def own_model():                                         # a model with its own copies of the weights
        m = oracle_model(wl)
        m.weights = [w.copy() for w in m.weights]
        return m
    plain, reg = own_model(), own_model()
    h_a, h_b = [h.copy() for h in hist0], [h.copy() for h in hist0]
    omodel.gas_train_step(plain, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), h_a, labels, lr)
    omodel.gas_train_step(reg, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), h_b, labels, lr, reg_weight=lam, reg_eps=eps)
    # the regulariser's gradients at the same (pre-update) activations
    fresh = own_model()
    h_c = [h.copy() for h in hist0]
    _, (val, x0, h0, saved) = omodel.gas_batch_forward_kept(fresh, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), h_c)
    for l in (1, 2):
        x = omodel.layer_input(fresh, l, np.ascontiguousarray(n_id, dtype=np.int32), sg.nb, x0, h0, saved, h_c)
        _, dw = omodel.lipschitz_reg_grad(fresh, l, x, eps[l - 1], rp, cl, val, sg.nb)
        assert np.abs(dw).max() > 0
        diff = f64(plain.weights[l - 1]) - f64(reg.weights[l - 1])
        assert np.abs(diff - lr * lam * f64(dw)).max() <= 2e-6 * max(1.0, np.abs(lr * lam * f64(dw)).max())
    for a, b in zip(h_a, h_b):
        assert np.array_equal(a, b)                          # the forward pass (and so the pushes) is the same
