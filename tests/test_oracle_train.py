"""Pins for the oracle's loss, its gradient-descent update and a whole optimisation step (CPU only).

The loss is compared with torch's own cross-entropy and its autograd gradient in float64, with closed forms
(uniform logits, shift invariance, rows of the gradient sum to zero) and with a case that overflows a naive
exponential; the update with its closed form; the whole step on a batch that is the whole graph with one
full-batch gradient-descent step of a float64 autograd model; and several epochs of mini-batch steps with
the two things training must do on a learnable target: the loss falls and the exact full-batch model, run
with the trained weights, classifies far above chance."""
import numpy as np
import pytest
import torch

from gas_inputs import rng, configs, batches
from oracle import ops, model as omodel
from tests.util import to_np, f64, oracle_model
from tests.test_oracle_gas import _workload, _sub, _hist
from tests.test_oracle_backward import _torch_replica


def _logits(n=57, c=9, dtype=torch.float32, scale=3.0):
    a = rng.normal_matrix(21, 600, n, c, dtype=dtype) * scale
    lab = rng.randint(21, 601, torch.arange(n), c).to(torch.int32)
    return a, lab


def test_softmax_xent_matches_torch_cross_entropy_and_autograd():
    a, lab = _logits()
    lab[5] = -1
    lab[11] = -1
    scale = 1.0 / 55
    loss_rows, loss_sum, g = ops.softmax_xent(to_np(a), to_np(lab), scale=scale)
    t = a.double().requires_grad_()
    per_row = torch.nn.functional.cross_entropy(t, lab.long(), ignore_index=-1, reduction="none")
    (per_row.sum() * scale).backward()
    assert np.abs(loss_rows - per_row.detach().numpy()).max() <= 1e-6
    assert abs(loss_sum - per_row.sum().item()) <= 1e-9 * per_row.sum().item()
    assert np.abs(g - t.grad.numpy()).max() <= 1e-7 * np.abs(t.grad.numpy()).max()
    assert loss_rows[5] == 0 and not g[5].any() and not g[11].any()
    # the probabilities of a row sum to one: its gradient sums to zero
    assert np.abs(f64(g).sum(axis=1)).max() <= 1e-7


def test_softmax_xent_closed_forms():
    n, c = 6, 7
    lab = np.arange(n, dtype=np.int32) % c
    # equal logits: p = 1/C, loss = log C, gradient 1/C off the label and 1/C - 1 on it
    loss_rows, loss_sum, g = ops.softmax_xent(np.full((n, c), 2.5, np.float32), lab)
    assert np.allclose(loss_rows, np.log(c), rtol=1e-7) and np.isclose(loss_sum, n * np.log(c), rtol=1e-12)
    want = np.full((n, c), 1.0 / c)
    want[np.arange(n), lab] -= 1.0
    assert np.abs(g - want).max() <= 1e-7
    # adding a constant to a row changes nothing; logits of +-1000 neither overflow nor lose the answer
    a, lab2 = _logits(40, 5)
    r0 = ops.softmax_xent(to_np(a), to_np(lab2))
    r1 = ops.softmax_xent(to_np(a) + np.float32(64.0), to_np(lab2))
    assert np.abs(r0[0] - r1[0]).max() <= 2e-5 and np.abs(r0[2] - r1[2]).max() <= 2e-6
    big = np.array([[1000.0, -1000.0, 0.0], [-1000.0, 1000.0, 0.0]], np.float32)
    loss_rows, _, g = ops.softmax_xent(big, np.array([0, 0], np.int32))
    assert loss_rows[0] == 0.0 and loss_rows[1] == 2000.0
    assert np.array_equal(g, np.array([[0, 0, 0], [-1, 1, 0]], np.float32))
    # a confident wrong answer costs more than a confident right one, and the gradient pushes the label's logit up
    assert g[1, 0] < 0


def test_softmax_xent_bf16_storage():
    a, lab = _logits(64, 16, dtype=torch.bfloat16)
    loss_rows, loss_sum, g = ops.softmax_xent(to_np(a), to_np(lab), scale=0.25)
    t = a.double().requires_grad_()
    per_row = torch.nn.functional.cross_entropy(t, lab.long(), reduction="none")
    (per_row.sum() * 0.25).backward()
    assert np.abs(loss_rows - per_row.detach().numpy()).max() <= 1e-6 * (1 + per_row.max().item())
    want = to_np(t.grad.to(torch.bfloat16))            # torch's own round-to-nearest-even of the exact gradient
    assert g.dtype == np.uint16 and np.array_equal(g, want)


def test_sgd_step_closed_form():
    w = to_np(rng.normal_matrix(22, 610, 13, 7))
    dw = to_np(rng.normal_matrix(22, 611, 13, 7))
    w0 = w.copy()
    ops.sgd_step(w, dw, 0.0, 0.3)
    assert np.array_equal(w, w0)                       # zero learning rate: nothing moves
    ops.sgd_step(w, dw, 0.05, 0.0)
    assert np.array_equal(w, (f64(w0) - 0.05 * f64(dw)).astype(np.float32))
    w = w0.copy()
    ops.sgd_step(w, dw, 0.05, 0.01)
    assert np.array_equal(w, (f64(w0) - 0.05 * (f64(dw) + 0.01 * f64(w0))).astype(np.float32))
    # zero gradient with decay shrinks every weight by the same factor
    w = w0.copy()
    ops.sgd_step(w, np.zeros_like(dw), 0.5, 0.1)
    assert np.abs(w - 0.95 * f64(w0)).max() <= 1e-7
    # bf16 storage: one rounding of the exact result
    wb = rng.normal_matrix(22, 612, 8, 8, dtype=torch.bfloat16)
    wbn = to_np(wb).copy()
    ops.sgd_step(wbn, dw[:8, :7].copy().repeat(2, axis=1)[:, :8].copy(), 0.1, 0.0)
    want = (wb.double() - 0.1 * torch.from_numpy(f64(dw[:8, :7].repeat(2, axis=1)[:, :8]))).to(torch.bfloat16)
    assert np.array_equal(wbn, to_np(want))


def test_gradient_clipping_matches_the_library_routine_and_its_closed_forms():
    """Clipping by the global norm (Section 3): the scale and the clipped update against torch's clip_grad_norm_
    followed by a plain step, in float64; a norm below the bound changes nothing; above it the clipped gradients
    have exactly the bound as their norm."""
    shapes = [(13, 7), (7, 5), (5, 5)]
    ws = [to_np(rng.normal_matrix(23, 620 + i, *sh)) for i, sh in enumerate(shapes)]
    dws = [to_np(rng.normal_matrix(23, 630 + i, *sh)) * (3.0 + i) for i, sh in enumerate(shapes)]
    total = float(np.sqrt(sum((f64(d) ** 2).sum() for d in dws)))
    for max_norm in (0.5, total * 2.0):
        params = [torch.from_numpy(f64(w)).requires_grad_() for w in ws]
        for p, d in zip(params, dws):
            p.grad = torch.from_numpy(f64(d)).clone()
        torch.nn.utils.clip_grad_norm_(params, max_norm)
        scale = ops.clip_scale([ops.sq_norm(d) for d in dws], max_norm)
        for p, d in zip(params, dws):
            assert np.abs(p.grad.numpy() - scale * f64(d)).max() <= 1e-12 * np.abs(f64(d)).max()
        if max_norm > total:
            assert scale == 1.0
        else:
            clipped = float(np.sqrt(sum(((scale * f64(d)) ** 2).sum() for d in dws)))
            assert abs(clipped - max_norm) <= 1e-5 * max_norm
        # the model-level update: every matrix moves by lr * scale * gradient
        m = omodel.Model("gcn", [w.copy() for w in ws])
        omodel.apply_sgd(m, {i: d for i, d in enumerate(dws)}, 0.1, 0.0, max_norm)
        for w_new, w0, p in zip(m.weights, ws, params):
            want = (f64(w0) - 0.1 * p.grad.numpy()).astype(np.float32)
            assert np.abs(f64(w_new) - f64(want)).max() <= 2e-7 * max(1.0, np.abs(f64(want)).max())
    assert abs(ops.sq_norm(np.array([3.0, 4.0], dtype=np.float32)) - 25.0) == 0.0


@pytest.mark.parametrize("op", ["gcn", "gin", "gcnii"])
def test_whole_graph_step_is_one_full_batch_gradient_descent_step(op):
    """With the whole graph as the batch there is no halo and no history is read: the step must be plain
    gradient descent on the exact model's cross-entropy (autograd, float64)."""
    wl = _workload(op, layers=2, n=192)
    g, m = wl.graph, oracle_model(wl)
    whole = torch.cat(wl.batches)
    sg, n_id, rp, cl = _sub(wl, whole)
    assert sg.nh == 0 and sg.nb == g.n
    f_out = m.weights[-1][1].shape[1] if op == "gin" else m.weights[-1].shape[1]
    labels = to_np(configs.block_labels(g, f_out, 5, unlabelled=0.25))
    lab_b = labels[n_id]
    n_lab = int((lab_b >= 0).sum())
    assert 0 < n_lab < g.n
    lr, wd = 0.2, 0.01
    hist = _hist(wl)
    # float64 autograd: the loss's gradient at the output, then the chain rule through the replica
    y_t, _ = _torch_replica(wl, m, sg, n_id, rp, cl, hist, np.zeros((g.n, f_out)))
    p = torch.softmax(torch.from_numpy(y_t), dim=1).numpy()
    g_out = p.copy()
    g_out[np.arange(g.n), np.maximum(lab_b, 0)] -= 1.0
    g_out[lab_b < 0] = 0.0
    g_out /= n_lab
    _, grads_t = _torch_replica(wl, m, sg, n_id, rp, cl, hist, g_out)
    want_loss = float(-np.log(p[np.arange(g.n), np.maximum(lab_b, 0)])[lab_b >= 0].sum() / n_lab)

    before = [tuple(w.copy() for w in ws) if op == "gin" else ws.copy() for ws in m.weights]
    w_in0 = None if m.w_in is None else m.w_in.copy()
    loss = omodel.gas_train_step(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), hist, labels, lr, wd)
    assert abs(loss - want_loss) <= 1e-5 * want_loss

    def close(new, old, grad):
        want = f64(old) - lr * (grad + wd * f64(old))
        moved = np.abs(want - f64(old)).max()
        return np.abs(f64(new) - want).max() <= 1e-4 * moved + 1e-7 and moved > 1e-5
    for l in range(m.n_layers):
        if op == "gin":
            assert close(m.weights[l][0], before[l][0], grads_t[l][0]) and close(m.weights[l][1], before[l][1], grads_t[l][1])
        else:
            assert close(m.weights[l], before[l], grads_t[l]), l
    if op == "gcnii":
        assert close(m.w_in, w_in0, grads_t["w_in"])


def learnable_workload(op="gcn", n=384, f=12, dtype=torch.float32):
    """8 communities, 4 classes, batches of 2 blocks, features that carry the class weakly."""
    cfg = configs.config(0)
    cfg.op, cfg.n, cfg.n_blocks, cfg.seed, cfg.blocks_per_batch, cfg.dtype = op, n, 8, 1, 2, dtype
    cfg.graph = dict(kind="sbm_bernoulli", p_in=0.1, p_out=0.005)
    cfg.self_loops = op != "gin"
    cfg.widths = [f + 3, f + 1, 4]
    if op == "gcnii":                 # one width throughout: the f-wide output serves as logits, 4 of them used
        cfg.widths, cfg.alpha = [f + 3, f, f, f], 0.1
    if op == "gin":
        cfg.gin_hidden, cfg.gin_eps = f + 5, 0.0
    wl = configs.build_workload(cfg)
    wl.x = configs.class_features(wl.graph, 4, f + 3, 7, 0.5, dtype=dtype)
    labels = configs.block_labels(wl.graph, 4, 7, unlabelled=0.3)
    truth = configs.block_labels(wl.graph, 4, 7)
    return wl, labels, truth


def test_mini_batch_training_learns_the_block_labels():
    wl, labels, truth = learnable_workload()
    g, m = wl.graph, oracle_model(wl)
    labels, truth = to_np(labels), to_np(truth)
    assert set(np.unique(labels)) == {-1, 0, 1, 2, 3} and len(wl.batches) == 4
    hist = _hist(wl)
    subs = [_sub(wl, b) for b in wl.batches]
    rowptr, col = to_np(g.rowptr).astype(np.int32), to_np(g.col)

    def accuracy():
        y = omodel.full_batch_forward(m, rowptr, col, to_np(wl.x))[-1]
        return float((y.argmax(axis=1) == truth)[labels < 0].mean())      # nodes the loss never saw
    acc0 = accuracy()
    losses = []
    for epoch in range(20):
        tot = 0.0
        for sg, n_id, rp, cl in subs:
            tot += omodel.gas_train_step(m, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), hist, labels, 1.0, 0.0)
        losses.append(tot / len(subs))
    assert losses[0] > 1.0 and losses[-1] < 0.1 * losses[0], losses
    assert acc0 < 0.6 and accuracy() > 0.9, (acc0, accuracy())
