"""GPU parity of whole-model training passes of PNA and GAT (operator appendix) through the histories: the forward
output against the oracle end to end, and every gradient against the oracle's backward pass run on the activations
the library stored (a unit within rounding of zero, or two neighbours within rounding of a tie for min / max, may
fall either way in two correct forward passes; both sides therefore read masks and extremes off the same stored
tensors, and the gradients are compared at the usual bar).  Then gradient-descent steps over several batches."""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, rng
from oracle import model as omodel
from oracle import ops as oops
from tests.util import to_np, node_rel_err, max_rel_err

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}
# gradients pass through up to 3 L rounded tensors on the way down (same factor as for the other operators)
GTOL = {torch.float32: 2e-5, torch.bfloat16: 2e-2}


def _batch(g, bl, b, self_loops, f):
    from paper_2106_05609_amd import executor
    sg = batches.batch_subgraph(g, bl[b], self_loops)
    d = lambda t: t.to("cuda")
    bg = executor.BatchGraph(sg.nb, d(sg.n_id), d(sg.rowptr), d(sg.col), None, d(sg.colptr), d(sg.row), max_F=f,
                             normalise=False, csc_pos=d(sg.csc_perm).int())
    return sg, bg


@pytest.mark.parametrize("cfg_id,scale,dtype,f,f1", [(1, 0.1, torch.float32, 64, 32), (2, 0.01, torch.float32, 100, 28),
                                                      (4, 0.0005, torch.bfloat16, 64, 64)])
def test_pna_training_pass_matches_oracle(cfg_id, scale, dtype, f, f1):
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    L = 3
    x = rng.normal_matrix(cfg.seed, 1300, g.n, f, dtype=dtype)
    ws = [(rng.glorot_uniform(cfg.seed, 1301 + 2 * l, 2 * f, f1, dtype=dtype),
           rng.glorot_uniform(cfg.seed, 1302 + 2 * l, f + 9 * f1, f, dtype=dtype)) for l in range(L)]
    hist = [rng.normal_matrix(cfg.seed, 1310 + l, g.n, f, dtype=dtype) for l in range(L - 1)]
    hs_cpu, hs_gpu = [to_np(h).copy() for h in hist], [h.to("cuda") for h in hist]
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    d = lambda t: t.to("cuda")
    ws_gpu, ws_cpu = [(d(a), d(b)) for a, b in ws], [(to_np(a), to_np(b)) for a, b in ws]
    sg, bg = _batch(g, bl, 0, False, f)
    assert sg.nh > 0
    gout = rng.normal_matrix(cfg.seed, 1320, sg.nb, f, dtype=dtype)
    y, grads, kept = executor.pna_train_batch(ws_gpu, delta, bg, d(x), hs_gpu, d(gout))
    n_id, rp, cl = to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)
    want_y, _ = omodel.pna_batch_forward_kept(ws_cpu, delta, n_id, rp, cl, sg.nb, to_np(x), hs_cpu)
    tol = TOL[dtype] * (3 if dtype == torch.float32 else 1)          # as for the forward test of this model
    assert node_rel_err(to_np(y), want_y) <= tol
    for a, c in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), c) <= tol
    kept_cpu = [tuple(to_np(t) for t in layer) for layer in kept]
    want = omodel.pna_batch_backward(ws_cpu, delta, rp, cl, sg.nb, kept_cpu, to_np(gout))
    for l in range(L):
        for k in range(2):
            e = max_rel_err(to_np(grads[l][k]), want[l][k])
            assert e <= GTOL[dtype], (l, k, e)
    # run to run: fixed order everywhere
    y2, grads2, _ = executor.pna_train_batch(ws_gpu, delta, bg, d(x), hs_gpu, d(gout), do_push=False)
    assert torch.equal(y, y2) and all(torch.equal(a, b) for l in range(L) for a, b in zip(grads[l], grads2[l]))


@pytest.mark.parametrize("cfg_id,scale,dtype,f,heads", [(1, 0.1, torch.float32, 64, 1), (2, 0.01, torch.float32, 100, 5),
                                                         (4, 0.0005, torch.bfloat16, 128, 8), (1, 0.1, torch.float32, 64, 4)])
def test_gat_training_pass_matches_oracle(cfg_id, scale, dtype, f, heads):
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    L = 3
    x = rng.normal_matrix(cfg.seed, 1400, g.n, f, dtype=dtype)
    ws = [(rng.glorot_uniform(cfg.seed, 1401 + 3 * l, f, f, dtype=dtype), rng.normal(cfg.seed, 1402 + 3 * l, 0, f, dtype=dtype) * 0.3,
           rng.normal(cfg.seed, 1403 + 3 * l, 0, f, dtype=dtype) * 0.3) for l in range(L)]
    hist = [rng.normal_matrix(cfg.seed, 1410 + l, g.n, f, dtype=dtype) for l in range(L - 1)]
    hs_cpu, hs_gpu = [to_np(h).copy() for h in hist], [h.to("cuda") for h in hist]
    d = lambda t: t.to("cuda")
    ws_gpu, ws_cpu = [tuple(d(t) for t in w) for w in ws], [tuple(to_np(t) for t in w) for w in ws]
    sg, bg = _batch(g, bl, 0, True, f)
    assert sg.nh > 0
    gout = rng.normal_matrix(cfg.seed, 1420, sg.nb, f, dtype=dtype)
    y, grads, kept = executor.gat_train_batch(ws_gpu, bg, d(x), hs_gpu, d(gout), heads=heads)
    n_id, rp, cl = to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)
    want_y, _ = omodel.gat_batch_forward_kept(ws_cpu, n_id, rp, cl, sg.nb, to_np(x), hs_cpu, heads=heads)
    tol = TOL[dtype] * (3 if dtype == torch.float32 else 1)
    assert node_rel_err(to_np(y), want_y) <= tol
    kept_cpu = [tuple(to_np(t) for t in layer) for layer in kept]
    want = omodel.gat_batch_backward(ws_cpu, rp, cl, sg.nb, kept_cpu, to_np(gout), heads=heads)
    for l in range(L):
        e = max_rel_err(to_np(grads[l][0]), want[l][0])
        assert e <= GTOL[dtype], (l, e)
        # the two vector gradients are sums over all entries: against the size of the larger of the two
        scale = max(np.abs(want[l][1]).max(), np.abs(want[l][2]).max())
        for k in (1, 2):
            e = np.abs(to_np(grads[l][k]) - want[l][k]).max() / scale
            assert e <= GTOL[dtype], (l, k, e)
    y2, grads2, _ = executor.gat_train_batch(ws_gpu, bg, d(x), hs_gpu, d(gout), heads=heads, do_push=False)
    assert torch.equal(y, y2) and all(torch.equal(a, b) for l in range(L) for a, b in zip(grads[l], grads2[l]))


@pytest.mark.parametrize("kind", ["pna", "gat"])
def test_gradient_descent_steps_follow_the_oracle(kind):
    """Four optimisation steps over consecutive mini-batches (softmax cross-entropy on the in-batch nodes, plain
    gradient descent, histories pushed and pulled as in Algorithm 1), fp32: the losses and the final weights follow
    the oracle's run of the same steps."""
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    cfg = configs.config(1, 0.05)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    f, f1, L, classes, lr = 32, 16, 2, 8, 0.05
    dt = torch.float32
    x = rng.normal_matrix(cfg.seed, 1500, g.n, f, dtype=dt)
    labels = (rng.permutation(cfg.seed, 1501, g.n) % classes).to(torch.int32)
    widths = [f] * L + [classes]
    if kind == "pna":
        ws = [(rng.glorot_uniform(cfg.seed, 1510 + 2 * l, 2 * widths[l], f1, dtype=dt),
               rng.glorot_uniform(cfg.seed, 1511 + 2 * l, widths[l] + 9 * f1, widths[l + 1], dtype=dt)) for l in range(L)]
    else:
        ws = [(rng.glorot_uniform(cfg.seed, 1520 + 3 * l, widths[l], widths[l + 1], dtype=dt),
               rng.normal(cfg.seed, 1521 + 3 * l, 0, widths[l + 1], dtype=dt) * 0.3,
               rng.normal(cfg.seed, 1522 + 3 * l, 0, widths[l + 1], dtype=dt) * 0.3) for l in range(L)]
    d = lambda t: t.to("cuda")
    ws_gpu = [tuple(d(t).clone() for t in w) for w in ws]
    ws_cpu = [tuple(to_np(t).copy() for t in w) for w in ws]
    hs_gpu = [torch.zeros((g.n, f), dtype=dt, device="cuda") for _ in range(L - 1)]
    hs_cpu = [np.zeros((g.n, f), dtype=np.float32) for _ in range(L - 1)]
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    losses = []
    for step in range(4):
        sg, bg = _batch(g, bl, step % len(bl), kind == "gat", f)
        n_id, rp, cl = to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)
        lab = labels[sg.n_id[:sg.nb].long()].contiguous()
        loss_sum = torch.zeros(1, device="cuda")

        def loss_grad(y):
            gy = torch.empty_like(y)
            gas.gas_softmax_xent(y, d(lab), gy, torch.empty(sg.nb, device="cuda"), loss_sum, scale=1.0 / sg.nb)
            return gy
        if kind == "pna":
            _, grads, _ = executor.pna_train_batch(ws_gpu, delta, bg, d(x), hs_gpu, loss_grad)
            y_cpu, kept = omodel.pna_batch_forward_kept(ws_cpu, delta, n_id, rp, cl, sg.nb, to_np(x), hs_cpu)
        else:
            _, grads, _ = executor.gat_train_batch(ws_gpu, bg, d(x), hs_gpu, loss_grad)
            y_cpu, kept = omodel.gat_batch_forward_kept(ws_cpu, n_id, rp, cl, sg.nb, to_np(x), hs_cpu)
        _, want_loss, g_cpu = oops.softmax_xent(y_cpu, to_np(lab), scale=1.0 / sg.nb)
        if kind == "pna":
            grads_cpu = omodel.pna_batch_backward(ws_cpu, delta, rp, cl, sg.nb, kept, g_cpu)
        else:
            grads_cpu = omodel.gat_batch_backward(ws_cpu, rp, cl, sg.nb, kept, g_cpu)
        executor.sgd_update(ws_gpu, grads, lr)
        for l in range(L):
            for w, dw in zip(ws_cpu[l], grads_cpu[l]):
                oops.sgd_step(w, np.ascontiguousarray(dw), lr)
        got_loss = float(loss_sum.item()) / sg.nb
        losses.append(got_loss)
        assert abs(got_loss - want_loss / sg.nb) <= 1e-4 * abs(want_loss / sg.nb), (step, got_loss, want_loss / sg.nb)
    # weights after four steps: the two runs may differ in a ReLU mask or an extreme here and there (see the
    # module text), which moves single gradient entries; the weights stay together far more closely than the
    # steps moved them
    for l in range(L):
        for a, b, w0 in zip(ws_gpu[l], ws_cpu[l], ws[l]):
            moved = np.abs(b - to_np(w0)).max()
            assert moved > 0
            assert np.abs(to_np(a) - b).max() <= 1e-3 * moved + 1e-5 * np.abs(b).max(), (l, np.abs(to_np(a) - b).max(), moved)
