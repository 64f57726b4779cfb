"""GPU parity of the loss, the gradient-descent update and whole optimisation steps of Algorithm 1's loop
body: call by call against the oracle, then epochs of mini-batch steps (weights, histories and losses after
the epoch against the oracle's), then the property training must have on a learnable target."""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, rng
from oracle import ops as oops, model as omodel
from tests.util import to_np, max_rel_err, node_rel_err, oracle_model
from tests.test_gpu_gas import _gpu_model, _gpu_batch
from tests.test_oracle_train import learnable_workload

pytestmark = pytest.mark.gpu
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


@pytest.fixture(scope="module")
def gas():
    import paper_2106_05609_amd as g
    g.lib()
    return g


def dev(t):
    return t.to("cuda")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,C,ld", [(1000, 64, 64), (333, 100, 104), (50, 1, 1), (5000, 256, 256), (77, 4, 4),
                                     (130, 300, 300), (0, 8, 8)])
def test_softmax_xent_parity(gas, dtype, M, C, ld):
    a = rng.normal_matrix(10, 700, M, ld, dtype=dtype) * 4.0
    lab = rng.randint(10, 701, torch.arange(M), C + 1).to(torch.int32) - 1          # -1 (unlabelled) .. C-1
    scale = 1.0 / max(1, M)
    g = torch.full((M, ld), 7.0, dtype=dtype, device="cuda")
    loss_rows = torch.full((M,), float("nan"), device="cuda")
    loss_sum = torch.full((1,), float("nan"), device="cuda")
    gas.gas_softmax_xent(dev(a)[:, :C], dev(lab), g[:, :C], loss_rows, loss_sum, scale=scale)
    if M == 0:
        assert float(loss_sum) == 0.0                  # the empty sum, and no kernel ran on no rows
        return
    want_rows, want_sum, want_g = oops.softmax_xent(to_np(a)[:, :C], to_np(lab), scale=scale)
    assert np.abs(to_np(loss_rows) - want_rows).max() <= 1e-5 * max(1.0, np.abs(want_rows).max())
    assert abs(float(loss_sum) - want_sum) <= 1e-5 * max(1.0, want_sum)
    # a gradient row is scale * (p - onehot): its rounding error is relative to scale (p and onehot are of order one),
    # not to what is left of a confident row after the subtraction
    assert node_rel_err(to_np(g[:, :C]), want_g, scale=np.full(M, scale)) <= TOL[dtype] or not want_g.any()
    unl = to_np(lab) < 0
    assert not to_np(g[:, :C])[unl].any() and not to_np(loss_rows)[unl].any()
    if ld > C:
        assert (g[:, C:] == 7.0).all()
    # a label beyond the last class is skipped like an unlabelled row, never read out of the row
    lab2 = lab.clone()
    lab2[:] = C
    gas.gas_softmax_xent(dev(a)[:, :C], dev(lab2), g[:, :C], loss_rows, loss_sum)
    assert float(loss_sum) == 0.0 and not to_np(g[:, :C]).any()
    with pytest.raises(gas.GasError):
        gas.gas_softmax_xent(g[:, :C], dev(lab), g[:, :C], loss_rows)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [(256, 256), (100, 47), (1, 1), (3, 1000)])
def test_sgd_step_parity(gas, dtype, shape):
    w = rng.glorot_uniform(10, 710, shape[0], shape[1], dtype=dtype)
    dw = rng.normal_matrix(10, 711, shape[0], shape[1]) * 0.1
    for lr, wd in ((0.05, 0.0), (0.3, 0.01), (0.0, 0.5)):
        w_dev = dev(w.clone())
        gas.gas_sgd_step(w_dev, dev(dw), lr, wd)
        want = to_np(w).copy()
        oops.sgd_step(want, to_np(dw), lr, wd)
        if lr == 0.0:
            assert np.array_equal(to_np(w_dev), to_np(w))
        assert max_rel_err(to_np(w_dev), want) <= (2e-7 if dtype == torch.float32 else 2 ** -8)


def _both_models(wl):
    cfg = wl.cfg
    hs_cpu = [to_np(h).copy() for h in configs.make_histories(cfg, init="zeros")]
    hs_gpu = [h.to("cuda") for h in configs.make_histories(cfg, init="zeros")]
    return oracle_model(wl), _gpu_model(wl), hs_cpu, hs_gpu


def _weights(m):
    out = []
    for w in m.weights:
        out += list(w) if isinstance(w, (tuple, list)) else [w]
    if m.w_in is not None:
        out.append(m.w_in)
    return out


@pytest.mark.parametrize("op,dtype", [("gcn", torch.float32), ("gin", torch.float32), ("gin", torch.bfloat16),
                                       ("gcnii", torch.float32)])
def test_training_epochs_match_oracle(gas, op, dtype):
    """Epochs over all four batches: every step's loss, and the weights and histories afterwards.  Two epochs
    in fp32; one, with a smaller step, in bf16, where a descent trajectory amplifies the storage rounding of
    every weight and history row from step to step (the per-call bar is what the other tests hold)."""
    from paper_2106_05609_amd import executor
    wl, labels, _ = learnable_workload(op, dtype=dtype)
    g = wl.graph
    om, gm, hs_cpu, hs_gpu = _both_models(wl)
    deg_dev, x_dev, lab_dev = g.deg.to("cuda"), wl.x.to("cuda"), labels.to("cuda")
    lr, wd = (0.05 if op == "gin" else 0.5), 0.001
    if dtype == torch.bfloat16:
        lr = 0.01
    tol = 2e-5 if dtype == torch.float32 else 2e-2
    for epoch in range(2 if dtype == torch.float32 else 1):
        for b in wl.batches:
            sg = batches.batch_subgraph(g, b, wl.cfg.self_loops)
            bg = _gpu_batch(wl, sg, deg_dev)
            lab_b = lab_dev[bg.n_id[:sg.nb].long()].contiguous()
            loss_sum, n_lab, _, _ = executor.train_step(gm, bg, x_dev, hs_gpu, lab_b, lr, wd)
            want = omodel.gas_train_step(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(g.deg),
                                         to_np(wl.x), hs_cpu, to_np(labels), lr, wd)
            got = float(loss_sum) / n_lab
            assert abs(got - want) <= (1e-4 if dtype == torch.float32 else 2e-2) * max(1.0, want), (epoch, got, want)
    for a, b in zip(_weights(gm), _weights(om)):
        assert max_rel_err(to_np(a), b) <= tol, max_rel_err(to_np(a), b)
    for a, b in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), b) <= tol, node_rel_err(to_np(a), b)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gradient_clipping_parity(gas, dtype):
    """Section 3's gradient clipping: squared norms, the common factor formed on the device, the clipped update."""
    shapes = [(256, 256), (100, 36), (8, 8), (1, 5)]
    ws = [rng.normal_matrix(15, 700 + i, *sh, dtype=dtype) for i, sh in enumerate(shapes)]
    dws = [rng.normal_matrix(15, 710 + i, *sh) * (0.5 + i) for i, sh in enumerate(shapes)]
    sq = torch.full((len(shapes),), float("nan"), device="cuda")
    for k, d in enumerate(dws):
        gas.gas_sq_norm(d.to("cuda"), sq[k:k + 1])
    want_sq = np.array([oops.sq_norm(to_np(d)) for d in dws])
    assert np.abs(to_np(sq) - want_sq).max() <= 1e-6 * want_sq.max()
    total = float(np.sqrt(want_sq.sum()))
    for max_norm in (0.25 * total, 4.0 * total):
        scale = oops.clip_scale(want_sq, max_norm)
        for w, d in zip(ws, dws):
            wd = w.to("cuda").clone()
            gas.gas_sgd_step_clipped(wd, d.to("cuda"), 0.1, sq, max_norm, weight_decay=0.01)
            wo = to_np(w).copy()
            oops.sgd_step(wo, np.ascontiguousarray((to_np(d).astype(np.float64) * scale).astype(np.float32)), 0.1, 0.01)
            assert max_rel_err(to_np(wd), wo) <= TOL[dtype]
            if max_norm > total:                     # no clipping: the bits of the plain step
                wp = w.to("cuda").clone()
                gas.gas_sgd_step(wp, d.to("cuda"), 0.1, weight_decay=0.01)
                assert torch.equal(wp, wd)
    with pytest.raises(gas.GasError):
        gas.gas_sgd_step_clipped(ws[0].to("cuda"), dws[0].to("cuda"), 0.1, sq, 0.0)


def test_training_step_with_clipping_matches_oracle(gas):
    from paper_2106_05609_amd import executor
    wl, labels, _ = learnable_workload("gcn", dtype=torch.float32)
    g = wl.graph
    om, gm, hs_cpu, hs_gpu = _both_models(wl)
    deg_dev, x_dev, lab_dev = g.deg.to("cuda"), wl.x.to("cuda"), labels.to("cuda")
    for b in wl.batches[:2]:
        sg = batches.batch_subgraph(g, b, wl.cfg.self_loops)
        bg = _gpu_batch(wl, sg, deg_dev)
        lab_b = lab_dev[bg.n_id[:sg.nb].long()].contiguous()
        loss_sum, n_lab, _, grads = executor.train_step(gm, bg, x_dev, hs_gpu, lab_b, 0.5, 0.001, max_norm=0.05)
        norm = float(np.sqrt(sum(oops.sq_norm(to_np(grads[l])) for l in range(gm.n_layers))))
        assert norm > 0.05                           # the bound is active in this case
        want = omodel.gas_train_step(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(g.deg),
                                     to_np(wl.x), hs_cpu, to_np(labels), 0.5, 0.001, max_norm=0.05)
        assert abs(float(loss_sum) / n_lab - want) <= 1e-4 * max(1.0, want)
    for a, b in zip(_weights(gm), _weights(om)):
        assert max_rel_err(to_np(a), b) <= 2e-5


@pytest.mark.parametrize("op,dtype", [("gcn", torch.float32), ("gin", torch.bfloat16)])
def test_training_on_the_gpu_learns(gas, op, dtype):
    """What holds at any size: the loss falls and nodes the loss never saw are classified far above chance by
    a forward pass with the trained weights."""
    from paper_2106_05609_amd import executor
    wl, labels, truth = learnable_workload(op, dtype=dtype)
    g = wl.graph
    _, gm, _, hs_gpu = _both_models(wl)
    deg_dev, x_dev, lab_dev = g.deg.to("cuda"), wl.x.to("cuda"), labels.to("cuda")
    bgs = []
    for b in wl.batches:
        sg = batches.batch_subgraph(g, b, wl.cfg.self_loops)
        bgs.append((sg, _gpu_batch(wl, sg, deg_dev)))
    losses = []
    lr = 1.0 if op == "gcn" else 0.05
    for epoch in range(20):
        tot = 0.0
        for sg, bg in bgs:
            lab_b = lab_dev[bg.n_id[:sg.nb].long()].contiguous()
            loss_sum, n_lab, _, _ = executor.train_step(gm, bg, x_dev, hs_gpu, lab_b, lr)
            tot += float(loss_sum) / n_lab
        losses.append(tot / len(bgs))
    assert losses[-1] < 0.3 * losses[0], losses
    hit = tot_n = 0
    for sg, bg in bgs:
        y = executor.forward_batch(gm, bg, x_dev, hs_gpu, do_push=False)
        ids = bg.n_id[:sg.nb].long()
        held = lab_dev[ids] < 0
        hit += int(((y.float().argmax(dim=1) == truth.to("cuda")[ids]) & held).sum())
        tot_n += int(held.sum())
    assert hit / tot_n > 0.85, hit / tot_n


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,F,ld", [(1000, 256, 256), (333, 100, 104), (50, 7, 7), (0, 8, 8)])
def test_axpy_and_row_distance_parity(gas, dtype, M, F, ld):
    x = rng.normal_matrix(13, 1200, M, ld, dtype=dtype)
    e = rng.normal_matrix(13, 1201, M, ld, dtype=dtype)
    y = torch.full((M, ld), 3.0, dtype=dtype, device="cuda")
    gas.gas_axpy(dev(x)[:, :F], dev(e)[:, :F], y[:, :F], 0.25)
    dist = torch.full((M,), float("nan"), device="cuda")
    total = torch.full((1,), float("nan"), device="cuda")
    gas.gas_row_distance(dev(x)[:, :F], y[:, :F], dist, total)
    if M == 0:
        assert float(total) == 0.0
        return
    want = oops.axpy(to_np(x)[:, :F], to_np(e)[:, :F], 0.25)
    if dtype == torch.float32:
        assert node_rel_err(to_np(y[:, :F]), want) <= 2e-7
    else:
        assert np.array_equal(to_np(y[:, :F]), want)            # one rounding of an exact fp32 result on both sides
    if ld > F:
        assert (y[:, F:] == 3.0).all()
    d_want, t_want = oops.row_distance(to_np(x)[:, :F], to_np(y[:, :F]))
    assert np.abs(to_np(dist) - d_want).max() <= 1e-5 * d_want.max()
    assert abs(float(total) - t_want) <= 1e-5 * t_want


@pytest.mark.parametrize("op,dtype,layer", [("gcn", torch.float32, 1), ("gcn", torch.float32, 2), ("gin", torch.float32, 1),
                                             ("gin", torch.bfloat16, 1), ("gcnii", torch.float32, 2)])
def test_lipschitz_regulariser_matches_oracle(gas, op, dtype, layer):
    """Eq. (3): one layer applied to the mini-batch tensor and to its perturbed copy, mean row distance."""
    from paper_2106_05609_amd import executor
    wl, _, _ = learnable_workload(op, dtype=dtype)
    g = wl.graph
    om, gm = oracle_model(wl), _gpu_model(wl)
    sg = batches.batch_subgraph(g, wl.batches[1], wl.cfg.self_loops)
    bg = _gpu_batch(wl, sg, g.deg.to("cuda"))
    n_id, rp, cl = to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)
    val = oops.gcn_norm(rp, cl, n_id, to_np(g.deg)) if op != "gin" else None
    f_in = (om.weights[layer - 1][0] if op == "gin" else om.weights[layer - 1]).shape[0]
    x = rng.normal_matrix(14, 1210, sg.nv, f_in, dtype=dtype)
    eps = rng.ball_matrix(14, 1211, sg.nv, f_in, 0.5, dtype=dtype)
    h0 = torch.relu(rng.normal_matrix(14, 1212, sg.nv, f_in, dtype=dtype)) if op == "gcnii" else None
    total, nb = executor.lipschitz_reg(gm, layer, bg, x.to("cuda"), eps.to("cuda"), None if h0 is None else h0.to("cuda"))
    want = omodel.lipschitz_reg(om, layer, to_np(x), to_np(eps), rp, cl, val, sg.nb, None if h0 is None else to_np(h0))
    got = float(total) / nb
    # the loss is a difference of two rounded outputs: its error is the outputs' tolerance relative to their size
    y = omodel.layer_forward(om, layer, to_np(x), None if h0 is None else to_np(h0), rp, cl, val, sg.nb)
    scale = np.abs(oops.to_f64(y)).max() * np.sqrt(y.shape[1])
    assert want > 0 and abs(got - want) <= TOL[dtype] * scale, (got, want, scale)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,F,ld", [(1000, 256, 256), (333, 100, 104), (50, 7, 7), (0, 8, 8), (4099, 512, 512), (777, 64, 72),
                                    (129, 520, 520), (65, 8, 8), (1, 16, 16)])
def test_row_dot_parity(gas, dtype, M, F, ld):
    """gas_row_dot (the reduction behind the gradient of GIN's eps) against the oracle's float64 inner products."""
    a = rng.normal_matrix(18, 1400, M, ld, dtype=dtype)
    b = rng.normal_matrix(18, 1401, M, ld, dtype=dtype)
    dot = torch.full((max(M, 1),), float("nan"), device="cuda")
    total = torch.full((1,), float("nan"), device="cuda")
    gas.gas_row_dot(a.to("cuda")[:, :F], b.to("cuda")[:, :F], dot, total)
    if M == 0:
        assert float(total) == 0.0
        return
    want, want_sum = oops.row_dot(to_np(a)[:, :F], to_np(b)[:, :F])
    mag = (np.abs(oops.to_f64(to_np(a)[:, :F])) * np.abs(oops.to_f64(to_np(b)[:, :F]))).sum(axis=1)
    assert (np.abs(to_np(dot[:M]) - want) <= 2e-6 * mag + 1e-30).all()
    assert abs(float(total) - want_sum) <= 1e-6 * mag.sum()
    d2, t2 = torch.empty_like(dot), torch.empty_like(total)
    gas.gas_row_dot(a.to("cuda")[:, :F], b.to("cuda")[:, :F], d2, t2)
    assert torch.equal(dot[:M], d2[:M]) and torch.equal(total, t2)              # fixed order


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,F,ld", [(1000, 256, 256), (333, 100, 104), (50, 7, 7), (0, 8, 8)])
def test_row_distance_gradient_parity(gas, dtype, M, F, ld):
    a = rng.normal_matrix(16, 1300, M, ld, dtype=dtype)
    b = rng.normal_matrix(16, 1301, M, ld, dtype=dtype)
    if M > 5:
        b[5] = a[5]                                          # equal rows: zero gradient, no division by zero
    g = torch.full((M, ld), float("nan"), dtype=dtype, device="cuda")
    gas.gas_row_distance_bwd(a.to("cuda")[:, :F], b.to("cuda")[:, :F], g[:, :F], scale=0.125)
    if M == 0:
        return
    want = oops.row_distance_bwd(to_np(a)[:, :F], to_np(b)[:, :F], 0.125)
    assert node_rel_err(to_np(g[:, :F]), want) <= TOL[dtype]
    assert not to_np(g[5, :F].float()).any()


@pytest.mark.parametrize("op,layer", [("gcn", 1), ("gcn", 2), ("gin", 1), ("gcnii", 2)])
def test_lipschitz_regulariser_gradient_matches_oracle(gas, op, layer):
    """Eq. (3) differentiated with respect to the layer's weights: loss and gradient against the oracle (itself
    pinned to float64 autograd).  fp32: the gradient divides by the distance of two rounded outputs, which in
    bf16 storage is known to a few per cent only, so the bf16 bar is held call by call instead."""
    from paper_2106_05609_amd import executor
    wl, _, _ = learnable_workload(op, dtype=torch.float32)
    g = wl.graph
    om, gm = oracle_model(wl), _gpu_model(wl)
    sg = batches.batch_subgraph(g, wl.batches[1], wl.cfg.self_loops)
    bg = _gpu_batch(wl, sg, g.deg.to("cuda"))
    n_id, rp, cl = to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)
    val = oops.gcn_norm(rp, cl, n_id, to_np(g.deg)) if op != "gin" else None
    f_in = (om.weights[layer - 1][0] if op == "gin" else om.weights[layer - 1]).shape[0]
    x = rng.normal_matrix(17, 1310, sg.nv, f_in)
    eps = rng.ball_matrix(17, 1311, sg.nv, f_in, 0.5)
    h0 = torch.relu(rng.normal_matrix(17, 1312, sg.nv, f_in)) if op == "gcnii" else None
    total, nb, dw = executor.lipschitz_reg_grad(gm, layer, bg, x.to("cuda"), eps.to("cuda"),
                                                None if h0 is None else h0.to("cuda"))
    loss, want = omodel.lipschitz_reg_grad(om, layer, to_np(x), to_np(eps), rp, cl, val, sg.nb,
                                           None if h0 is None else to_np(h0))
    assert abs(float(total) / nb - loss) <= 1e-4 * loss
    for a, b in zip(dw if op == "gin" else (dw,), want if op == "gin" else (want,)):
        assert max_rel_err(to_np(a), b) <= 2e-4, max_rel_err(to_np(a), b)


@pytest.mark.parametrize("op", ["gcn", "gin"])
def test_training_step_with_the_regulariser_matches_oracle(gas, op):
    """loss + lambda * sum_l Eq. (3) in the training step: two steps on two batches, weights and histories."""
    from paper_2106_05609_amd import executor
    wl, labels, _ = learnable_workload(op, dtype=torch.float32)
    g = wl.graph
    om, gm, hs_cpu, hs_gpu = _both_models(wl)
    deg_dev, x_dev, lab_dev = g.deg.to("cuda"), wl.x.to("cuda"), labels.to("cuda")
    lr, lam = (0.05 if op == "gin" else 0.5), 0.3
    for k, b in enumerate(wl.batches[:2]):
        sg = batches.batch_subgraph(g, b, wl.cfg.self_loops)
        bg = _gpu_batch(wl, sg, deg_dev)
        lab_b = lab_dev[bg.n_id[:sg.nb].long()].contiguous()
        widths = [(w[0] if op == "gin" else w).shape[0] for w in om.weights]
        eps = [rng.ball_matrix(18, 1400 + 10 * k + l, sg.nv, f, 0.3) for l, f in enumerate(widths)]
        loss_sum, n_lab, _, _ = executor.train_step(gm, bg, x_dev, hs_gpu, lab_b, lr, reg_weight=lam,
                                                    reg_eps=[e.to("cuda") for e in eps])
        want = omodel.gas_train_step(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(g.deg),
                                     to_np(wl.x), hs_cpu, to_np(labels), lr, reg_weight=lam,
                                     reg_eps=[to_np(e) for e in eps])
        assert abs(float(loss_sum) / n_lab - want) <= 1e-4 * max(1.0, want)
    for a, b in zip(_weights(gm), _weights(om)):
        assert max_rel_err(to_np(a), b) <= 1e-4, max_rel_err(to_np(a), b)
    for a, b in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), b) <= 2e-5
