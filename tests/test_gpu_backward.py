"""GPU parity of the backward pass: the three new calls element by element against the oracle, then a whole
mini-batch forward + backward (all weight gradients) for GCN, GIN (fp32 and bf16) and GCNII."""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches, rng
from oracle import ops as oops, model as omodel
from tests.util import to_np, max_rel_err, node_rel_err, oracle_model
from tests.test_gpu_gas import _gpu_model, _gpu_batch

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
@pytest.mark.parametrize("M,F,ld", [(1000, 256, 256), (333, 100, 104), (50, 7, 7), (5000, 64, 64)])
def test_relu_bwd_bit_exact(gas, dtype, M, F, ld):
    gy = rng.normal_matrix(9, 600, M, ld, dtype=dtype)
    y = torch.relu(rng.normal_matrix(9, 601, M, ld, dtype=dtype))
    gp = torch.full((M, ld), 5.0, dtype=dtype, device="cuda")
    gas.gas_relu_bwd(dev(gy)[:, :F], dev(y)[:, :F], gp[:, :F])
    want = oops.relu_bwd(to_np(gy)[:, :F], to_np(y)[:, :F])
    assert np.array_equal(to_np(gp[:, :F]), want)
    if ld > F:
        assert (gp[:, F:] == 5.0).all()
    g2 = dev(gy.clone())
    gas.gas_relu_bwd(g2[:, :F], dev(y)[:, :F], g2[:, :F])           # in place
    assert np.array_equal(to_np(g2[:, :F]), want)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,K,N", [(1000, 256, 256), (4500, 256, 256), (4200, 128, 256), (257, 72, 200), (300, 15, 20),
                                    (5000, 64, 64), (129, 256, 128)])
def test_linear_bwd_input_parity(gas, dtype, M, K, N):
    """K = F_in, N = F_out of the forward transform: gp [M, N] -> gz [M, K]."""
    gp = rng.normal_matrix(9, 610, M, N, dtype=dtype)
    w = rng.glorot_uniform(9, 611, K, N, dtype=dtype)
    mask = torch.relu(rng.normal_matrix(9, 612, M, K, dtype=dtype))
    for use_mask in (False, True):
        gz = torch.full((M, K), float("nan"), dtype=dtype, device="cuda")
        gas.gas_linear_bwd_input(dev(gp), dev(w), gz, mask=dev(mask) if use_mask else None)
        want = oops.linear_bwd_input(to_np(gp), to_np(w), mask=to_np(mask) if use_mask else None)
        assert node_rel_err(to_np(gz), want) <= TOL[dtype], (M, K, N, use_mask)
        if use_mask:
            assert np.array_equal(to_np(gz) == 0, want == 0) or dtype == torch.bfloat16
    if K == N:
        gz = torch.full((M, K), float("nan"), dtype=dtype, device="cuda")
        gas.gas_linear_bwd_input(dev(gp), dev(w), gz, c_identity=0.6, c_weight=0.4)
        want = oops.linear_bwd_input(to_np(gp), to_np(w), c_identity=0.6, c_weight=0.4)
        assert node_rel_err(to_np(gz), want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,K,N", [(10000, 256, 256), (4097, 128, 256), (5000, 100, 64), (300, 15, 20), (9000, 72, 200),
                                    (1, 8, 8), (5000, 200, 136), (8193, 256, 192)])
def test_linear_bwd_weight_parity(gas, dtype, M, K, N):
    z = rng.normal_matrix(9, 620, M, K, dtype=dtype)
    gp = rng.normal_matrix(9, 621, M, N, dtype=dtype)
    dw = torch.full((K, N), float("nan"), device="cuda")
    nbytes = gas.gas_linear_bwd_weight_workspace(M, K, N)
    # one fp32 partial per slab of rows; slabs hold between 128 and 4096 rows, depending on the shape only
    assert nbytes % (K * N * 4) == 0 and -(-M // 4096) <= nbytes // (K * N * 4) <= -(-M // 128)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    gas.gas_linear_bwd_weight(dev(z), dev(gp), dw, ws, c_weight=0.5)
    want = oops.linear_bwd_weight(to_np(z), to_np(gp), c_weight=0.5)
    # the sum itself is fp32 with fp32 output in both dtypes: inputs are exact in bf16 too
    assert max_rel_err(to_np(dw), want) <= 1e-5, (dtype, M, K, N)
    dw2 = torch.full((K, N), float("nan"), device="cuda")
    gas.gas_linear_bwd_weight(dev(z), dev(gp), dw2, ws, c_weight=0.5)
    assert torch.equal(dw, dw2)                                      # fixed summation order
    with pytest.raises(gas.GasError):
        gas.gas_linear_bwd_weight(dev(z), dev(gp), dw, ws[: max(0, nbytes - 4)], c_weight=0.5)


@pytest.mark.parametrize("cfg_id,scale,dtype,fused", [(1, 0.1, None, False), (2, 0.02, None, False), (3, 0.05, None, False),
                                                       (4, 0.001, None, False), (4, 0.0006, torch.float32, False),
                                                       (3, 0.05, None, True), (3, 1.0, None, True), (0, 1.0, None, True),
                                                       (2, 0.02, None, True)])
def test_batch_backward_matches_oracle(cfg_id, scale, dtype, fused):
    """fused: halo rows read in place; configs 0 and 3 (narrow fp32) then run each layer's forward as one launch."""
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    if dtype is not None:
        cfg.dtype = dtype
    if cfg.op == "gcnii":
        cfg.widths = cfg.widths[:6]          # 4 propagation layers are enough for the chain rule
    wl = configs.build_workload(cfg)
    g = wl.graph
    hs_cpu = [to_np(h).copy() for h in configs.make_histories(cfg, init="normal")]
    hs_gpu = [h.to("cuda") for h in configs.make_histories(cfg, init="normal")]
    om, gm = oracle_model(wl), _gpu_model(wl)
    sg = batches.batch_subgraph(g, wl.batches[0], cfg.self_loops)
    bg = _gpu_batch(wl, sg, g.deg.to("cuda"))
    f_out = cfg.widths[-1]
    grad_out = rng.normal_matrix(cfg.seed, 630, sg.nb, f_out, dtype=cfg.dtype)
    y_gpu, grads_gpu, kept = executor.train_batch(gm, bg, wl.x.to("cuda"), hs_gpu, grad_out.to("cuda"), fused=fused)
    n_id, rp, cl = to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col)
    y_cpu, _ = omodel.gas_batch_train(om, n_id, rp, cl, sg.nb, to_np(g.deg), to_np(wl.x), hs_cpu, to_np(grad_out))
    tol = TOL[cfg.dtype]
    assert node_rel_err(to_np(y_gpu), y_cpu) <= tol                   # forward, end to end
    # The backward pass is a function of the activations the forward pass kept; a hidden unit within rounding
    # of zero may fall on either side of the ReLU in two correct forward passes, so both sides read the masks
    # off the SAME stored activations (the library's), and the gradients are then compared at the usual bar.
    val = oops.gcn_norm(rp, cl, n_id, to_np(g.deg)) if cfg.op != "gin" else None
    np_or_none = lambda t: None if t is None else to_np(t)
    saved = [(to_np(z), np_or_none(h), to_np(yl)) for z, h, yl in kept["layers"]]
    grads_cpu = omodel.gas_batch_backward(om, n_id, rp, cl, sg.nb, val, to_np(kept["x0"]), np_or_none(kept["h0"]),
                                          saved, to_np(grad_out))
    gtol = 2e-5 if cfg.dtype == torch.float32 else 2e-2      # gradients pass through up to 2L rounded tensors
    for l in range(om.n_layers):
        if cfg.op == "gin":
            for a, b in zip(grads_gpu[l], grads_cpu[l]):
                assert max_rel_err(to_np(a), b) <= gtol, (l, max_rel_err(to_np(a), b))
        else:
            assert max_rel_err(to_np(grads_gpu[l]), grads_cpu[l]) <= gtol, (l, max_rel_err(to_np(grads_gpu[l]), grads_cpu[l]))
    if cfg.op == "gcnii":
        assert max_rel_err(to_np(grads_gpu["w_in"]), grads_cpu["w_in"]) <= gtol
    if cfg.op == "gin":
        # gradient of every layer's eps: a sum over all in-batch rows and features, measured against the sum of
        # the magnitudes of its terms (the signed sum can cancel to anything)
        got, want = to_np(grads_gpu["eps"]).astype(np.float64), grads_cpu["eps"]
        for l in range(om.n_layers):
            x_in = to_np(kept["x0"]) if l == 0 else saved[l - 1][2]
            gz_mag = np.abs(oops.to_f64(np.asarray(x_in[:sg.nb]))).max() * sg.nb * x_in.shape[1]
            assert abs(got[l] - want[l]) <= gtol * max(abs(want[l]), 1e-6 * gz_mag), (l, got[l], want[l])


@pytest.mark.parametrize("cfg_id,scale", [(1, 0.1), (4, 0.001)])
def test_training_forward_in_place_gives_the_same_bits(cfg_id, scale):
    """train_batch with the halo rows read in place (no pull): outputs, gradients and histories bit for bit."""
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    wl = configs.build_workload(cfg)
    g = wl.graph
    gm = _gpu_model(wl)
    sg = batches.batch_subgraph(g, wl.batches[0], cfg.self_loops)
    bg = _gpu_batch(wl, sg, g.deg.to("cuda"))
    grad_out = rng.normal_matrix(cfg.seed, 640, sg.nb, cfg.widths[-1], dtype=cfg.dtype).to("cuda")
    res = []
    for fused in (False, True):
        hs = [h.to("cuda") for h in configs.make_histories(cfg, init="normal")]
        y, grads, _ = executor.train_batch(gm, bg, wl.x.to("cuda"), hs, grad_out, fused=fused)
        res.append((y, grads, hs))
    (y0, g0, h0), (y1, g1, h1) = res
    assert torch.equal(y0, y1)
    for l in range(gm.n_layers):
        a, b = g0[l], g1[l]
        for u, v in zip(a if isinstance(a, tuple) else (a,), b if isinstance(b, tuple) else (b,)):
            assert torch.equal(u, v)
    for u, v in zip(h0, h1):
        assert torch.equal(u, v)
