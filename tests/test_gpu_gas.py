"""GPU parity of the whole mini-batch execution (all layers, pushes and pulls
through the C ABI) against the oracle's Algorithm-1 executor, for the five
benchmark configurations (full size where the oracle finishes in seconds,
scaled node counts otherwise; the full-size cases are in test_gpu_fullsize)."""
import numpy as np
import pytest
import torch

from gas_inputs import configs, batches
from oracle import model as omodel
from tests.util import to_np, node_rel_err, oracle_model

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def _gpu_model(wl):
    from paper_2106_05609_amd import executor
    d = lambda t: t.to("cuda")
    ws = [(d(a), d(b)) for a, b in wl.weights] if wl.cfg.op == "gin" else [d(w) for w in wl.weights]
    return executor.Model(wl.cfg.op, ws, None if wl.w_in is None else d(wl.w_in), wl.cfg.alpha, wl.cfg.gin_eps)


def _gpu_batch(wl, sg, deg_dev):
    from paper_2106_05609_amd import executor
    d = lambda t: t.to("cuda")
    return executor.BatchGraph(sg.nb, d(sg.n_id), d(sg.rowptr), d(sg.col), deg_dev, d(sg.colptr), d(sg.row),
                               max_F=max(wl.cfg.widths + [wl.cfg.gin_hidden]), normalise=wl.cfg.op != "gin")


def _run_both(wl, batch_ids, hist_init, sweeps=1, check_layers=True):
    from paper_2106_05609_amd import executor
    cfg, g = wl.cfg, wl.graph
    hs_cpu = [to_np(h).copy() for h in configs.make_histories(cfg, init=hist_init)]
    hs_gpu = [torch.from_numpy(h.view(np.int16) if h.dtype == np.uint16 else h).to("cuda") for h in hs_cpu]
    if cfg.dtype == torch.bfloat16:
        hs_gpu = [h.view(torch.bfloat16) for h in hs_gpu]
    om, gm = oracle_model(wl), _gpu_model(wl)
    x_dev, deg_dev = wl.x.to("cuda"), g.deg.to("cuda")
    worst = 0.0
    for sweep in range(sweeps):
        for b in batch_ids:
            sg = batches.batch_subgraph(g, wl.batches[b], cfg.self_loops)
            bg = _gpu_batch(wl, sg, deg_dev)
            y_gpu, layers_gpu = executor.forward_batch(gm, bg, x_dev, hs_gpu, keep_layers=True)
            y_cpu, layers_cpu = omodel.gas_batch_forward(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb,
                                                         to_np(g.deg), to_np(wl.x), hs_cpu, return_layers=True)
            torch.cuda.synchronize()
            if check_layers:
                for l, (a, c) in enumerate(zip(layers_gpu, layers_cpu[:-1])):
                    e = node_rel_err(to_np(a), c)
                    assert e <= TOL[cfg.dtype], (cfg.name, sweep, b, "layer", l + 1, e)
            e = node_rel_err(to_np(y_gpu), y_cpu)
            worst = max(worst, e)
            assert e <= TOL[cfg.dtype], (cfg.name, sweep, b, "output", e)
    for l, (a, c) in enumerate(zip(hs_gpu, hs_cpu)):
        e = node_rel_err(to_np(a), c)
        assert e <= TOL[cfg.dtype], (cfg.name, "history", l, e)
    return worst, hs_gpu, y_gpu


def test_config0_tiny_gcn_two_sweeps_from_zero_history():
    wl = configs.build_workload(configs.config(0))
    _, hs_gpu, _ = _run_both(wl, range(4), "zeros", sweeps=2)
    # after one sweep the single history is exact, so sweep 2 equals the full-batch model
    om = oracle_model(wl)
    exact = omodel.full_batch_forward(om, to_np(wl.graph.rowptr), to_np(wl.graph.col), to_np(wl.x))
    assert node_rel_err(to_np(hs_gpu[0]), exact[0]) <= 1e-5


def test_config1_mid_gcn_full_size_first_batch():
    wl = configs.build_workload(configs.config(1))
    sg = batches.batch_subgraph(wl.graph, wl.batches[0], True)
    assert sg.nb == 50_000 and sg.nnz > 500_000
    _run_both(wl, [0], "normal")


def test_config2_large_gcn_scaled():
    wl = configs.build_workload(configs.config(2, 0.02))
    _run_both(wl, [0, 1], "normal")


def test_config3_deep_gcnii_scaled_and_full():
    wl = configs.build_workload(configs.config(3, 0.1))
    _run_both(wl, [0, 3], "normal")
    wl = configs.build_workload(configs.config(3))
    _run_both(wl, [0], "normal", check_layers=False)


def test_config4_huge_gin_bf16_scaled():
    wl = configs.build_workload(configs.config(4, 0.001))
    assert wl.cfg.dtype == torch.bfloat16 and wl.cfg.op == "gin"
    _run_both(wl, [0, 5], "normal")


def test_gin_fp32_small():
    cfg = configs.config(4, 0.0004)
    cfg.dtype = torch.float32
    wl = configs.build_workload(cfg)
    _run_both(wl, [1], "normal")


@pytest.mark.parametrize("cfg_id,scale", [(1, 0.1), (2, 0.02), (4, 0.001), (3, 0.1), (3, 1.0), (0, 1.0)])
def test_fused_execution_matches_oracle(cfg_id, scale):
    """Algorithm 1 with the halo rows read in place by the aggregation: same outputs and histories.  The narrow
    fp32 configurations (0 and 3) take the one-launch layer (gas_spmm_linear), the wide ones the two-kernel form."""
    from paper_2106_05609_amd import executor
    cfg0 = configs.config(cfg_id, scale)
    if cfg0.op == "gcnii":
        cfg0.widths = cfg0.widths[:8]        # 6 propagation layers
    wl = configs.build_workload(cfg0)
    cfg, g = wl.cfg, wl.graph
    hs_cpu = [to_np(h).copy() for h in configs.make_histories(cfg, init="normal")]
    hs_gpu = [h.to("cuda") for h in configs.make_histories(cfg, init="normal")]
    om, gm = oracle_model(wl), _gpu_model(wl)
    x_dev, deg_dev = wl.x.to("cuda"), g.deg.to("cuda")
    for b in (0, 1):
        sg = batches.batch_subgraph(g, wl.batches[b], cfg.self_loops)
        bg = _gpu_batch(wl, sg, deg_dev)
        y_gpu = executor.forward_batch_fused(gm, bg, x_dev, hs_gpu)
        y_cpu = omodel.gas_batch_forward(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(g.deg),
                                         to_np(wl.x), hs_cpu)
        assert node_rel_err(to_np(y_gpu), y_cpu) <= TOL[cfg.dtype]
    for a, c in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), c) <= TOL[cfg.dtype]


def test_paper_overhead_workload_matches_oracle():
    """The paper's synthetic runtime workload (Section 6 "Experiments", fast mini-batch execution): 4-layer GIN, batch of 4,000 nodes x 60 links,
    out-of-batch nodes x 60 links, at ratio 1; both history-access variants against the oracle."""
    from gas_inputs import graphs, rng
    from paper_2106_05609_amd import executor
    nb, F, L = 4000, 64, 4
    g = graphs.batch_with_outside_links(nb, 4000, 60, seed=0)
    sg = batches.batch_subgraph(g, torch.arange(nb), False)
    assert sg.nb == nb and sg.nh == 4000 and abs((sg.col >= nb).sum().item() / (sg.col < nb).sum().item() - 1.0) < 0.02
    ws = [(rng.glorot_uniform(0, 400 + 2 * l, F, F), rng.glorot_uniform(0, 401 + 2 * l, F, F)) for l in range(L)]
    x = rng.normal_matrix(0, 410, g.n, F)
    hist = [rng.normal_matrix(0, 411 + l, g.n, F) for l in range(L - 1)]
    om = omodel.Model("gin", [(to_np(a), to_np(b)) for a, b in ws])
    want = omodel.gas_batch_forward(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), nb, to_np(g.deg), to_np(x),
                                    [to_np(h).copy() for h in hist])
    d = lambda t: t.to("cuda")
    gm = executor.Model("gin", [(d(a), d(b)) for a, b in ws])
    bg = executor.BatchGraph(nb, d(sg.n_id), d(sg.rowptr), d(sg.col), None, None, None, max_F=F, normalise=False)
    for fn in (executor.forward_batch, executor.forward_batch_fused):
        y = fn(gm, bg, d(x), [d(h).clone() for h in hist])
        assert node_rel_err(to_np(y), want) <= 1e-5, fn.__name__


@pytest.mark.parametrize("cfg_id,scale,dtype", [(1, 0.1, torch.float32), (2, 0.02, torch.float32), (1, 0.1, torch.bfloat16)])
@pytest.mark.parametrize("fused", [False, True])
def test_appnp_matches_oracle(cfg_id, scale, dtype, fused):
    """APPNP (operator appendix): graph-agnostic prediction, then 5 weight-free propagation steps through the
    histories; outputs of two batches and the histories afterwards against the oracle."""
    from gas_inputs import rng
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    f_in, f_hid, f_out, K, alpha = 100, 256, 64, 5, 0.1
    x = rng.normal_matrix(cfg.seed, 830, g.n, f_in, dtype=dtype)
    w1 = rng.glorot_uniform(cfg.seed, 831, f_in if dtype == torch.float32 else 104, f_hid, dtype=dtype)
    if dtype == torch.bfloat16:
        x = rng.normal_matrix(cfg.seed, 830, g.n, 104, dtype=dtype)
    w2 = rng.glorot_uniform(cfg.seed, 832, f_hid, f_out, dtype=dtype)
    hist = [rng.normal_matrix(cfg.seed, 840 + l, g.n, f_out, dtype=dtype) for l in range(K - 1)]
    hs_cpu = [to_np(h).copy() for h in hist]
    hs_gpu = [h.to("cuda") for h in hist]
    d = lambda t: t.to("cuda")
    deg_dev = d(g.deg)
    for b in (0, 1):
        sg = batches.batch_subgraph(g, bl[b], True)
        bg = executor.BatchGraph(sg.nb, d(sg.n_id), d(sg.rowptr), d(sg.col), deg_dev, d(sg.colptr), d(sg.row),
                                 max_F=f_out, normalise=True)
        y = executor.appnp_forward_batch(d(w1), d(w2), alpha, K, bg, d(x), hs_gpu, fused=fused)
        want = omodel.appnp_batch_forward(to_np(w1), to_np(w2), alpha, K, to_np(sg.n_id), to_np(sg.rowptr),
                                          to_np(sg.col), sg.nb, to_np(g.deg), to_np(x), hs_cpu)
        assert node_rel_err(to_np(y), want) <= TOL[dtype], (b, node_rel_err(to_np(y), want))
    for a, c in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), c) <= TOL[dtype]


@pytest.mark.parametrize("cfg_id,scale,dtype,f,f1", [(1, 0.1, torch.float32, 64, 32), (2, 0.01, torch.float32, 100, 28),
                                                      (4, 0.0005, torch.bfloat16, 64, 64)])
def test_pna_model_matches_oracle(cfg_id, scale, dtype, f, f1):
    """Three PNA layers (operator appendix) through the histories, two batches, against the oracle."""
    from gas_inputs import rng
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    L = 3
    x = rng.normal_matrix(cfg.seed, 860, g.n, f, dtype=dtype)
    ws = [(rng.glorot_uniform(cfg.seed, 861 + 2 * l, 2 * f, f1, dtype=dtype),
           rng.glorot_uniform(cfg.seed, 862 + 2 * l, f + 9 * f1, f, dtype=dtype)) for l in range(L)]
    hist = [rng.normal_matrix(cfg.seed, 870 + l, g.n, f, dtype=dtype) for l in range(L - 1)]
    hs_cpu = [to_np(h).copy() for h in hist]
    hs_gpu = [h.to("cuda") for h in hist]
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    d = lambda t: t.to("cuda")
    ws_gpu = [(d(a), d(b)) for a, b in ws]
    ws_cpu = [(to_np(a), to_np(b)) for a, b in ws]
    tol = TOL[dtype] * (3 if dtype == torch.float32 else 1)      # three layers of three GEMMs each on top of the sums
    for b in (0, 1):
        sg = batches.batch_subgraph(g, bl[b], False)
        bg = executor.BatchGraph(sg.nb, d(sg.n_id), d(sg.rowptr), d(sg.col), None, None, None, max_F=f, normalise=False)
        y = executor.pna_forward_batch(ws_gpu, delta, bg, d(x), hs_gpu)
        want = omodel.pna_batch_forward(ws_cpu, delta, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(x),
                                        hs_cpu)
        assert node_rel_err(to_np(y), want) <= tol, (b, node_rel_err(to_np(y), want))
    for a, c in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), c) <= tol


@pytest.mark.parametrize("cfg_id,scale,dtype,f,heads", [(1, 0.1, torch.float32, 64, 1), (2, 0.01, torch.float32, 100, 1),
                                                         (4, 0.0005, torch.bfloat16, 128, 1), (1, 0.1, torch.float32, 64, 4),
                                                         (4, 0.0005, torch.bfloat16, 128, 8), (2, 0.01, torch.float32, 100, 5)])
def test_gat_model_matches_oracle(cfg_id, scale, dtype, f, heads):
    """Three GAT layers (operator appendix; one head, or several heads on blocks of columns) through the histories,
    two batches, against the oracle."""
    from gas_inputs import rng
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    L = 3
    x = rng.normal_matrix(cfg.seed, 880, g.n, f, dtype=dtype)
    ws = [(rng.glorot_uniform(cfg.seed, 881 + 3 * l, f, f, dtype=dtype), rng.normal(cfg.seed, 882 + 3 * l, 0, f, dtype=dtype) * 0.3,
           rng.normal(cfg.seed, 883 + 3 * l, 0, f, dtype=dtype) * 0.3) for l in range(L)]
    hist = [rng.normal_matrix(cfg.seed, 890 + l, g.n, f, dtype=dtype) for l in range(L - 1)]
    hs_cpu = [to_np(h).copy() for h in hist]
    hs_gpu = [h.to("cuda") for h in hist]
    d = lambda t: t.to("cuda")
    ws_gpu = [tuple(d(t) for t in w) for w in ws]
    ws_cpu = [tuple(to_np(t) for t in w) for w in ws]
    tol = TOL[dtype] * (2 if dtype == torch.float32 else 1)
    for b in (0, 1):
        sg = batches.batch_subgraph(g, bl[b], True)
        bg = executor.BatchGraph(sg.nb, d(sg.n_id), d(sg.rowptr), d(sg.col), None, None, None, max_F=f, normalise=False)
        y = executor.gat_forward_batch(ws_gpu, bg, d(x), hs_gpu, heads=heads)
        want = omodel.gat_batch_forward(ws_cpu, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(x), hs_cpu,
                                        heads=heads)
        assert node_rel_err(to_np(y), want) <= tol, (b, node_rel_err(to_np(y), want))
    for a, c in zip(hs_gpu, hs_cpu):
        assert node_rel_err(to_np(a), c) <= tol


@pytest.mark.parametrize("cfg_id,scale", [(1, 0.1), (4, 0.001), (3, 0.1)])
def test_host_histories_with_concurrent_transfers(cfg_id, scale):
    """Histories in pinned host memory, pulled ahead and pushed behind the computation on their own streams
    (Section 5 "PyGAS"): two sweeps over all batches give, bit for bit, the outputs and tables of the run with the
    tables in device memory, and the oracle's within tolerance."""
    from paper_2106_05609_amd import executor
    import paper_2106_05609_amd as gas
    cfg0 = configs.config(cfg_id, scale)
    if cfg0.op == "gcnii":
        cfg0.widths = cfg0.widths[:6]
    wl = configs.build_workload(cfg0)
    cfg, g = wl.cfg, wl.graph
    init = [h for h in configs.make_histories(cfg, init="normal")]
    hs_cpu = [to_np(h).copy() for h in init]
    hs_dev = [h.to("cuda") for h in init]
    pinned = [h.clone().pin_memory() for h in init]
    hs_host = [gas.HostTable(t) for t in pinned]
    om, gm = oracle_model(wl), _gpu_model(wl)
    x_dev, deg_dev = wl.x.to("cuda"), g.deg.to("cuda")
    pipe = executor.HostPipeline(torch.device("cuda"))
    order = list(range(min(4, len(wl.batches)))) * 2
    bgs = {}
    for k, b in enumerate(order):
        if b not in bgs:
            sg = batches.batch_subgraph(g, wl.batches[b], cfg.self_loops)
            bgs[b] = (sg, _gpu_batch(wl, sg, deg_dev))
        sg, bg = bgs[b]
        y_dev = executor.forward_batch(gm, bg, x_dev, hs_dev)
        y_host = executor.forward_batch_host(gm, bg, x_dev, hs_host, pipe)
        assert torch.equal(y_dev, y_host), (k, b)
        if k < 2:
            y_cpu = omodel.gas_batch_forward(om, to_np(sg.n_id), to_np(sg.rowptr), to_np(sg.col), sg.nb, to_np(g.deg),
                                             to_np(wl.x), hs_cpu)
            assert node_rel_err(to_np(y_host), y_cpu) <= TOL[cfg.dtype]
    pipe.join()
    torch.cuda.synchronize()
    for a, t in zip(hs_dev, pinned):
        assert torch.equal(a.cpu(), t)
