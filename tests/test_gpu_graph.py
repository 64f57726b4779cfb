"""A whole-model forward pass captured as a HIP graph: no forward call allocates or waits, so the capture is legal,
and every replay (with eager work and synchronisation between replays) gives the bits of the eager pass."""
import pytest
import torch

from gas_inputs import configs, batches
from tests.test_gpu_gas import _gpu_model, _gpu_batch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg_id,scale,fused", [(0, 1.0, False), (0, 1.0, True), (3, 0.05, False), (3, 0.05, True), (4, 0.0005, True)])
def test_forward_replays_bit_identical(cfg_id, scale, fused):
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    if cfg.op == "gcnii":
        cfg.widths = cfg.widths[:10]
    wl = configs.build_workload(cfg)
    g = wl.graph
    gm = _gpu_model(wl)
    sg = batches.batch_subgraph(g, wl.batches[0], cfg.self_loops)
    bg = _gpu_batch(wl, sg, g.deg.to("cuda"))
    if fused:
        bg.src                                           # built once, outside the capture (it allocates)
    hist = [h.to("cuda") for h in configs.make_histories(cfg, init="normal")]
    x = wl.x.to("cuda")
    run = executor.forward_batch_fused if fused else executor.forward_batch
    fwd = lambda: run(gm, bg, x, hist)
    y_eager = fwd().clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fwd()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        y_graph = fwd()
    for _ in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager)
        assert torch.equal(fwd(), y_eager)               # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("cfg_id,scale,fused", [(0, 1.0, True), (3, 0.05, True), (1, 0.1, False)])
def test_training_step_replays_bit_identical(cfg_id, scale, fused):
    """A whole training step (forward, loss, backward, update) captured as a HIP graph: three replays leave the
    weights and histories that three eager steps from the same state leave."""
    from paper_2106_05609_amd import executor
    cfg = configs.config(cfg_id, scale)
    if cfg.op == "gcnii":
        cfg.widths = cfg.widths[:10]
    wl = configs.build_workload(cfg)
    g = wl.graph
    gm = _gpu_model(wl)
    sg = batches.batch_subgraph(g, wl.batches[0], cfg.self_loops)
    bg = _gpu_batch(wl, sg, g.deg.to("cuda"))
    if fused:
        bg.src
    if cfg.op == "gcnii":
        bg.plan_t_all                                    # plans are built outside the capture
    hist = [h.to("cuda") for h in configs.make_histories(cfg, init="normal")]
    x = wl.x.to("cuda")
    labels = configs.block_labels(g, min(cfg.widths[-1], 16), cfg.seed, unlabelled=0.5).to("cuda")
    lab_b = labels[bg.n_id[:sg.nb].long()].contiguous()
    n_lab = int((lab_b >= 0).sum())
    state = [w for pair in gm.weights for w in (pair if isinstance(pair, tuple) else (pair,))] + hist
    if gm.w_in is not None:
        state.append(gm.w_in)
    step = lambda: executor.train_step(gm, bg, x, hist, lab_b, 0.05, n_labelled=n_lab, fused=fused)
    start = [t.clone() for t in state]
    for _ in range(3):
        step()
    want = [t.clone() for t in state]
    assert not all(torch.equal(a, b) for a, b in zip(want, start))       # the steps did change the weights
    for t, t0 in zip(state, start):
        t.copy_(t0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        graph.replay()
        torch.cuda.synchronize()
    for a, b in zip(state, want):
        assert torch.equal(a, b)
