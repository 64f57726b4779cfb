#!/usr/bin/env python3
"""One epoch of Algorithm 1 on a benchmark configuration: for every mini-batch, forward through all layers with
Push/Pull of the histories, softmax cross-entropy on the in-batch nodes, backward with the histories held constant,
gradient-descent update.  Every step is a C-ABI call (executor.train_step).  --op pna / --op gat train a PNA or GAT
model of the configuration's widths on its graph and batches instead (executor.pna_train_batch / gat_train_batch;
PNA with messages of a quarter of the layer width, GAT with four heads).  With --graph every mini-batch's whole
training step (it neither allocates behind the allocator's back nor waits) is also captured as a HIP graph; the
epochs are then timed both ways from the same state and the weights and histories afterwards must be the same bits.
One JSON line on stdout."""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=2)
    p.add_argument("--scale", type=float, default=1.0)
    p.add_argument("--epochs", type=int, default=2, help="timed epochs after one warm-up epoch")
    p.add_argument("--separate", action="store_true", help="pull the halo rows instead of reading them in place")
    p.add_argument("--graph", action="store_true", help="also replay every mini-batch's training step as a HIP graph")
    p.add_argument("--op", default=None, choices=["pna", "gat"], help="train this operator instead of the configuration's")
    p.add_argument("--heads", type=int, default=4, help="attention heads of --op gat")
    p.add_argument("--lr", type=float, default=0.0, help="step size (default: 0.01 for GCN; 1e-10 for GIN, whose unnormalised sums of N(0,1) features give logits of order 1e5)")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_train.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import configs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config, args.scale)
    lr = args.lr if args.lr > 0 else (1e-10 if cfg.op == "gin" else 0.01)
    fused = not args.separate
    t0 = time.time()
    wl = configs.build_workload(cfg, device=dev)
    g = wl.graph
    n_classes = cfg.widths[-1]
    labels = configs.block_labels(g, min(n_classes, 16), cfg.seed, unlabelled=0.5).to(dev)
    ws = [(a.clone(), b.clone()) for a, b in wl.weights] if cfg.op == "gin" else [w.clone() for w in wl.weights]
    gm = executor.Model(cfg.op, ws, wl.w_in.clone() if cfg.op == "gcnii" else None, cfg.alpha, cfg.gin_eps)
    hist = configs.make_histories(cfg, device=dev, init="zeros")
    if args.op:
        if args.graph:
            sys.exit("bench_train.py: --graph is for the configuration's own operator")
        wd, dt = cfg.widths, cfg.dtype
        L = len(wd) - 1
        hist = [torch.zeros((g.n, wd[l + 1]), dtype=dt, device=dev) for l in range(L - 1)]
        if args.op == "pna":
            ws = [(rng.glorot_uniform(cfg.seed, 1800 + 2 * l, 2 * wd[l], max(8, wd[l + 1] // 4), dev, dt),
                   rng.glorot_uniform(cfg.seed, 1801 + 2 * l, wd[l] + 9 * max(8, wd[l + 1] // 4), wd[l + 1], dev, dt))
                  for l in range(L)]
        else:
            ws = [(rng.glorot_uniform(cfg.seed, 1810 + 3 * l, wd[l], wd[l + 1], dev, dt),
                   rng.normal(cfg.seed, 1811 + 3 * l, 0, wd[l + 1], dev, dt) * 0.1,
                   rng.normal(cfg.seed, 1812 + 3 * l, 0, wd[l + 1], dev, dt) * 0.1) for l in range(L)]
        delta = float(torch.log(g.deg.double() + 1.0).mean())
        lr = args.lr if args.lr > 0 else 1e-6
    bgs = []
    for b in wl.batches:
        sg = batches.batch_subgraph(g, b, cfg.self_loops or args.op == "gat")
        bg = executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, sg.colptr, sg.row,
                                 max_F=max(cfg.widths + [cfg.gin_hidden]), normalise=cfg.op != "gin" and not args.op,
                                 csc_pos=sg.csc_perm.to(torch.int32))
        if args.op:
            bg.plan_t_all                                          # the backward aggregations' plan, built once
        lab_b = labels[sg.n_id[:sg.nb].long()].contiguous()
        bgs.append((bg, lab_b, int((lab_b >= 0).sum()), sg.nnz))
    torch.cuda.synchronize()
    print(f"[train] {cfg.name}: N={g.n} nnz={g.nnz}, {len(bgs)} batches, {len(ws)} layers, built in {time.time() - t0:.1f}s",
          file=sys.stderr, flush=True)

    def epoch():
        tot = torch.zeros(1, device=dev)
        n = 0
        for bg, lab_b, n_lab, _ in bgs:
            if args.op:
                loss_sum = torch.zeros(1, device=dev)

                def loss_grad(y):
                    gy = torch.empty_like(y)
                    gas.gas_softmax_xent(y, lab_b, gy, torch.empty(bg.nb, device=dev), loss_sum, scale=1.0 / max(1, n_lab))
                    return gy
                if args.op == "pna":
                    _, grads, _ = executor.pna_train_batch(ws, delta, bg, wl.x, hist, loss_grad)
                else:
                    _, grads, _ = executor.gat_train_batch(ws, bg, wl.x, hist, loss_grad, heads=args.heads)
                executor.sgd_update(ws, grads, lr)
            else:
                loss_sum, _, _, _ = executor.train_step(gm, bg, wl.x, hist, lab_b, lr, n_labelled=n_lab, fused=fused)
            tot += loss_sum
            n += n_lab
        return tot, n
    losses = []
    tot, n = epoch()                                              # warm-up (and the histories' first fill)
    losses.append(float(tot) / n)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.epochs):
        tot, n = epoch()
        losses.append(float(tot) / n)                             # one read-back per epoch
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.epochs
    edges = sum(nnz for *_, nnz in bgs) * len(ws)                 # entries aggregated per epoch, forward
    graph = None
    if args.graph:
        state = [w for pair in ws for w in (pair if isinstance(pair, tuple) else (pair,))] + list(hist)
        if gm.w_in is not None:
            state.append(gm.w_in)
        for bg, *_ in bgs:
            if fused:
                bg.src                                            # built before any capture (it allocates)
            if cfg.op == "gcnii":
                bg.plan_t_all

        def run_epochs(step_fns):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.epochs):
                for f in step_fns:
                    f()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / args.epochs
        start = [t.clone() for t in state]
        eager_fns = [(lambda bg=bg, lab_b=lab_b, n_lab=n_lab: executor.train_step(gm, bg, wl.x, hist, lab_b, lr, n_labelled=n_lab,
                                                                                  fused=fused))
                     for bg, lab_b, n_lab, _ in bgs]
        sec_eager = run_epochs(eager_fns)
        after_eager = [t.clone() for t in state]
        for t, t0_ in zip(state, start):
            t.copy_(t0_)
        graphs, pool = [], None
        for f in eager_fns:                                       # capture only: nothing runs, the state stays put
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, pool=pool):
                f()
            pool = pool or gr.pool()
            graphs.append(gr)
        sec_graph = run_epochs([gr.replay for gr in graphs])
        same = all(torch.equal(a, b) for a, b in zip(state, after_eager))
        graph = {"epoch_s_eager": round(sec_eager, 5), "epoch_s_graph": round(sec_graph, 5),
                 "speedup": round(sec_eager / sec_graph, 2), "state_bit_identical": same}
        print(f"[train] from one state: eager epoch {sec_eager * 1e3:.2f} ms, graph replay {sec_graph * 1e3:.2f} ms "
              f"(x{sec_eager / sec_graph:.2f}), weights and histories identical: {same}", file=sys.stderr, flush=True)
        if not same:
            sys.exit("bench_train.py: the replayed epochs left different weights or histories")
    out = {"workload": f"configs[{args.config}] {cfg.name}{' as a ' + args.op.upper() + ' model' if args.op else ''}: one training epoch "
                       f"over {len(bgs)} mini-batches, {len(ws)} layers",
           "epoch_s": round(sec, 4), "batches": len(bgs), "ms_per_training_step": round(sec / len(bgs) * 1e3, 4),
           "forward_edges_per_s": round(edges / sec, 1), "nodes_per_s": round(g.n / sec, 1),
           "mean_loss_per_epoch": [round(x, 5) for x in losses], "dtype": "f32" if cfg.dtype == torch.float32 else "bf16"}
    if graph:
        out["graph_replay"] = graph
    print(f"[train] epoch {sec * 1e3:.2f} ms = {len(bgs)} steps of {sec / len(bgs) * 1e3:.3f} ms, {edges / sec / 1e9:.2f} G forward edges/s, losses {out['mean_loss_per_epoch']}",
          file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
