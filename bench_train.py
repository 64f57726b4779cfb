#!/usr/bin/env python3
"""One epoch of Algorithm 1 on a benchmark configuration: for every mini-batch, forward through all layers with
Push/Pull of the histories, softmax cross-entropy on the in-batch nodes, backward with the histories held constant,
gradient-descent update.  Every step is a C-ABI call (executor.train_step).  One JSON line on stdout."""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=2)
    p.add_argument("--scale", type=float, default=1.0)
    p.add_argument("--epochs", type=int, default=2, help="timed epochs after one warm-up epoch")
    p.add_argument("--separate", action="store_true", help="pull the halo rows instead of reading them in place")
    p.add_argument("--lr", type=float, default=0.0, help="step size (default: 0.01 for GCN; 1e-10 for GIN, whose unnormalised sums of N(0,1) features give logits of order 1e5)")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_train.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import configs, batches
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config, args.scale)
    lr = args.lr if args.lr > 0 else (1e-10 if cfg.op == "gin" else 0.01)
    if cfg.op == "gcnii":
        sys.exit("bench_train.py: use a GCN or GIN configuration (0, 1, 2, 4)")
    t0 = time.time()
    wl = configs.build_workload(cfg, device=dev)
    g = wl.graph
    n_classes = cfg.widths[-1]
    labels = configs.block_labels(g, min(n_classes, 16), cfg.seed, unlabelled=0.5).to(dev)
    ws = [(a.clone(), b.clone()) for a, b in wl.weights] if cfg.op == "gin" else [w.clone() for w in wl.weights]
    gm = executor.Model(cfg.op, ws, None, cfg.alpha, cfg.gin_eps)
    hist = configs.make_histories(cfg, device=dev, init="zeros")
    bgs = []
    for b in wl.batches:
        sg = batches.batch_subgraph(g, b, cfg.self_loops)
        bg = executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, sg.colptr, sg.row,
                                 max_F=max(cfg.widths + [cfg.gin_hidden]), normalise=cfg.op != "gin")
        lab_b = labels[sg.n_id[:sg.nb].long()].contiguous()
        bgs.append((bg, lab_b, int((lab_b >= 0).sum()), sg.nnz))
    torch.cuda.synchronize()
    print(f"[train] {cfg.name}: N={g.n} nnz={g.nnz}, {len(bgs)} batches, {len(ws)} layers, built in {time.time() - t0:.1f}s",
          file=sys.stderr, flush=True)

    def epoch():
        tot = torch.zeros(1, device=dev)
        n = 0
        for bg, lab_b, n_lab, _ in bgs:
            loss_sum, _, _, _ = executor.train_step(gm, bg, wl.x, hist, lab_b, lr, n_labelled=n_lab, fused=not args.separate)
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
    out = {"workload": f"configs[{args.config}] {cfg.name}: one training epoch over {len(bgs)} mini-batches, {len(ws)} layers",
           "epoch_s": round(sec, 4), "forward_edges_per_s": round(edges / sec, 1), "nodes_per_s": round(g.n / sec, 1),
           "mean_loss_per_epoch": [round(x, 5) for x in losses], "dtype": "f32" if cfg.dtype == torch.float32 else "bf16"}
    print(f"[train] epoch {sec * 1e3:.1f} ms, {edges / sec / 1e9:.2f} G forward edges/s, losses {out['mean_loss_per_epoch']}",
          file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
