#!/usr/bin/env python3
"""Whole-model forward of one mini-batch, eager against a captured HIP graph, on the launch-bound configurations.

Config 3 (64-layer GCNII, 21 k-node batches) and config 0 (2-layer GCN, 512-node batches) spend their time in launch
overhead, not in the kernels: every layer is four small launches.  None of the forward calls allocates or waits, so a
whole forward pass is captured once (torch.cuda.graph on the stream the calls are given) and replayed.  Every replay
is compared bit for bit with the eager result.  One JSON line on stdout, a table on stderr."""
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
    p.add_argument("--configs", type=int, nargs="+", default=[3, 0, 1])
    p.add_argument("--reps", type=int, default=20)
    p.add_argument("--in-place", action="store_true",
                   help="the in-place forward: halo rows read by the aggregation, push in the transform's epilogue")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_graph.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import configs, batches
    gas.lib()
    dev = torch.device("cuda:0")
    out = {"runs": []}
    for c in args.configs:
        cfg = configs.config(c)
        wl = configs.build_workload(cfg, device=dev)
        g = wl.graph
        sg = batches.batch_subgraph(g, wl.batches[0], cfg.self_loops)
        ws = [(a, b) for a, b in wl.weights] if cfg.op == "gin" else list(wl.weights)
        gm = executor.Model(cfg.op, ws, wl.w_in, cfg.alpha, cfg.gin_eps)
        bg = executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, sg.colptr, sg.row,
                                 max_F=max(cfg.widths + [cfg.gin_hidden]), normalise=cfg.op != "gin")
        hist = configs.make_histories(cfg, device=dev, init="normal")
        run = executor.forward_batch_fused if args.in_place else executor.forward_batch
        bg.src                                           # built once, before any capture (it allocates)
        fwd = lambda: run(gm, bg, wl.x, hist)
        y_eager = fwd().clone()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.reps):
            fwd()
        torch.cuda.synchronize()
        ms_eager = (time.perf_counter() - t0) / args.reps * 1e3
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(2):
                fwd()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            y_graph = fwd()
        ok = True
        for _ in range(3):                               # replays with eager work and synchronisation between them
            graph.replay()
            torch.cuda.synchronize()
            ok = ok and torch.equal(y_graph, y_eager)
            ok = ok and torch.equal(fwd(), y_eager)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.reps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) / args.reps * 1e3
        n_layers = gm.n_layers
        rec = {"config": c, "name": cfg.name, "in_place": args.in_place, "layers": n_layers, "nb": sg.nb, "eager_ms": round(ms_eager, 4),
               "graph_ms": round(ms_graph, 4), "speedup": round(ms_eager / ms_graph, 2), "replays_bit_identical": ok}
        out["runs"].append(rec)
        print(f"configs[{c}] {cfg.name:14s} {n_layers:3d} layers  eager {ms_eager:8.3f} ms  graph {ms_graph:8.3f} ms  "
              f"x{ms_eager / ms_graph:.2f}  replays identical: {ok}", file=sys.stderr, flush=True)
        if not ok:
            sys.exit("bench_graph.py: a replay differs from the eager result")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
