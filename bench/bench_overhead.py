#!/usr/bin/env python3
"""The paper's synthetic runtime experiment (Section 6 "Experiments", "fast mini-batch
execution"; the figure on runtime overhead versus inter-/intra-connectivity):
a 4-layer GIN, a mini-batch of exactly 4,000 nodes each linked to 60 others
inside the batch, and a varying number of out-of-batch nodes each linked to 60
in-batch nodes.  For every ratio of inter- to intra-batch links it times one
forward pass of the batch through all layers (aggregation, MLP, push, and the
history access) and prints the overhead over the same batch without any
out-of-batch neighbours.

The paper compares a serial and a concurrent host-memory transfer scheme; here
the histories are in HBM, so the two variants are: halo rows pulled into the
mini-batch tensor by a separate launch ("separate"), and halo rows read in
place by the aggregation ("in-place").  The hidden width is not stated in the
paper: 256 is used.  With --host the history tables are in pinned host memory
instead, as in the paper, and the two variants are the paper's own: history
access in Algorithm 1's order on the compute stream ("host-serial"), and pulls
issued ahead / pushes behind the computation on their own streams
("host-concurrent", executor.forward_batch_host; the next pass's pulls still
wait for this pass's pushes, so results do not change).  One JSON line on
stdout, a table on stderr.
"""
import argparse
import json
import sys
import os

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--ratios", type=float, nargs="+", default=[0.0, 0.1, 0.25, 0.5, 1.0, 1.5, 2.0, 2.5, 3.0])
    p.add_argument("--width", type=int, default=256)
    p.add_argument("--layers", type=int, default=4)
    p.add_argument("--dtype", choices=["f32", "bf16"], default="f32")
    p.add_argument("--reps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--host", action="store_true", help="history tables in pinned host memory: serial against "
                                                        "concurrent transfers")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_overhead.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import graphs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    dt = torch.float32 if args.dtype == "f32" else torch.bfloat16
    nb, links, F, L = 4000, 60, args.width, args.layers
    ws = [(rng.glorot_uniform(0, 400 + 2 * l, F, F, dev, dt), rng.glorot_uniform(0, 401 + 2 * l, F, F, dev, dt))
          for l in range(L)]
    model = executor.Model("gin", ws)
    rows = []
    base = {}
    for ratio in args.ratios:
        n_out = int(round(ratio * nb))
        g = graphs.batch_with_outside_links(nb, n_out, links, seed=0, device=dev)
        sg = batches.batch_subgraph(g, torch.arange(nb), False)
        bg = executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, None, None, max_F=F, normalise=False)
        x = rng.normal_matrix(0, 410, g.n, F, dev, dt)
        hist = [rng.normal_matrix(0, 411 + l, g.n, F, dev, dt) for l in range(L - 1)]
        intra = int((sg.col < nb).sum())
        res = {"ratio_requested": ratio, "n_outside": n_out, "intra_entries": intra,
               "inter_entries": sg.nnz - intra, "ratio": round((sg.nnz - intra) / max(1, intra), 3)}
        if args.host:
            hist = [gas.HostTable(h.cpu().pin_memory()) for h in hist]
            pipe = executor.HostPipeline(dev)

            def concurrent(model, bg, x, hist):
                return executor.forward_batch_host(model, bg, x, hist, pipe)
            variants = (("host-serial", executor.forward_batch), ("host-concurrent", concurrent))
        else:
            variants = (("separate", executor.forward_batch), ("in-place", executor.forward_batch_fused))
        names = [v[0] for v in variants]
        for name, fn in variants:
            for _ in range(args.warmup):
                fn(model, bg, x, hist)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(args.reps):
                fn(model, bg, x, hist)
            if args.host:
                pipe.join()         # the timed region ends when the last push has landed
            b.record()
            torch.cuda.synchronize()
            res[name + "_ms"] = a.elapsed_time(b) / args.reps
        if not base:
            base = {k: v for k, v in res.items() if k.endswith("_ms")}
        for name in names:
            res[name + "_overhead_pct"] = round(100.0 * (res[name + "_ms"] / base[name + "_ms"] - 1.0), 1)
        rows.append(res)
        print(f"ratio {res['ratio']:5.2f}  outside {n_out:6d}  " + "  ".join(
            f"{name} {res[name + '_ms']:.4f} ms (+{res[name + '_overhead_pct']:5.1f} %)" for name in names),
            file=sys.stderr, flush=True)
    print(json.dumps({"histories": "pinned host memory" if args.host else "HBM",
                      "workload": f"{L}-layer GIN, width {F}, {args.dtype}, batch of {nb} nodes x {links} links, "
                                  "out-of-batch nodes x 60 links; forward pass of one batch",
                      "paper": "serial history access raises runtime by up to 350 %, concurrent access leaves only the "
                               "extra aggregation (up to about 25 % for ratios of real datasets, 0.1-2.5), on a GeForce "
                               "RTX 2080 Ti with histories in host memory",
                      "rows": rows}))


if __name__ == "__main__":
    main()
