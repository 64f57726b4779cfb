#!/usr/bin/env python3
"""The in-place aggregation (gas_spmm_hist, middle layer) on EVERY mini-batch of a benchmark configuration, not only
the first one that bench.py times: batch sizes, heavy rows and chunks of each plan, time and entries per second.
The batches of the power-law configurations differ a lot (the one that holds the hubs has several times the
entries of the others); the rate should not.  A table on stdout."""
import argparse
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=4)
    p.add_argument("--reps", type=int, default=10)
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_all_batches.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd.layer_step import LayerStep
    from gas_inputs import configs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config)
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    tables = None
    for b in range(len(bl)):
        sg = batches.batch_subgraph(g, bl[b], cfg.self_loops)
        kw = {} if tables is None else dict(tables_in=[tables[0]], table_out=tables[1])
        ls = LayerStep(cfg, g, sg, rng, dev, **kw)
        if tables is None:
            tables = (ls.hist_in, ls.hist_out)              # every batch gathers from the same table
        bg = ls.bg

        def run():
            if ls.gin:
                gas.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, None, ls.x[:ls.nb], ls.hist_in, ls.z, diag=ls.diag)
            else:
                gas.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, ls.x[:ls.nb], ls.hist_in, ls.z)
        for _ in range(3):
            run()
        torch.cuda.synchronize()
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.reps):
            run()
        e.record()
        torch.cuda.synchronize()
        t = a.elapsed_time(e) / args.reps
        d = bg.plan.describe()
        longest = int((sg.rowptr[1:] - sg.rowptr[:-1]).max())
        print(f"batch {b:2d}: nb {sg.nb:,} nh {sg.nh:,} entries {sg.nnz:,} longest row {longest:,} heavy rows {d['n_heavy']:,} "
              f"chunks {d['n_chunks']:,}: gas_spmm_hist {t:.3f} ms, {sg.nnz / t / 1e6:.2f} G entries/s", flush=True)
        del ls, bg, sg


if __name__ == "__main__":
    main()
