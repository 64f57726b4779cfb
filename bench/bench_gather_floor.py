#!/usr/bin/env python3
"""What bounds the in-place aggregation: the same gas_spmm_hist call on a benchmark configuration's first batch
(same pattern, same plan, same output), with every gathered index replaced by one inside a table of R rows.  Small R:
every gather is an L2 hit, and what remains is the kernel's own floor; R of the size of the Infinity Cache: every L2
miss is answered by that cache; large R at random: the rate at which this machine delivers rows it has to fetch from
HBM.  The real sources are timed first.  One JSON line on stdout, a table on stderr."""
import argparse
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=4)
    p.add_argument("--reps", type=int, default=10)
    p.add_argument("--rows", type=int, nargs="*", default=[1 << 12, 1 << 16, 1 << 19, 1 << 21])
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_gather_floor.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd.layer_step import LayerStep
    from gas_inputs import configs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config)
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], cfg.self_loops)
    ls = LayerStep(cfg, g, sg, rng, dev)
    bg = ls.bg
    row_bytes = ls.x.shape[1] * ls.x.element_size()

    def timed(src):
        def run():
            if ls.gin:
                gas.gas_spmm_hist(bg.plan, bg.rowptr, src, None, ls.x[:ls.nb], ls.hist_in, ls.z, diag=ls.diag)
            else:
                gas.gas_spmm_hist(bg.plan, bg.rowptr, src, bg.val, ls.x[:ls.nb], ls.hist_in, ls.z)
        for _ in range(3):
            run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.reps):
            run()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.reps
    nnz = bg.src.numel()
    out = {"workload": f"configs[{args.config}] {cfg.name}: gas_spmm_hist, middle layer, first batch", "nnz_b": nnz,
           "row_bytes": row_bytes, "ms": {}}
    t = timed(bg.src)
    out["ms"]["real sources"] = round(t, 3)
    print(f"{'real sources':44s} {t:8.3f} ms  {nnz * row_bytes / t / 1e6:8.0f} GB/s at the lanes", file=sys.stderr, flush=True)
    k = torch.arange(nnz, device=dev, dtype=torch.int64)
    for rows in args.rows:
        rows = min(rows, ls.nb)
        # rows 0 .. R-1 of the mini-batch tensor, scattered by a multiplicative hash of the entry's position
        folded = ((k * 2654435761) % rows).to(torch.int32)
        t = timed(folded)
        label = f"all gathers within {rows} rows ({rows * row_bytes / 2**20:.0f} MiB)"
        out["ms"][label] = round(t, 3)
        print(f"{label:44s} {t:8.3f} ms  {nnz * row_bytes / t / 1e6:8.0f} GB/s at the lanes", file=sys.stderr, flush=True)
        del folded
    print(json.dumps(out))


if __name__ == "__main__":
    main()
