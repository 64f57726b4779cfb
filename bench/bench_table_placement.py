#!/usr/bin/env python3
"""Where a history table lies decides how fast its rows are gathered: the same in-place aggregation (config 4, first
batch, same data) and the same pull of the halo rows, timed against copies of the 25.6 GB table that were allocated
at different moments of ONE process: first thing, out of the framework's cache after the graph was generated and
freed, freshly after that cache was emptied, and last (by the generator of the table's contents).  Prints the
memory and compute partition modes the box reports, then one line per table."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    if not torch.cuda.is_available():
        sys.exit("bench_table_placement.py: no GPU visible")
    try:
        print(subprocess.run(["rocm-smi", "--showmemorypartition", "--showcomputepartition"], capture_output=True, text=True,
                             timeout=30).stdout[-600:], flush=True)
    except Exception as e:                                        # the tool is optional: the timings do not need it
        print("rocm-smi not available:", e, flush=True)
    import paper_2106_05609_amd as gas
    from gas_inputs import configs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(4)
    F, dt = 256, torch.bfloat16

    def timed(fn, n=6):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    tables = [("allocated first", torch.empty((cfg.n, F), dtype=dt, device=dev))]
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], cfg.self_loops)
    nb = sg.nb
    del g
    tables.append(("from the framework's cache, after the graph", torch.empty((cfg.n, F), dtype=dt, device=dev)))
    torch.cuda.empty_cache()
    tables.append(("fresh, after the cache was emptied", torch.empty((cfg.n, F), dtype=dt, device=dev)))
    tables.append(("fresh, the next one", torch.empty((cfg.n, F), dtype=dt, device=dev)))
    ref = rng.normal_matrix(cfg.seed, 200, cfg.n, F, dev, dt)
    tables.append(("allocated last, by the generator", ref))
    x = rng.normal_matrix(cfg.seed, 210, sg.nv, F, dev, dt)
    z = torch.empty((nb, F), dtype=dt, device=dev)
    src = torch.empty_like(sg.col)
    gas.gas_fuse_sources(sg.col, nb, sg.n_id, src)
    plan = gas.gas_plan_create(sg.rowptr, sg.nnz, F, ind=src)
    idx = sg.n_id[nb:]
    dst = torch.empty((idx.numel(), F), dtype=dt, device=dev)
    for rep in range(2):                                          # twice, the second time in reverse order
        for name, t in (tables if rep == 0 else tables[::-1]):
            if t is not ref:
                t.copy_(ref)
            ms = timed(lambda: gas.gas_spmm_hist(plan, sg.rowptr, src, None, x[:nb], t, z, diag=1.0))
            mp = timed(lambda: gas.gas_pull(t, idx, dst))
            print(f"{name:46s} at 0x{t.data_ptr():x}: gas_spmm_hist {ms:.3f} ms, gas_pull of the halo rows {mp:.3f} ms",
                  flush=True)


if __name__ == "__main__":
    main()
