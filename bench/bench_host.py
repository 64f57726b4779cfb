#!/usr/bin/env python3
"""History tables in host memory (the paper's arrangement, Section 5 "PyGAS"): forward passes over consecutive
mini-batches of a benchmark configuration with

  hbm              the tables in device memory (executor.forward_batch), for reference;
  host-serial      the tables in pinned host memory, pulls and pushes in Algorithm 1's order on the compute stream;
  host-concurrent  the same tables, every layer's halo rows pulled ahead on one stream and every layer's output
                   pushed behind the computation on another (executor.forward_batch_host).

With --disk DIR a fourth variant keeps the tables in files under DIR (executor.forward_batch_disk: host threads
gather the rows into pinned buffers, copies run beside the computation), and the file path itself is measured with
the same 100,000 rows.

All give the same bits (tests/test_gpu_gas.py, tests/test_gpu_disk.py).  Before the sweeps the host link itself is measured with
100,000 rows of 1 KiB each way: a pull alone, a push alone, and both at once on two streams (and, for comparison,
the copy engines moving the same contiguous bytes both ways at once).  One JSON line on stdout, a table on stderr.
"""
import argparse
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=1)
    p.add_argument("--scale", type=float, default=1.0)
    p.add_argument("--batches", type=int, default=4, help="consecutive mini-batches per sweep")
    p.add_argument("--reps", type=int, default=5, help="timed sweeps")
    p.add_argument("--disk", default=None, help="directory for history tables kept in files (adds the disk variant)")
    p.add_argument("--io-threads", type=int, default=8)
    p.add_argument("--disk-calls", action="store_true", help="pread / pwrite instead of the mapped file")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_host.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import configs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config, args.scale)
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)[: args.batches]
    dt, widths, gin = cfg.dtype, cfg.widths, cfg.op == "gin"
    L = len(widths) - 1 if cfg.op != "gcnii" else len(widths) - 2
    if gin:
        ws = [(rng.glorot_uniform(cfg.seed, 100 + 2 * l, widths[l], cfg.gin_hidden, dev, dt),
               rng.glorot_uniform(cfg.seed, 101 + 2 * l, cfg.gin_hidden, widths[l + 1], dev, dt)) for l in range(L)]
        model = executor.Model("gin", ws, gin_eps=cfg.gin_eps)
    elif cfg.op == "gcnii":
        w_in = rng.glorot_uniform(cfg.seed, 99, widths[0], widths[1], dev, dt)
        ws = [rng.glorot_uniform(cfg.seed, 100 + l, widths[l + 1], widths[l + 2], dev, dt) for l in range(L)]
        model = executor.Model("gcnii", ws, w_in=w_in, alpha=cfg.alpha)
    else:
        ws = [rng.glorot_uniform(cfg.seed, 100 + l, widths[l], widths[l + 1], dev, dt) for l in range(L)]
        model = executor.Model("gcn", ws)
    x = rng.normal_matrix(cfg.seed, 110, g.n, widths[0], dev, dt)
    bgs, halo, inb = [], 0, 0
    for b in bl:
        sg = batches.batch_subgraph(g, b, cfg.self_loops)
        bgs.append(executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, None, None, max_F=max(widths),
                                       normalise=not gin))
        halo, inb = halo + sg.nh, inb + sg.nb
    hw = [model.out_width(l) for l in range(L - 1)]
    s = 4 if dt == torch.float32 else 2
    moved = sum((halo + inb) * w * s for w in hw)               # bytes over the host link per sweep
    hbm = [torch.zeros((g.n, w), dtype=dt, device=dev) for w in hw]
    host = [gas.HostTable(torch.zeros((g.n, w), dtype=dt).pin_memory()) for w in hw]
    pipe = executor.HostPipeline(dev)

    def timed(fn, reps=10):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        pipe.join()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    n_link = min(100000, g.n)
    t_in, t_out = (gas.HostTable(torch.zeros((n_link, 256)).pin_memory()) for _ in range(2))
    d_in, d_out = torch.empty((n_link, 256), device=dev), torch.ones((n_link, 256), device=dev)
    rows = rng.permutation(cfg.seed, 120, n_link).to(torch.int32).to(dev)

    def both(pull, push):
        cur = torch.cuda.current_stream()
        pipe.pull.wait_stream(cur)
        pipe.push.wait_stream(cur)
        with torch.cuda.stream(pipe.pull):
            pull()
        with torch.cuda.stream(pipe.push):
            push()
    k_pull, k_push = (lambda: gas.gas_pull(t_in, rows, d_in)), (lambda: gas.gas_push(d_out, rows, t_out))
    e_pull = lambda: d_in.copy_(t_in.tensor, non_blocking=True)
    e_push = lambda: t_out.tensor.copy_(d_out, non_blocking=True)
    gb = n_link * 1024 / 1e9
    link = {"GB_each_way": round(gb, 4), "pull_ms": timed(k_pull), "push_ms": timed(k_push),
            "pull_and_push_ms": timed(lambda: both(k_pull, k_push)),
            "copy_engines_both_ways_ms": timed(lambda: both(e_pull, e_push))}
    link = {k: round(v, 3) for k, v in link.items()}
    print(f"host link, {gb:.3f} GB each way: pull {link['pull_ms']} ms, push {link['push_ms']} ms, both at once "
          f"{link['pull_and_push_ms']} ms ({2 * gb / link['pull_and_push_ms'] * 1e3:.1f} GB/s); copy engines both ways "
          f"{link['copy_engines_both_ways_ms']} ms", file=sys.stderr, flush=True)
    disk, dpipe = None, None
    if args.disk:
        import time
        os.makedirs(args.disk, exist_ok=True)
        probe = gas.DiskTable(os.path.join(args.disk, "probe.bin"), n_link, 256, torch.float32, create=True,
                              io_threads=args.io_threads, calls=args.disk_calls)
        rows_host = rows.cpu()

        def wall(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            return (time.perf_counter() - t0) / reps * 1e3
        link["disk_push_ms"] = round(wall(lambda: probe.wait(probe.push(d_out, rows_host))), 3)
        link["disk_pull_ms"] = round(wall(lambda: probe.wait(probe.pull(rows_host, d_in))), 3)
        link["disk_push_range_ms"] = round(wall(lambda: probe.wait(probe.push(d_out, None, base=0))), 3)
        link["disk_pull_range_ms"] = round(wall(lambda: probe.wait(probe.pull(None, d_in, base=0))), 3)
        print(f"file path, {gb:.3f} GB: scattered rows pull {link['disk_pull_ms']} ms, push {link['disk_push_ms']} ms; "
              f"one range pull {link['disk_pull_range_ms']} ms, push {link['disk_push_range_ms']} ms "
              f"({args.io_threads} I/O threads)", file=sys.stderr, flush=True)
        probe.close()
        os.remove(os.path.join(args.disk, "probe.bin"))
        disk = [gas.DiskTable(os.path.join(args.disk, f"hist{l}.bin"), g.n, w, dt, create=True,
                              io_threads=args.io_threads, calls=args.disk_calls) for l, w in enumerate(hw)]
        dpipe = executor.DiskPipeline()
    del t_in, t_out, d_in, d_out

    def sweep(kind):
        for bg in bgs:
            if kind == "hbm":
                executor.forward_batch(model, bg, x, hbm)
            elif kind == "host-serial":
                executor.forward_batch(model, bg, x, host)
            elif kind == "disk":
                executor.forward_batch_disk(model, bg, x, disk, dpipe)
            else:
                executor.forward_batch_host(model, bg, x, host, pipe)
        if kind == "host-concurrent":
            pipe.join()
        if kind == "disk":
            dpipe.join()

    out = {"config": cfg.name, "host_link": link, "batches": len(bgs), "layers": L, "history_tables": len(hw),
           "rows_pulled_per_sweep": halo, "rows_pushed_per_sweep": inb, "host_link_GB_per_sweep": round(moved / 1e9, 3),
           "ms_per_batch": {}}
    for kind in ("hbm", "host-serial", "host-concurrent") + (("disk",) if disk else ()):
        import time
        for _ in range(2):
            sweep(kind)
        torch.cuda.synchronize()
        t0 = time.perf_counter()                    # the disk variant waits on the host, so wall time for all
        for _ in range(args.reps):
            sweep(kind)
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) * 1e3 / args.reps / len(bgs)
        out["ms_per_batch"][kind] = round(t, 4)
        print(f"{kind:16s} {t:9.3f} ms per batch", file=sys.stderr, flush=True)
    same = all(torch.equal(a.cpu(), h.tensor) for a, h in zip(hbm, host))
    if disk:
        for a, t in zip(hbm, disk):
            back = torch.empty(a.shape, dtype=a.dtype)
            t.read_rows(back)
            same = same and torch.equal(a.cpu(), back)
            t.close()
            os.remove(t.path)
    out["tables_identical"] = same
    rate = 2 * gb / link["pull_and_push_ms"] * 1e3          # GB/s with both directions busy
    out["link_bound_ms_per_batch"] = round(moved / len(bgs) / 1e6 / rate, 3)
    print(f"tables identical: {same}; {moved / 1e9:.3f} GB per sweep over the host link", file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
