#!/usr/bin/env python3
"""Benchmark of the GAS layer step on one MI355X.

A step is one pass of the whole hot path over one mini-batch of the synthetic
workload, for a middle layer (hidden width in and out):

    gas_pull    halo rows of the mini-batch tensor <- history table l
    gas_spmm    aggregation over the batch subgraph
    gas_linear  dense transform (+ReLU)             (gas_mlp2 for GIN)
    gas_push    in-batch rows -> history table l+1
    gas_spmm_t  backward aggregation over the CSC copy

It is timed in two forms that give the same result bit for bit: as these five
launches ("separate"), and with the aggregation reading the halo rows from the
history table itself and the transform storing its rows to the next table as
well (gas_spmm_hist, gas_linear_push / gas_mlp2_push: "in-place", no pull or
push launch, no halo copy, the transform's output is not re-read).
The headline value is the in-place form; the other one is reported beside it.

All inputs are resident in HBM before the timed region.  Prints one JSON line
with the whole-step throughput in aggregated edges per second, the roofline of
the dominant call (the aggregation) and the CPU oracle timed on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--config", type=int, default=4, help="benchmark configuration 0..4")
    p.add_argument("--scale", type=float, default=1.0, help="shrink the node count (debugging only)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--skip-spmm-t", action="store_true",
                   help="profiling aid: leave the backward aggregation out, so that the per-kernel averages of a "
                        "trace are those of the forward aggregation alone (the reported value is then not the metric)")
    p.add_argument("--path", choices=["both", "separate", "in-place"], default="both",
                   help="separate: pull, aggregate, transform, push, backward aggregate as five launches; in-place: the "
                        "aggregation reads the halo rows from the history table itself (gas_spmm_hist, same result bit "
                        "for bit, no pull launch); both (default): time K steps of each, headline = in-place")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also launch three plain 1 GiB contiguous copies (gas_pull without an index) before the "
                        "timed region: a kernel of known traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE by")
    p.add_argument("--cpu-sample-rows", type=int, default=0, help="rows of the batch the oracle is timed on")
    return p.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import configs, batches, rng

    gas.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config, args.scale)
    t0 = time.time()
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], cfg.self_loops)
    torch.cuda.synchronize()
    nb, nh, nv, nnz = sg.nb, sg.nh, sg.nv, sg.nnz
    nnz_t = int(sg.colptr[nb].item())            # entries in in-batch columns (backward over the batch only)
    log(f"[bench] {cfg.name}: N={g.n} nnz={g.nnz} | batch nb={nb} nh={nh} nnz_b={nnz} nnz_bt={nnz_t} "
        f"max_row={int((sg.rowptr[1:] - sg.rowptr[:-1]).max())} | generated in {time.time() - t0:.1f}s")

    from paper_2106_05609_amd.layer_step import LayerStep, NAMES as names
    ls = LayerStep(cfg, g, sg, rng, dev)
    F, dt, gin = ls.F, ls.dt, ls.gin

    if args.calibrate_copy:
        src = torch.ones((1 << 20, 256), dtype=torch.float32, device=dev)      # exactly 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            gas.gas_pull(src, None, dst, base=0, n=1 << 20)
        torch.cuda.synchronize()
        del src, dst

    by = ls.algorithmic_bytes()                   # what the method must move at least once, per launch
    spmm_hi = by.pop("spmm_no_reuse")             # no reuse of gathered rows at all
    flops = 2.0 * nb * F * F * (2 if gin else 1)
    edges = nnz + (0 if args.skip_spmm_t else nnz_t)

    def measure(fused):
        """W warm-up steps, then exactly K timed steps bracketed by synchronisation; per-call times from
        events recorded on the stream the kernels run on."""
        def step(ev=None):
            ls.run(None if ev is None else (lambda i: ev[i].record()), skip_spmm_t=args.skip_spmm_t, fused=fused)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(evs[k])
        torch.cuda.synchronize()
        ms_step = (time.perf_counter() - t0) / args.steps * 1e3
        per = {n: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, n in enumerate(names)}
        tag = "in-place" if fused else "separate"
        if fused:
            # the push is part of the transform call: its share = that call minus the plain transform, timed after
            # the K steps on the same buffers
            pe = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
            for a, b in pe:
                a.record()
                ls.transform(push=False)
                b.record()
            torch.cuda.synchronize()
            plain = sum(a.elapsed_time(b) for a, b in pe) / args.steps
            per["linear_push"] = per["linear"] + per["push"]
            per["linear"] = min(plain, per["linear_push"])
            per["push"] = per["linear_push"] - per["linear"]
        bytes_of = dict(by)
        if fused:
            bytes_of["push"] = by["push_in_epilogue"]
        kern = {}
        for n in names:
            if fused and n == "pull":
                continue                         # no such launch: the aggregation reads the history itself
            key = {"spmm": "spmm_hist", "linear": "linear_alone", "push": "push_in_epilogue"}.get(n, n) if fused else n
            if per[n] < 0.02 and fused and n == "push":
                # the transform is not bound by its stores: the extra output copy costs nothing measurable
                kern[key] = {"ms": round(per[n], 4), "alg_GB": round(bytes_of[n] / 1e9, 4), "alg_GBps": None,
                             "pct_hbm_peak": None}
                log(f"[bench] {tag:8s} {key:16s} {per[n]:8.3f} ms  alg {bytes_of[n] / 1e9:7.3f} GB  (hidden in the transform)")
                continue
            gbs = bytes_of[n] / (max(per[n], 1e-6) * 1e-3) / 1e9
            kern[key] = {"ms": round(per[n], 4), "alg_GB": round(bytes_of[n] / 1e9, 4), "alg_GBps": round(gbs, 1),
                         "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 2)}
            log(f"[bench] {tag:8s} {key:16s} {per[n]:8.3f} ms  alg {bytes_of[n] / 1e9:7.3f} GB  {gbs:8.1f} GB/s  "
                f"{100 * gbs / HBM_PEAK_GBS:5.1f}% of peak")
        sk = "spmm_hist" if fused else "spmm"
        lk = "linear_alone" if fused else "linear"
        mfma_peak = 157.3 if dt == torch.float32 else 2500.0        # dense MFMA TFLOP/s of the operand type
        kern[lk]["TFLOPs"] = round(flops / (per["linear"] * 1e-3) / 1e12, 2)
        kern[lk]["mfma_util"] = round(kern[lk]["TFLOPs"] / mfma_peak, 4)
        if fused:
            kern["linear_push"] = {"ms": round(per["linear_push"], 4),
                                   "TFLOPs": round(flops / (per["linear_push"] * 1e-3) / 1e12, 2)}
        kern[sk]["edges_per_s"] = round(nnz / (per["spmm"] * 1e-3), 1)
        kern[sk]["gathered_GBps"] = round(spmm_hi / (per["spmm"] * 1e-3) / 1e9, 1)
        t3 = (per["spmm"] + per["push"] + (0.0 if fused else per["pull"])) * 1e-3
        # bytes of the three operations as separate launches (pull + aggregation + push); the in-place variant
        # does the same work without writing and re-reading the halo copy and without re-reading the transform's
        # output, so its own byte count is smaller
        hbm3 = (by["pull"] + by["spmm"] + by["push"]) / t3 / 1e9
        hbm3_own = ((by["spmm"] + by["push_in_epilogue"]) / t3 / 1e9) if fused else hbm3
        step_sum = sum(per[n] for n in names)
        log(f"[bench] {tag:8s} step {ms_step:.3f} ms (sum of kernels {step_sum:.3f}) | pull+aggregate+push "
            f"{hbm3:.1f} GB/s = {100 * hbm3 / HBM_PEAK_GBS:.1f}% of HBM peak on the separate-launch byte count"
            + (f" ({hbm3_own:.1f} GB/s on its own byte count)" if fused else "")
            + f" | aggregation gathers {kern[sk]['gathered_GBps']} GB/s | transform {kern[lk]['TFLOPs']} TFLOP/s")
        return {"ms_per_step": ms_step, "value": edges / (ms_step * 1e-3), "kernels": kern, "per": per,
                "hbm_pull_spmm_push": {"GBps": round(hbm3, 1), "pct_of_peak": round(100 * hbm3 / HBM_PEAK_GBS, 2),
                                       "GBps_own_bytes": round(hbm3_own, 1)}}

    res = {}
    if args.path in ("separate", "both"):
        res["separate"] = measure(False)
    if args.path in ("in-place", "both"):
        res["in-place"] = measure(True)
    head = res.get("in-place") or res["separate"]
    fused_head = "in-place" in res
    per = head.pop("per")
    spmm_gbs = by["spmm"] / (per["spmm"] * 1e-3) / 1e9
    traffic = load_traffic(args.config, args.scale)
    out = {
        "metric": "GAS layer step: edges aggregated/sec + achieved HBM GB/s (% of peak), 1 GPU",
        "value": head["value"], "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if dt == torch.float32 else "bf16", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: middle layer {F}->{F}, first batch; "
                               + ("aggregate (halo rows read from the history table in place) + transform with the "
                                  "push in its epilogue + backward aggregate" if fused_head else
                                  "pull + aggregate + transform + push + backward aggregate"),
                   "N": g.n, "nnz": g.nnz, "nb": nb, "nh": nh, "nnz_b": nnz, "nnz_bt": nnz_t, "F": F,
                   "scale": args.scale},
        "hbm_pull_spmm_push": head["hbm_pull_spmm_push"],
        "kernels": head["kernels"],
        "roofline": {"kernel": ("gas_spmm_hist" if fused_head else "gas_spmm")
                               + " = spmm_chunk_kernel + spmm_heavy_reduce_kernel + spmm_rows_kernel", "bound": "hbm",
                     "achieved": round(spmm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(spmm_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                     # the two other figures of the aggregation: the measured traffic and the gathered bytes per second
                     "traffic_GBps": None if traffic is None else round(traffic / (per["spmm"] * 1e-3) / 1e9, 1),
                     "gathered_GBps": round(spmm_hi / (per["spmm"] * 1e-3) / 1e9, 1)},
    }
    if fused_head and "separate" in res:
        res["separate"].pop("per")
        out["separate_launches"] = res["separate"]   # the same step as five launches, pull included
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, g, sg, ls.hist_in, ls.x, ls.w1 if gin else ls.w,
                                           ls.w2 if gin else None, ls.gz, F, args.cpu_sample_rows)
    print(json.dumps(out), flush=True)


def load_traffic(config, scale):
    """HBM bytes per aggregation launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if scale != 1.0 or not os.path.exists(path):
        return None
    try:
        with open(path) as f:
            return json.load(f).get(f"config{config}", {}).get("spmm_bytes")
    except Exception:
        return None


def cpu_baseline(cfg, g, sg, hist_in, x, w, w2, gz, F, sample_rows):
    """The oracle's own pull + spmm + linear + push + spmm_t on the first rows of
    the same batch, sized for roughly 10-30 s of CPU work."""
    import numpy as np
    from oracle import ops as oops
    from tests.util import to_np
    nb = sg.nb
    rowptr = sg.rowptr.cpu().numpy()
    colall = sg.col.cpu().numpy()
    if sample_rows <= 0:
        # every k-th row of the batch, so that the sample has the batch's degree mix
        sample_rows = int(min(nb, max(1, round(nb * 24_000_000 / max(1, rowptr[-1])))))
    m = min(sample_rows, nb)
    rows = np.unique(np.linspace(0, nb - 1, m).astype(np.int64))
    m = rows.size
    lens = rowptr[rows + 1] - rowptr[rows]
    rp = np.zeros(m + 1, dtype=np.int32)
    rp[1:] = np.cumsum(lens)
    e = int(rp[-1])
    col = np.concatenate([colall[rowptr[r]:rowptr[r + 1]] for r in rows]).astype(np.int32)
    # renumber the sampled rows 0..m-1 in front (they stay "in-batch"), everything else behind them
    remap = np.full(sg.nv, -1, dtype=np.int64)
    remap[rows] = np.arange(m)
    others = np.setdiff1d(np.unique(col), rows)
    remap[others] = m + np.arange(others.size)
    col = remap[col].astype(np.int32)
    order = np.concatenate([rows, others])            # old local id of every new local id
    gin = cfg.op == "gin"
    n_id = sg.n_id.cpu().numpy()
    val = None if gin else oops.gcn_norm(rp, col, np.ascontiguousarray(n_id[order]), g.deg.cpu().numpy())
    dev_order = torch.from_numpy(order).to(x.device)
    xs = to_np(x[dev_order])                            # compact mini-batch tensor: sampled rows, then their neighbours
    n_halo = others.size
    hist_rows = to_np(hist_in[sg.n_id[dev_order[m:]].long()])   # compact stand-in for the history table
    idx_local = np.arange(n_halo, dtype=np.int32)
    wn = to_np(w)
    w2n = None if w2 is None else to_np(w2)
    gzn = to_np(gz[dev_order[:m]])
    hist_out = np.zeros((m, F), dtype=xs.dtype)
    t0 = time.perf_counter()
    xs[m:] = oops.pull(hist_rows, idx_local)
    t1 = time.perf_counter()
    z = oops.spmm(rp, col, val, xs, diag=(1.0 + cfg.gin_eps) if gin else 0.0)
    t2 = time.perf_counter()
    y = oops.mlp2(z, wn, w2n, relu_out=True) if gin else oops.linear(z, wn, relu=True)
    t3 = time.perf_counter()
    oops.push(y, np.arange(m, dtype=np.int32), hist_out)
    t4 = time.perf_counter()
    oops.spmm_t(rp, col, val, gzn, m, diag=(1.0 + cfg.gin_eps) if gin else 0.0)
    t5 = time.perf_counter()
    nnz_t = int((col < m).sum())
    total = t5 - t0
    log(f"[bench] oracle on {m} rows / {e} entries: pull {t1 - t0:.2f}s spmm {t2 - t1:.2f}s linear {t3 - t2:.2f}s "
        f"push {t4 - t3:.3f}s spmm_t {t5 - t4:.2f}s ({oops.num_threads()} threads)")
    return {"value": (e + nnz_t) / total, "unit": "edges/s", "cores": oops.num_threads(), "kind": "oracle",
            "sample": f"{m} evenly spaced in-batch rows of the same batch ({e} entries, {n_halo} neighbour rows pulled), "
                      f"same five calls, {total:.1f} s"}


if __name__ == "__main__":
    main()
