#!/usr/bin/env python3
"""Benchmark of the GAS layer step on one MI355X.

A step is one pass of the whole hot path over one mini-batch of the synthetic
workload for one layer:

    gas_pull    rows from outside the batch <- history table l (layer 1: every row <- the feature table)
    gas_spmm    aggregation over the batch subgraph
    gas_linear  dense transform (+ReLU)             (gas_mlp2 for GIN)
    gas_push    in-batch rows -> history table l+1  (not after the last layer)
    gas_spmm_t  backward aggregation over the CSC copy (not for layer 1)

It is timed in two forms that give the same result bit for bit: as these
launches ("separate"), and with the aggregation reading the rows from outside
the batch from their table itself and the transform storing its rows to the
next table as well (gas_spmm_hist, gas_linear_push / gas_mlp2_push:
"in-place").  The headline value is the in-place form of the middle layer of
config 4; config 2 and the first and last layers of both are reported beside
it under "configs".

All inputs are resident in HBM before the timed region.  Prints one JSON line
with the whole-step throughput in aggregated edges per second, the roofline of
the dominant call (the aggregation) against the published HBM peak and against
a plain device copy timed in the same run, the per-batch set-up time, and the
CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "GAS layer step: edges aggregated/sec + achieved HBM GB/s (% of peak), 1 GPU"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--config", type=int, default=None,
                   help="benchmark configuration 0..4; default: config 4 (headline) and config 2")
    p.add_argument("--layers", default="first,middle,last", help="which layers to time (the headline is the middle one)")
    p.add_argument("--scale", type=float, default=1.0, help="shrink the node count (debugging only)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--skip-spmm-t", action="store_true",
                   help="profiling aid: leave the backward aggregation out, so that the per-kernel averages of a "
                        "trace are those of the forward aggregation alone (the reported value is then not the metric)")
    p.add_argument("--only-spmm-t", action="store_true",
                   help="profiling aid: run the backward aggregation alone (its kernels share their names with the "
                        "forward aggregation's; the reported value is then not the metric)")
    p.add_argument("--path", choices=["both", "separate", "in-place"], default="both",
                   help="separate: pull, aggregate, transform, push, backward aggregate as five launches; in-place: the "
                        "aggregation reads the halo rows from the history table itself (gas_spmm_hist, same result bit "
                        "for bit, no pull launch); both (default): time K steps of each, headline = in-place")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="profiling aid: three extra plain 1 GiB copies after the timed ones, a kernel of known traffic "
                        "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE by")
    p.add_argument("--table-candidates", type=int, default=2,
                   help="allocations of the table the aggregation gathers from to try before the timed region (the "
                        "fastest is kept, all their times are reported under table_placement_ms; 1 = take what comes)")
    p.add_argument("--plan", default="", help="tuning aid: gas_plan_options as key=value,... (heavy_threshold, chunk, "
                                              "min_chunk, window_rows, xcd_ranges); the defaults are what is shipped")
    p.add_argument("--cpu-sample-rows", type=int, default=0, help="rows of the batch the oracle is timed on")
    return p.parse_args()


def measure_copy(gas, dev, extra=0):
    """GB/s of a plain 1 GiB device-to-device copy through the library's own row-copy kernel
    (gas_pull without an index): the ceiling this machine reaches for streaming, read + write."""
    src = torch.ones((1 << 20, 256), dtype=torch.float32, device=dev)          # exactly 1 GiB
    dst = torch.empty_like(src)
    for _ in range(3):
        gas.gas_pull(src, None, dst, base=0, n=1 << 20)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
    torch.cuda.synchronize()
    for i in range(10):
        ev[i].record()
        gas.gas_pull(src, None, dst, base=0, n=1 << 20)
    ev[10].record()
    torch.cuda.synchronize()
    ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(10))[5]
    for _ in range(extra):
        gas.gas_pull(src, None, dst, base=0, n=1 << 20)
    torch.cuda.synchronize()
    return 2.0 * (1 << 30) / (ms * 1e-3) / 1e9


def plan_options(args):
    return {k: int(v) for k, v in (kv.split("=") for kv in args.plan.split(",") if kv)} or None


def pct(gbs):
    return round(100 * gbs / HBM_PEAK_GBS, 2)


def measure(ls, args, fused):
    """W warm-up steps, then exactly K timed steps bracketed by synchronisation; per-call times from
    events recorded on the stream the kernels run on."""
    from paper_2106_05609_amd.layer_step import NAMES as names
    by = ls.algorithmic_bytes()
    spmm_hi = by["spmm_no_reuse"]
    tag = "in-place" if fused else "separate"

    def step(ev=None):
        ls.run(None if ev is None else (lambda i: ev[i].record()), skip_spmm_t=args.skip_spmm_t, fused=fused,
               only_spmm_t=args.only_spmm_t)
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
    if fused and ls.does_push:
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
        bytes_of["pull"] = by["pull_in_place"]
    kern = {}
    for n in names:
        if bytes_of[n] == 0:
            continue                         # no such launch in this form or for this layer
        key = {"spmm": "spmm_hist", "linear": "linear_alone", "push": "push_in_epilogue",
               "pull": "pull_in_batch_rows"}.get(n, n) if fused else n
        if per[n] < 0.02 and fused and n == "push":
            # the transform is not bound by its stores: the extra output copy costs nothing measurable
            kern[key] = {"ms": round(per[n], 4), "alg_GB": round(bytes_of[n] / 1e9, 4), "alg_GBps": None,
                         "pct_hbm_peak": None}
            log(f"[bench] {tag:8s} {key:18s} {per[n]:8.3f} ms  alg {bytes_of[n] / 1e9:7.3f} GB  (hidden in the transform)")
            continue
        gbs = bytes_of[n] / (max(per[n], 1e-6) * 1e-3) / 1e9
        kern[key] = {"ms": round(per[n], 4), "alg_GB": round(bytes_of[n] / 1e9, 4), "alg_GBps": round(gbs, 1),
                     "pct_hbm_peak": pct(gbs)}
        log(f"[bench] {tag:8s} {key:18s} {per[n]:8.3f} ms  alg {bytes_of[n] / 1e9:7.3f} GB  {gbs:8.1f} GB/s  "
            f"{pct(gbs):5.1f}% of peak")
    sk = "spmm_hist" if fused else "spmm"
    lk = "linear_alone" if fused else "linear"
    mfma_peak = 157.3 if ls.dt == torch.float32 else 2500.0        # dense MFMA TFLOP/s of the operand type
    kern[lk]["TFLOPs"] = round(ls.flops() / (max(per["linear"], 1e-6) * 1e-3) / 1e12, 2)
    kern[lk]["mfma_util"] = round(kern[lk]["TFLOPs"] / mfma_peak, 4)
    if fused and ls.does_push:
        kern["linear_push"] = {"ms": round(per["linear_push"], 4),
                               "TFLOPs": round(ls.flops() / (max(per["linear_push"], 1e-6) * 1e-3) / 1e12, 2)}
    kern[sk]["edges_per_s"] = round(ls.nnz / (max(per["spmm"], 1e-6) * 1e-3), 1)
    kern[sk]["gathered_GBps"] = round(spmm_hi / (max(per["spmm"], 1e-6) * 1e-3) / 1e9, 1)
    # pull + aggregation + push, three ways:
    #  five_launch_literal  bytes of the three operations as separate launches / the time those launches take
    #  in_place_own_bytes   the in-place form's own, smaller byte count (no halo copy written and re-read, the
    #                       transform's output not re-read) / the time it needs for that work
    #  work_equivalent      the separate-launch byte count / the in-place form's time: not a bandwidth (the in-place
    #                       form moves no such bytes), only how fast the same work gets done
    t3 = max(per["pull"] + per["spmm"] + per["push"], 1e-6) * 1e-3
    lit = by["pull"] + by["spmm"] + by["push"]
    own = bytes_of["pull"] + by["spmm"] + bytes_of["push"]
    hbm = {}
    if fused:
        hbm["in_place_own_bytes"] = {"GBps": round(own / t3 / 1e9, 1), "pct_of_peak": pct(own / t3 / 1e9)}
        hbm["work_equivalent"] = {"GBps": round(lit / t3 / 1e9, 1), "pct_of_peak": pct(lit / t3 / 1e9)}
    else:
        hbm["five_launch_literal"] = {"GBps": round(lit / t3 / 1e9, 1), "pct_of_peak": pct(lit / t3 / 1e9)}
    edges = ls.nnz + (ls.nnz_t if ls.does_spmm_t and not args.skip_spmm_t else 0)
    log(f"[bench] {tag:8s} {ls.kind} layer: step {ms_step:.3f} ms (sum of calls {sum(per[n] for n in names):.3f}) | "
        f"pull+aggregate+push {json.dumps(hbm)} | transform {kern[lk]['TFLOPs']} TFLOP/s")
    return {"ms_per_step": round(ms_step, 4), "edges_per_s": round(edges / (ms_step * 1e-3), 1), "kernels": kern,
            "hbm_pull_spmm_push": hbm, "_per": per, "_by": by}


def run_config(gas, cfg_id, args, dev, layers, want_baseline):
    from paper_2106_05609_amd.layer_step import LayerStep
    from gas_inputs import configs, batches, rng
    cfg = configs.config(cfg_id, args.scale)
    # The big tables first, while the device memory is untouched: where the driver puts tens of gigabytes decides up
    # to 10 % of the time of the random gathers from them, and allocations made before anything else has used and
    # freed memory come out best most of the time; of several such candidates the fastest is kept (place_table).
    k = max(1, args.table_candidates) if args.path != "separate" else 1
    hidden, f0 = cfg.widths[-2], cfg.widths[0]
    pre_hidden = [torch.empty((cfg.n, hidden), dtype=cfg.dtype, device=dev) for _ in range(k)]
    pre_out = torch.empty((cfg.n, hidden), dtype=cfg.dtype, device=dev)
    pre_feat = [torch.empty((cfg.n, f0), dtype=cfg.dtype, device=dev) for _ in range(k if "first" in layers else 0)]
    es = 4 if cfg.dtype == torch.float32 else 2
    pools = tuple(torch.empty(cfg.n * max(cfg.widths) * es, dtype=torch.uint8, device=dev) for _ in range(2))
    t0 = time.time()
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], cfg.self_loops)
    torch.cuda.synchronize()
    nb, nh, nnz = sg.nb, sg.nh, sg.nnz
    nnz_t = int(sg.colptr[nb].item())            # entries in in-batch columns (backward over the batch only)
    log(f"[bench] {cfg.name}: N={g.n} nnz={g.nnz} | batch nb={nb} nh={nh} nnz_b={nnz} nnz_bt={nnz_t} "
        f"max_row={int((sg.rowptr[1:] - sg.rowptr[:-1]).max())} | generated in {time.time() - t0:.1f}s")
    out = {"name": cfg.name, "dtype": "f32" if cfg.dtype == torch.float32 else "bf16",
           "N": g.n, "nnz": g.nnz, "nb": nb, "nh": nh, "nnz_b": nnz, "nnz_bt": nnz_t, "layers": {}}
    bg, baseline, head = None, None, None
    for kind in layers:
        ls = LayerStep(cfg, g, sg, rng, dev, kind=kind, bg=bg, plan_options=plan_options(args),
                       tables_in=pre_feat if kind == "first" else pre_hidden, table_out=pre_out, pools=pools)
        if bg is None:
            bg = ls.bg
            out["setup_ms"] = bg.setup_ms           # once per batch subgraph, reused by every layer and epoch
            log(f"[bench] per-batch set-up (plans, coefficients, fused sources): {bg.setup_ms}")
        res = {"widths": [ls.F_in, ls.F_out]}
        if len(ls.candidates) > 1:
            res["table_placement_ms"] = ls.place_table(len(ls.candidates))
            log(f"[bench] {kind} layer: in-place aggregation on {len(res['table_placement_ms'])} allocations of its "
                f"table, kept first: {res['table_placement_ms']} ms")
            if kind == "first":
                pre_feat = list(ls.candidates)
            else:
                pre_hidden = list(ls.candidates)
        if args.path in ("separate", "both"):
            res["separate"] = measure(ls, args, False)
        if args.path in ("in-place", "both"):
            res["in-place"] = measure(ls, args, True)
        if kind == "middle":
            head = {k: dict(v) for k, v in res.items() if isinstance(v, dict)}
            head["F"] = ls.F_in
            if want_baseline:
                baseline = cpu_baseline(cfg, g, sg, ls.hist_in, ls.x, ls.w1 if ls.gin else ls.w,
                                        ls.w2 if ls.gin else None, ls.gz, ls.F_in, args.cpu_sample_rows)
        for form in ("separate", "in-place"):
            if form in res:
                res[form] = {k: v for k, v in res[form].items() if not k.startswith("_")}
        out["layers"][kind] = res
        del ls
        torch.cuda.empty_cache()
    del pre_hidden, pre_out, pre_feat, pools
    return out, head, baseline


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    import paper_2106_05609_amd as gas
    gas.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    layers = [k for k in ("first", "middle", "last") if k in args.layers.split(",")]
    if "middle" not in layers:
        layers.append("middle")                  # the headline layer is always timed
    cfg_ids = [args.config] if args.config is not None else [4, 2]

    copy_gbs = measure_copy(gas, dev, extra=3 if args.calibrate_copy else 0)
    log(f"[bench] plain 1 GiB device copy (gas_pull without an index): {copy_gbs:.1f} GB/s read + write = "
        f"{pct(copy_gbs):.1f}% of the published peak")

    per_cfg, head, baseline, head_id = {}, None, None, cfg_ids[0]
    for i, c in enumerate(cfg_ids):
        rec, h, b = run_config(gas, c, args, dev, layers, want_baseline=(i == 0 and not args.no_cpu_baseline))
        per_cfg[str(c)] = rec
        if i == 0:
            head, baseline = h, b
        torch.cuda.empty_cache()

    hrec = per_cfg[str(head_id)]
    form = "in-place" if "in-place" in head else "separate"
    hm = head[form]
    per, by = hm["_per"], hm["_by"]
    fused_head = form == "in-place"
    spmm_gbs = by["spmm"] / (max(per["spmm"], 1e-6) * 1e-3) / 1e9
    traffic, traffic_src = load_traffic(head_id, args.scale)
    F = head["F"]
    hbm = dict(hm["hbm_pull_spmm_push"])
    if "separate" in head and fused_head:
        hbm.update(head["separate"]["hbm_pull_spmm_push"])
    edges = hrec["nnz_b"] + (0 if args.skip_spmm_t else hrec["nnz_bt"])
    out = {
        "metric": METRIC,
        "value": edges / (hm["ms_per_step"] * 1e-3), "unit": "edges/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": hm["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": hrec["dtype"], "data": "synthetic",
        "config": {"workload": f"configs[{head_id}] {hrec['name']}: middle layer {F}->{F}, first batch; "
                               + ("aggregate (halo rows read from the history table in place) + transform with the "
                                  "push in its epilogue + backward aggregate" if fused_head else
                                  "pull + aggregate + transform + push + backward aggregate"),
                   "N": hrec["N"], "nnz": hrec["nnz"], "nb": hrec["nb"], "nh": hrec["nh"], "nnz_b": hrec["nnz_b"],
                   "nnz_bt": hrec["nnz_bt"], "F": F, "scale": args.scale},
        # pull + aggregation + push of the headline layer; pct_of_peak of the literal (five-launch) reading first
        "hbm_pull_spmm_push": hbm,
        "kernels": hm["kernels"],
        "roofline": {"kernel": ("gas_spmm_hist" if fused_head else "gas_spmm")
                               + " = spmm_chunk_kernel + spmm_heavy_reduce_kernel + spmm_rows_kernel", "bound": "hbm",
                     "achieved": round(spmm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(spmm_gbs / HBM_PEAK_GBS, 4),
                     # what this machine reaches for a plain device copy, timed in this run, and the same call against it
                     "attainable": round(copy_gbs, 1), "frac_of_attainable": round(spmm_gbs / copy_gbs, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "traffic_GBps": None if traffic is None else round(traffic / (max(per["spmm"], 1e-6) * 1e-3) / 1e9, 1),
                     "gathered_GBps": round(by["spmm_no_reuse"] / (max(per["spmm"], 1e-6) * 1e-3) / 1e9, 1)},
        "setup_ms": hrec.get("setup_ms"),
        "configs": per_cfg,
    }
    if baseline is not None:
        out["cpu_baseline"] = baseline
    print(json.dumps(out), flush=True)


def source_sha():
    """Hash of the sources of the aggregation kernels: a traffic figure measured with rocprofv3 counters is only
    reported while the kernels it was measured on are unchanged."""
    h = hashlib.sha256()
    for f in ("spmm.hip", "common.h"):
        with open(os.path.join(ROOT, "paper_2106_05609_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def load_traffic(config, scale):
    """HBM bytes per aggregation launch from the committed rocprofv3 counter summary, if there is one for
    this configuration AND it was measured on the kernel sources of this tree; else (None, why)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if scale != 1.0 or not os.path.exists(path):
        return None, None
    try:
        with open(path) as f:
            rec = json.load(f).get(f"config{config}", {})
    except Exception:
        return None, None
    if not rec:
        return None, None
    if rec.get("source_sha") != source_sha():
        return None, f"{rec.get('profile')} was measured on other kernel sources ({rec.get('source_sha')}): not reported"
    return rec.get("spmm_bytes"), f"{rec.get('profile')} @ sources {rec.get('source_sha')}"


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
