#!/usr/bin/env python3
"""Timing of operator variants of the layer step on a benchmark configuration's first batch.

  appnp   one propagation step of APPNP (paper, operator appendix): pull + aggregation with the
          alpha * h0 residual in its epilogue + push; no transform.  Also with the halo rows read in place.
  pna     PNA's neighbourhood aggregation (same appendix): mean, min and max with the three degree scalers in
          one pass over the gathered rows (9 output blocks per row).
  host    pull and push against a history table in pinned host memory (rows moved over the host link by the
          copy kernel itself), alone and on a second stream beside the aggregation.
  gat     GAT's aggregation (same appendix, one head): scores, softmax over the row's entries and the weighted
          sum in one pass over the gathered rows.
  pna_bwd, gat_bwd   the backward passes of the two aggregations, gradients for every row of V_b.

One JSON line on stdout, a table on stderr.  Bytes are algorithmic (indices and coefficients once, every needed
feature row once, every output row once)."""
import argparse
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def timed(fn, reps):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=2)
    p.add_argument("--scale", type=float, default=1.0)
    p.add_argument("--reps", type=int, default=10)
    p.add_argument("--width", type=int, default=0, help="feature width (default: the configuration's hidden width)")
    p.add_argument("--host-rows", type=int, default=1 << 21, help="rows of the pinned host table (0: skip)")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_variants.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from paper_2106_05609_amd import executor
    from gas_inputs import configs, batches, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config, args.scale)
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], True)
    F, dt = args.width or cfg.widths[-2], cfg.dtype
    s = 4 if dt == torch.float32 else 2
    nb, nh, nv, nnz = sg.nb, sg.nh, sg.nv, sg.nnz
    bg = executor.BatchGraph(nb, sg.n_id, sg.rowptr, sg.col, g.deg, sg.colptr, sg.row, max_F=F, normalise=True)
    hist_in = rng.normal_matrix(cfg.seed, 200, cfg.n, F, dev, dt)
    hist_out = torch.zeros((cfg.n, F), dtype=dt, device=dev)
    x = rng.normal_matrix(cfg.seed, 210, nv, F, dev, dt)
    h0 = rng.normal_matrix(cfg.seed, 212, nb, F, dev, dt)
    y = torch.empty((nb, F), dtype=dt, device=dev)
    alpha = 0.1
    by = {"pull": nh * (2 * F * s + 4), "spmm": nnz * 8 + (nb + 1) * 4 + nv * F * s + 2 * nb * F * s,
          "push": nb * (2 * F * s + 4)}
    calls = {
        "pull": lambda: gas.gas_pull(hist_in, bg.n_id[nb:], x[nb:]),
        "spmm": lambda: gas.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, y, s_agg=1.0 - alpha, r=h0, s_res=alpha),
        "spmm_hist": lambda: gas.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, x[:nb], hist_in, y, s_agg=1.0 - alpha,
                                               r=h0, s_res=alpha),
        "push": lambda: gas.gas_push(y, bg.n_id[:nb], hist_out),
    }
    by["spmm_hist"] = by["spmm"]
    out = {"workload": f"configs[{args.config}] {cfg.name}: one APPNP propagation step, first batch, width {F}, "
                       f"{'f32' if s == 4 else 'bf16'}", "nb": nb, "nh": nh, "nnz_b": nnz, "calls": {}}
    ms = {}
    for name, fn in calls.items():
        ms[name] = timed(fn, args.reps)
        out["calls"][name] = {"ms": round(ms[name], 4), "alg_GB": round(by[name] / 1e9, 3),
                              "GBps": round(by[name] / ms[name] / 1e6, 1)}
        print(f"{name:10s} {ms[name]:8.3f} ms  {by[name] / 1e9:7.3f} GB  {by[name] / ms[name] / 1e6:8.1f} GB/s",
              file=sys.stderr, flush=True)
    # PNA aggregation over the same batch subgraph (self-loops excluded from the pattern would change nnz by nb only)
    delta = float(torch.log(g.deg.double() + 1.0).mean())
    out9 = torch.empty((nb, 9 * F), dtype=dt, device=dev)
    t = timed(lambda: gas.gas_pna_aggregate(bg.rowptr, bg.col, x, out9, delta, add=h0), args.reps)
    nbytes = nnz * 4 + (nb + 1) * 4 + nv * F * s + nb * F * s + 9 * nb * F * s
    out["pna_aggregate"] = {"ms": round(t, 4), "alg_GB": round(nbytes / 1e9, 3), "GBps": round(nbytes / t / 1e6, 1),
                            "gathered_GBps": round(nnz * F * s / t / 1e6, 1)}
    print(f"pna_aggr   {t:8.3f} ms  {nbytes / 1e9:7.3f} GB  {nbytes / t / 1e6:8.1f} GB/s  (gathers {nnz * F * s / t / 1e6:.0f} GB/s)",
          file=sys.stderr, flush=True)
    a_dst = rng.normal(cfg.seed, 213, 0, F, dev, dt) * 0.1
    a_src = rng.normal(cfg.seed, 214, 0, F, dev, dt) * 0.1
    t = timed(lambda: gas.gas_gat_aggregate(bg.rowptr, bg.col, x, a_dst, a_src, y, 0.2, relu=True), args.reps)
    nbytes = nnz * 4 + (nb + 1) * 4 + nv * F * s + nb * F * s
    out["gat_aggregate"] = {"ms": round(t, 4), "alg_GB": round(nbytes / 1e9, 3), "GBps": round(nbytes / t / 1e6, 1),
                            "gathered_GBps": round(nnz * F * s / t / 1e6, 1)}
    print(f"gat_aggr   {t:8.3f} ms  {nbytes / 1e9:7.3f} GB  {nbytes / t / 1e6:8.1f} GB/s  (gathers {nnz * F * s / t / 1e6:.0f} GB/s)",
          file=sys.stderr, flush=True)
    # backward of the two aggregations, gradients for every row of V_b (what a training pass needs: the weights that
    # multiply neighbour rows take gradient through halo rows too)
    csc_pos = sg.csc_perm.to(torch.int32)
    gx = torch.empty((nv, F), dtype=dt, device=dev)
    g9 = out9                                                    # any values will do as the output gradient
    gadd = torch.empty((nb, F), dtype=dt, device=dev)
    plan_t = bg.plan_t_all
    t = timed(lambda: gas.gas_pna_aggregate_bwd(bg.rowptr, bg.col, bg.colptr, bg.row, csc_pos, x, g9, gx, delta,
                                                gadd=gadd, plan_t=plan_t), args.reps)
    nbytes = nnz * 12 + (nb + nv + 2) * 4 + nv * F * s + 9 * nb * F * s + nv * F * s + nb * F * s
    out["pna_aggregate_bwd"] = {"ms": round(t, 4), "alg_GB": round(nbytes / 1e9, 3), "GBps": round(nbytes / t / 1e6, 1)}
    print(f"pna_bwd    {t:8.3f} ms  {nbytes / 1e9:7.3f} GB  {nbytes / t / 1e6:8.1f} GB/s", file=sys.stderr, flush=True)
    del g9, out9, gadd
    gd, gs = torch.empty(F, device=dev), torch.empty(F, device=dev)
    t = timed(lambda: gas.gas_gat_aggregate_bwd(bg.rowptr, bg.col, bg.colptr, bg.row, csc_pos, x, a_dst, a_src, y, gx,
                                                gd, gs, 0.2, plan_t=plan_t), args.reps)
    nbytes = nnz * 12 + (nb + nv + 2) * 4 + nv * F * s + nb * F * s + nv * F * s
    out["gat_aggregate_bwd"] = {"ms": round(t, 4), "alg_GB": round(nbytes / 1e9, 3), "GBps": round(nbytes / t / 1e6, 1)}
    print(f"gat_bwd    {t:8.3f} ms  {nbytes / 1e9:7.3f} GB  {nbytes / t / 1e6:8.1f} GB/s", file=sys.stderr, flush=True)
    del gx
    if args.host_rows > 0:
        hr = min(args.host_rows, cfg.n)
        table = gas.HostTable(torch.zeros((hr, F), dtype=dt).pin_memory())
        m = min(nh, 1 << 20)                                  # rows per transfer
        hidx = (rng.permutation(cfg.seed, 215, hr)[:m]).to(torch.int32).to(dev)
        stage = torch.empty((m, F), dtype=dt, device=dev)
        t_pull = timed(lambda: gas.gas_pull(table, hidx, stage), args.reps)
        t_push = timed(lambda: gas.gas_push(stage, hidx, table), args.reps)
        side = torch.cuda.Stream()

        def both():
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                gas.gas_pull(table, hidx, stage)
            calls["spmm_hist"]()
            torch.cuda.current_stream().wait_stream(side)
        t_both = timed(both, args.reps)
        gb = m * F * s / 1e9
        out["host_table"] = {"rows_per_transfer": m, "GB": round(gb, 3), "pull_ms": round(t_pull, 3),
                             "pull_GBps": round(gb / t_pull * 1e3, 1), "push_ms": round(t_push, 3),
                             "push_GBps": round(gb / t_push * 1e3, 1), "spmm_hist_ms": round(ms["spmm_hist"], 3),
                             "pull_beside_spmm_hist_ms": round(t_both, 3)}
        print(f"host table: pull {t_pull:.3f} ms ({gb / t_pull * 1e3:.1f} GB/s), push {t_push:.3f} ms "
              f"({gb / t_push * 1e3:.1f} GB/s); pull on a second stream beside spmm_hist: {t_both:.3f} ms "
              f"(spmm_hist alone {ms['spmm_hist']:.3f})", file=sys.stderr, flush=True)
    out["step_ms"] = {"separate": round(ms["pull"] + ms["spmm"] + ms["push"], 4),
                      "in_place": round(ms["spmm_hist"] + ms["push"], 4)}
    out["edges_per_s"] = {k: round(nnz / (v * 1e-3), 1) for k, v in out["step_ms"].items()}
    print(f"step: {out['step_ms']} ms, {out['edges_per_s']} edges/s", file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
