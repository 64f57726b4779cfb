#!/usr/bin/env python3
"""Timing of the backward pass of one middle layer (256 -> 256) at the sizes of
the benchmark configurations: loss and its gradient, ReLU backward, input
gradient, weight gradient and the weight update, as the C-ABI calls a training
step makes.
One JSON line on stdout, a table on stderr."""
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
    p.add_argument("--reps", type=int, default=20)
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_backward.py: no GPU visible")
    import paper_2106_05609_amd as gas
    from gas_inputs import configs, rng
    gas.lib()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config)
    nb = cfg.n // cfg.n_blocks * cfg.blocks_per_batch
    F, dt = cfg.widths[-2], cfg.dtype
    s = 4 if dt == torch.float32 else 2
    z = rng.normal_matrix(0, 700, nb, F, dev, dt)
    y = torch.relu(rng.normal_matrix(0, 701, nb, F, dev, dt))
    gy = rng.normal_matrix(0, 702, nb, F, dev, dt)
    w = rng.glorot_uniform(0, 703, F, F, dev, dt)
    gp, gz = torch.empty_like(gy), torch.empty_like(z)
    dw = torch.zeros((F, F), dtype=torch.float32, device=dev)
    ws = torch.empty(gas.gas_linear_bwd_weight_workspace(nb, F, F), dtype=torch.uint8, device=dev)
    labels = (torch.arange(nb, device=dev) % F).to(torch.int32)
    loss_rows = torch.empty(nb, dtype=torch.float32, device=dev)
    loss_sum = torch.empty(1, dtype=torch.float32, device=dev)
    calls = {
        "softmax_xent": (lambda: gas.gas_softmax_xent(z, labels, gz, loss_rows, loss_sum, scale=1.0 / nb),
                         2 * nb * F * s + 12 * nb, 0.0),
        "sgd_step": (lambda: gas.gas_sgd_step(w, dw, 1e-9), F * F * (2 * s + 4), 0.0),
        "relu_bwd": (lambda: gas.gas_relu_bwd(gy, y, gp), 3 * nb * F * s, 0.0),
        "linear_bwd_input": (lambda: gas.gas_linear_bwd_input(gp, w, gz), 2 * nb * F * s + F * F * s, 2.0 * nb * F * F),
        "linear_bwd_weight": (lambda: gas.gas_linear_bwd_weight(z, gp, dw, ws), 2 * nb * F * s + F * F * 4, 2.0 * nb * F * F),
    }
    out = {"workload": f"configs[{args.config}] {cfg.name}: backward of the transform of one middle layer, "
                       f"{nb} rows, {F} -> {F}, {'f32' if s == 4 else 'bf16'}", "calls": {}}
    for name, (fn, nbytes, flops) in calls.items():
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.reps
        rec = {"ms": round(ms, 4), "alg_GB": round(nbytes / 1e9, 3), "GBps": round(nbytes / ms / 1e6, 1),
               "TFLOPs": round(flops / ms / 1e9, 1)}
        out["calls"][name] = rec
        print(f"{name:18s} {ms:8.3f} ms  {rec['GBps']:8.1f} GB/s  {rec['TFLOPs']:7.1f} TFLOP/s", file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
