#!/usr/bin/env python3
"""A trace-driven model of the L2 caches under the in-place aggregation's schedule, for the question "would another
schedule fetch less?".  The batch subgraph and its plan come from the library as they are (the chunk and group lists
the kernels walk, gas_plan_copy_lists); bench/l2_model.c replays the gathers of each XCD through an LRU cache of
feature rows (8 x 3.5 MB of 16 ways, 512 work items in flight per XCD, 8 gathers per turn) and counts the misses.
Printed: the model's bytes for the schedule as built (to set against the FETCH_SIZE counters in profiles/), and for the
alternatives that were weighed: every L2-sized window of the heavy rows' chunks private to one XCD; windows cut into
units of P chunks dealt to the XCDs in turn; the light rows' cold gathers kept from displacing the most popular
rows; lower thresholds for "heavy".  Needs a GPU only to generate the graph and build the plan; the model itself
runs on the host (gcc compiles it into a temporary directory).  A table on stdout."""
import argparse
import ctypes as C
import os
import subprocess
import sys
import tempfile

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def load_model():
    d = tempfile.mkdtemp(prefix="l2_model_")
    so = os.path.join(d, "libl2_model.so")
    subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-o", so, os.path.join(ROOT, "bench", "l2_model.c")])
    lib = C.CDLL(so)
    lib.l2_model.restype = C.c_longlong
    return lib


def main():
    p = argparse.ArgumentParser()
    p.add_argument("--config", type=int, default=2)
    p.add_argument("--slots", type=int, default=3584, help="feature rows per L2 (3.5 MB of 1 KiB rows)")
    p.add_argument("--stats-only", action="store_true", help="only the popularity of the gathered rows")
    args = p.parse_args()
    if not torch.cuda.is_available():
        sys.exit("l2_model.py: no GPU visible (the graph and the plan are built on the device)")
    import paper_2106_05609_amd as gas
    from gas_inputs import configs, batches
    gas.lib()
    lib = load_model()
    dev = torch.device("cuda:0")
    cfg = configs.config(args.config)
    g = configs.build_graph(cfg, device=dev)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    sg = batches.batch_subgraph(g, bl[0], cfg.self_loops)
    F = cfg.widths[-2]
    row_bytes = F * (4 if cfg.dtype == torch.float32 else 2)
    slots = args.slots * 1024 // row_bytes
    ptr = sg.rowptr.cpu().numpy().astype(np.int64)
    col = np.ascontiguousarray(sg.col.cpu().numpy())

    def model(items, xcd_start, cold=None):
        items = np.ascontiguousarray(items, dtype=np.int32)
        xs = np.ascontiguousarray(xcd_start, dtype=np.int32)
        hits = C.c_longlong(0)
        miss = lib.l2_model(col.ctypes.data_as(C.c_void_p), items.ctypes.data_as(C.c_void_p), xs.ctypes.data_as(C.c_void_p),
                            slots, 16, 512, 8, None if cold is None else cold.ctypes.data_as(C.c_void_p), C.byref(hits))
        return miss * row_bytes / 1e9

    def in_turn(items, block):
        """Blocks of `block` consecutive items go to the XCDs in turn (what the hardware does with workgroups)."""
        x = (np.arange(len(items)) // block) % 8
        order = np.argsort(x, kind="stable")
        return items[order], np.concatenate([[0], np.cumsum(np.bincount(x, minlength=8))])

    def lists(threshold=0):
        plan = gas.gas_plan_create(sg.rowptr, sg.nnz, F, ind=sg.col, options=dict(heavy_threshold=threshold))
        group, heavy, chunk = plan.lists()
        chunk = chunk.reshape(-1, 3)
        light = np.stack([ptr[group[0::2]], ptr[group[1::2]]], 1)
        return light, chunk[:, 1:3].copy()

    # how much reuse the batch offers at all
    count = np.bincount(col, minlength=int(col.max()) + 1)
    used = count[count > 0]
    by_count = np.sort(used)[::-1].cumsum() / col.size
    print(f"{col.size} entries name {used.size} rows; used once: {(used == 1).sum()}, twice: {(used == 2).sum()}; share of "
          "the entries held by the most popular rows: " +
          ", ".join(f"{k}: {100 * by_count[min(k, used.size) - 1]:.1f} %" for k in (4096, 8192, 32768, 131072, 262144)))
    if args.stats_only:
        return
    light, chunks = lists()
    partial_gb = len(chunks) * F * 4 * 2 / 1e9                       # written once, read once by the reduction
    print(f"configs[{args.config}] {cfg.name}, first batch, width {F}: {len(chunks)} chunks of heavy rows "
          f"({int((chunks[:, 1] - chunks[:, 0]).sum())} entries), {len(light)} groups of light rows")
    it, xs = in_turn(chunks, 4)
    as_built_heavy = model(it, xs)
    it, xs = in_turn(light, 4)
    as_built_light = model(it, xs)
    print(f"as built: heavy rows {as_built_heavy:.1f} GB of gathered rows + {partial_gb:.1f} GB of partial sums; "
          f"light rows {as_built_light:.1f} GB")
    # windows private to one XCD: the window-ordered chunk list cut into eight ranges of equal numbers of entries
    cost = np.cumsum(chunks[:, 1] - chunks[:, 0])
    xs = [0] + [int(np.searchsorted(cost, cost[-1] * x / 8)) for x in range(1, 8)] + [len(chunks)]
    print(f"heavy rows, every window private to one XCD: {model(chunks, xs):.1f} GB + {partial_gb:.1f} GB of partial sums")
    # units of P chunks dealt to the XCDs in turn
    for P in (256, 1024, 4096):
        it, xs = in_turn(chunks, P)
        print(f"heavy rows, units of {P} chunks dealt to the XCDs in turn: {model(it, xs):.1f} GB + {partial_gb:.1f} GB")
    # light rows with the gathers of unpopular rows kept from displacing the K most popular ones
    rank = np.empty(count.size, dtype=np.int64)
    rank[np.argsort(-count, kind="stable")] = np.arange(count.size)
    it, xs = in_turn(light, 4)
    for K in (1024, 2048, 3072):
        cold = (rank[col] >= K).astype(np.uint8)
        print(f"light rows, the {K} most popular rows protected: {model(it, xs, cold):.1f} GB")
    # lower thresholds
    for thr in (256, 128, 64):
        lg, ch = lists(thr)
        it, xs = in_turn(ch, 4)
        h = model(it, xs)
        it, xs = in_turn(lg, 4)
        l = model(it, xs)
        pg = len(ch) * F * 4 * 2 / 1e9
        print(f"heavy above {thr} entries: heavy rows {h:.1f} GB + {pg:.1f} GB of partial sums, light rows {l:.1f} GB, "
              f"total {h + pg + l:.1f} GB (as built: {as_built_heavy + partial_gb + as_built_light:.1f} GB)")


if __name__ == "__main__":
    main()
