"""The seeded input generators: simple undirected graphs, reproducible, with
the stated structure (CPU only)."""
from collections import deque

import numpy as np
import torch

from gas_inputs import configs, batches, graphs, rng
from tests.util import to_np


def _check_simple_undirected(g):
    rp, cl = to_np(g.rowptr), to_np(g.col)
    assert rp[0] == 0 and rp[-1] == cl.size and np.array_equal(np.diff(rp), to_np(g.deg))
    row = np.repeat(np.arange(g.n), np.diff(rp))
    assert (row != cl).all()                                         # no self-loops
    key = row.astype(np.int64) * g.n + cl
    assert (np.diff(key) > 0).all()                                  # sorted rows, no multi-edges
    assert np.array_equal(np.sort(cl.astype(np.int64) * g.n + row), key)   # symmetric


def test_generators_give_simple_undirected_graphs_of_the_stated_shape():
    g0 = configs.build_graph(configs.config(0))
    _check_simple_undirected(g0)
    assert g0.n == 2048 and g0.n_blocks == 4
    # expected degree 511*0.008 + 1536*0.0005 = 4.86
    assert abs(g0.nnz / g0.n - 4.86) < 0.3
    g1 = configs.build_graph(configs.config(1, 0.05))
    _check_simple_undirected(g1)
    assert abs(g1.nnz / g1.n - 10.0) < 0.3
    rp, cl = to_np(g1.rowptr), to_np(g1.col)
    row = np.repeat(np.arange(g1.n), np.diff(rp))
    bsz = g1.n // g1.n_blocks
    assert abs((row // bsz == cl // bsz).mean() - 0.85) < 0.02       # intra-block fraction
    g2 = configs.build_graph(configs.config(2, 0.01))
    _check_simple_undirected(g2)
    assert 40 < g2.nnz / g2.n <= 50 and int(g2.deg.max()) <= 880   # cap on the expected degree; realised one scatters around it


def test_generation_is_reproducible_and_seed_dependent():
    a = configs.build_workload(configs.config(2, 0.004))
    b = configs.build_workload(configs.config(2, 0.004))
    assert torch.equal(a.graph.col, b.graph.col) and torch.equal(a.x, b.x) and torch.equal(a.weights[1], b.weights[1])
    c = configs.config(2, 0.004)
    c.seed = 5
    c = configs.build_workload(c)
    assert not torch.equal(a.x, c.x) and a.graph.nnz != c.graph.nnz
    # chunked generation equals one-shot generation
    assert torch.equal(rng.normal_matrix(1, 2, 1000, 7, chunk_rows=64), rng.normal_matrix(1, 2, 1000, 7))
    x = rng.normal_matrix(1, 3, 4000, 50)
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01


def test_bfs_order_is_the_sequential_queue_order():
    g = graphs.chung_lu(3000, 2.1, 6.0, 200, seed=3)
    order = to_np(graphs.bfs_order(g, 3))
    rp, cl = to_np(g.rowptr), to_np(g.col)
    start = int(rng.randint(3, 8, torch.zeros(1, dtype=torch.int64), g.n))
    seen = np.zeros(g.n, bool)
    want = []
    nxt_unseen = 0
    q = deque([start])
    seen[start] = True
    while len(want) < g.n:
        if not q:
            while seen[nxt_unseen]:
                nxt_unseen += 1
            seen[nxt_unseen] = True
            q.append(nxt_unseen)
        v = q.popleft()
        want.append(v)
        for w in cl[rp[v]:rp[v + 1]]:
            if not seen[w]:
                seen[w] = True
                q.append(int(w))
    assert np.array_equal(order, np.array(want))
    h = graphs.relabel(g, torch.from_numpy(order), graphs.equal_block_ptr(g.n, 8))
    _check_simple_undirected(h)
    assert np.array_equal(np.sort(to_np(h.deg)), np.sort(to_np(g.deg)))
    assert np.array_equal(to_np(h.deg), to_np(g.deg)[order])


def test_split_partitions_the_nodes_and_halo_is_the_one_hop_ring():
    cfg = configs.config(3, 0.02)
    g = configs.build_graph(cfg)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    assert len(bl) == 8
    allv = torch.cat(bl)
    assert torch.equal(torch.sort(allv).values, torch.arange(g.n))
    sizes = to_np(g.block_ptr[1:] - g.block_ptr[:-1])
    assert sizes.max() - sizes.min() <= 1
    sg = batches.batch_subgraph(g, bl[0], True)
    n_id = to_np(sg.n_id)
    assert (np.diff(n_id[:sg.nb]) > 0).all() and (np.diff(n_id[sg.nb:]) > 0).all()
    rp, cl = to_np(g.rowptr), to_np(g.col)
    nbrs = set()
    for v in n_id[:sg.nb]:
        nbrs.update(cl[rp[v]:rp[v + 1]].tolist())
    assert set(n_id[sg.nb:].tolist()) == nbrs - set(n_id[:sg.nb].tolist())
    assert sg.nnz == sum(rp[v + 1] - rp[v] for v in n_id[:sg.nb]) + sg.nb
