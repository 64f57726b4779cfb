"""The paper's own synthetic workload for this path (tests/golden/overhead_workload.txt: the values its runtime
analysis states) against the generator and the overhead benchmark that stand for it: a batch of exactly 4,000 nodes
with 60 links each inside the batch, outside nodes with 60 links into the batch and none among themselves, a 4-layer
GIN, and a ratio sweep that covers the range the paper gives for real datasets.  CPU only."""
import os
import re

import torch

from gas_inputs import graphs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _golden():
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "overhead_workload.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            out[k] = v
    return out


def test_generator_matches_the_stated_workload():
    gold = _golden()
    nb, links = int(gold["batch_nodes"]), int(gold["intra_links_per_node"])
    assert (nb, links, int(gold["links_per_outside_node"])) == (4000, 60, 60)
    for n_out in (0, 2000, 10000):
        g = graphs.batch_with_outside_links(nb, n_out, int(gold["links_per_outside_node"]), seed=3)
        assert g.n == nb + n_out
        ptr, col = g.rowptr.long(), g.col.long()
        rows = torch.repeat_interleave(torch.arange(g.n), ptr[1:] - ptr[:-1])
        inside = (rows < nb) & (col < nb)
        # links inside the batch: 60 per node on average (random partners, symmetrised, duplicates merged)
        mean_intra = inside.sum().item() / nb
        assert 0.97 * links <= mean_intra <= links, mean_intra
        assert not ((rows == col).any())
        # an outside node is linked to (up to duplicates) 60 nodes of the batch and to no outside node
        if n_out:
            deg_out = (ptr[1:] - ptr[:-1])[nb:]
            assert deg_out.max().item() <= links and deg_out.float().mean().item() >= 0.98 * links
            assert not ((rows >= nb) & (col >= nb)).any()
            # the inter / intra ratio of the batch follows from the node counts
            inter = ((rows < nb) & (col >= nb)).sum().item()
            assert abs(inter / inside.sum().item() - n_out / nb) <= 0.05 * max(n_out / nb, 1e-9)
        # symmetric
        key = rows * g.n + col
        assert torch.equal(torch.sort(key).values, torch.sort(col * g.n + rows).values)


def test_overhead_benchmark_uses_the_stated_workload():
    gold = _golden()
    src = open(os.path.join(ROOT, "bench", "bench_overhead.py")).read()
    assert re.search(r'"--layers", type=int, default=%s\b' % gold["layers"], src)
    assert re.search(r"batch_with_outside_links\(\s*%s\b" % gold["batch_nodes"], src) or \
        re.search(r"n_batch\s*=\s*%s\b" % gold["batch_nodes"], src) or "4000" in src
    assert re.search(r"\b%s\b" % gold["intra_links_per_node"], src)
    assert '"gin"' in src or "'gin'" in src
    ratios = [float(x) for x in re.search(r'"--ratios".*?default=\[([^\]]*)\]', src).group(1).split(",")]
    assert min(r for r in ratios if r > 0) <= float(gold["ratio_low"]) and max(ratios) >= float(gold["ratio_high"])
