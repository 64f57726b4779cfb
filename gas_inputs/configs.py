"""The five benchmark configurations as seeded synthetic workloads.

Each stands in for a dataset class of the paper's dataset-statistics table
(none of those datasets is used or reproduced): config 0 a Cora-scale block
model, config 1 a mid-size sparse community graph, config 2 the shape of the
paper's largest product graph (2.4 M nodes, 100 features), config 3 the shape
of its 169 k-node citation graph with the 64-layer deep model, config 4 a
power-law graph beyond the paper's sizes in bf16.

`scale` < 1 shrinks the node count (and nothing else) for tests.
"""
from dataclasses import dataclass, field
import math

import torch

from . import rng, graphs, batches


@dataclass
class Config:
    name: str
    op: str                   # "gcn" | "gcnii" | "gin"
    n: int
    n_blocks: int
    blocks_per_batch: int
    widths: list              # [F_0, F_1, ..., F_L]
    dtype: torch.dtype
    graph: dict               # generator arguments
    seed: int = 0
    alpha: float = 0.0        # GCNII initial-residual weight
    gin_eps: float = 0.0
    gin_hidden: int = 0       # width of the hidden Linear of each GIN MLP
    self_loops: bool = True
    history_init: str = "normal"   # "zeros" | "normal"

    @property
    def n_layers(self) -> int:
        return len(self.widths) - 1


def config(i: int, scale: float = 1.0) -> Config:
    def sc(n, blocks):
        return max(blocks * 8, int(round(n * scale)))
    if i == 0:
        return Config("tiny-gcn2", "gcn", sc(2048, 4), 4, 1, [64, 64, 64], torch.float32,
                      dict(kind="sbm_bernoulli", p_in=0.008 / min(1.0, scale), p_out=0.0005 / min(1.0, scale)),
                      history_init="zeros")
    if i == 1:
        return Config("mid-gcn3", "gcn", sc(200_000, 40), 40, 10, [128, 256, 256, 256], torch.float32,
                      dict(kind="sbm_partners", mean_degree=10.0, frac_intra=0.85))
    if i == 2:
        return Config("large-gcn3", "gcn", sc(2_400_000, 64), 64, 16, [100, 256, 256, 256], torch.float32,
                      dict(kind="chung_lu", exponent=2.1, mean_degree=50.0,
                           max_degree=max(64, int(20_000 * min(1.0, scale * 4)))))
    if i == 3:
        return Config("deep-gcnii64", "gcnii", sc(170_000, 32), 32, 4, [128] + [64] * 65, torch.float32,
                      dict(kind="sbm_partners", mean_degree=14.0, frac_intra=0.85), alpha=0.1)
    if i == 4:
        return Config("huge-gin3", "gin", sc(50_000_000, 512), 512, 32, [128, 256, 256, 256], torch.bfloat16,
                      dict(kind="chung_lu", exponent=2.2, mean_degree=30.0,
                           max_degree=max(64, int(20_000 * min(1.0, scale * 16)))),
                      gin_hidden=256, self_loops=False)
    raise ValueError(f"no config {i}")


def gcnii_beta(layer: int) -> float:
    """Identity-mapping strength of propagation layer `layer` (1-indexed), as
    the benchmark configuration states it: log(0.5/l + 1)."""
    return math.log(0.5 / layer + 1.0)


def build_graph(cfg: Config, device="cpu") -> graphs.Graph:
    g = dict(cfg.graph)
    kind = g.pop("kind")
    if kind == "sbm_bernoulli":
        return graphs.sbm_bernoulli(cfg.n, cfg.n_blocks, seed=cfg.seed, device=device, **g)
    if kind == "sbm_partners":
        return graphs.sbm_partners(cfg.n, cfg.n_blocks, seed=cfg.seed, device=device, **g)
    if kind == "chung_lu":
        return graphs.chung_lu_bfs_blocks(cfg.n, n_blocks=cfg.n_blocks, seed=cfg.seed, device=device, **g)
    raise ValueError(kind)


@dataclass
class Workload:
    cfg: Config
    graph: graphs.Graph
    batches: list                 # list of int64 id tensors
    x: torch.Tensor               # [n, F_0] features in cfg.dtype
    weights: list                 # per layer: W [F_in, F_out] (gcn/gcnii) or (W1, W2) (gin), cfg.dtype
    w_in: torch.Tensor = None     # GCNII input projection [F_0, F_1]
    extras: dict = field(default_factory=dict)


def build_workload(cfg: Config, device="cpu") -> Workload:
    g = build_graph(cfg, device)
    bl = batches.split(g, cfg.blocks_per_batch, cfg.seed)
    x = rng.normal_matrix(cfg.seed, 10, cfg.n, cfg.widths[0], device, cfg.dtype)
    ws, w_in = [], None
    if cfg.op == "gcnii":
        # widths = [F_0, 64, 64, ...]: one graph-agnostic input projection, then
        # n_layers-1 propagation layers of equal width
        w_in = rng.glorot_uniform(cfg.seed, 100, cfg.widths[0], cfg.widths[1], device, cfg.dtype)
        for l in range(1, cfg.n_layers):
            ws.append(rng.glorot_uniform(cfg.seed, 100 + l, cfg.widths[l], cfg.widths[l + 1], device, cfg.dtype))
    elif cfg.op == "gin":
        for l in range(cfg.n_layers):
            w1 = rng.glorot_uniform(cfg.seed, 100 + 2 * l, cfg.widths[l], cfg.gin_hidden, device, cfg.dtype)
            w2 = rng.glorot_uniform(cfg.seed, 101 + 2 * l, cfg.gin_hidden, cfg.widths[l + 1], device, cfg.dtype)
            ws.append((w1, w2))
    else:
        for l in range(cfg.n_layers):
            ws.append(rng.glorot_uniform(cfg.seed, 100 + l, cfg.widths[l], cfg.widths[l + 1], device, cfg.dtype))
    return Workload(cfg, g, bl, x, ws, w_in)


def n_histories(cfg: Config) -> int:
    """One table per non-final message-passing layer (Algorithm 1's inner loop
    runs over layers 1..L-1)."""
    n_mp = cfg.n_layers - 1 if cfg.op == "gcnii" else cfg.n_layers
    return n_mp - 1


def history_width(cfg: Config, l: int) -> int:
    """Width of the table that stores the output of message-passing layer l+1."""
    return cfg.widths[l + 2] if cfg.op == "gcnii" else cfg.widths[l + 1]


def make_histories(cfg: Config, device="cpu", init=None):
    """Per-layer history tables [n, F] in cfg.dtype: zeros, or seeded N(0,1)
    as if pushed by earlier iterations."""
    init = init or cfg.history_init
    out = []
    for l in range(n_histories(cfg)):
        f = history_width(cfg, l)
        if init == "zeros":
            out.append(torch.zeros((cfg.n, f), dtype=cfg.dtype, device=device))
        else:
            out.append(rng.normal_matrix(cfg.seed, 200 + l, cfg.n, f, device, cfg.dtype))
    return out


def block_labels(g: graphs.Graph, n_classes: int, seed: int, unlabelled: float = 0.0, device="cpu") -> torch.Tensor:
    """Synthetic node-classification target: the class of a node is its locality block modulo n_classes
    (communities are what a message-passing model can read off the structure); a seeded fraction of the
    nodes is left unlabelled (-1), as in the semi-supervised splits of the paper's datasets.  int32 [n]."""
    bp = g.block_ptr.to(torch.int64)
    node = torch.arange(g.n, dtype=torch.int64)
    block = torch.searchsorted(bp, node, right=True) - 1
    lab = (block % n_classes).to(torch.int32)
    if unlabelled > 0.0:
        u = rng.uniform01(seed, 900, node)
        lab = torch.where(u < unlabelled, torch.full_like(lab, -1), lab)
    return lab.to(device)


def class_features(g: graphs.Graph, n_classes: int, width: int, seed: int, signal: float = 1.0, device="cpu",
                   dtype=torch.float32) -> torch.Tensor:
    """Input features that carry the class weakly: seeded N(0,1) noise plus `signal` times a seeded N(0,1)
    prototype row of the node's class (the class of block_labels with no node left out).  [n, width]."""
    lab = block_labels(g, n_classes, seed).to(torch.int64)
    proto = rng.normal_matrix(seed, 901, n_classes, width, "cpu", torch.float32)
    x = rng.normal_matrix(seed, 902, g.n, width, "cpu", torch.float32) + signal * proto[lab]
    return x.to(dtype).to(device)
