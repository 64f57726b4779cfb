"""Seeded synthetic graphs shaped like the paper's workloads.

Stochastic block models stand in for the small and mid-size citation-style
graphs of the paper's dataset table, capped Chung-Lu power-law graphs for its
large product/co-purchase graphs.  Graphs are simple and undirected: a
symmetric 0/1 adjacency without self-loops or multi-edges (the adjacency
matrix of the paper's Section 2 background), stored as CSR with sorted rows.

Everything here is structure.  None of the method's arithmetic (normalisation
coefficients, aggregation, transforms) lives in this module.
"""
from dataclasses import dataclass
import math

import torch

from . import rng


@dataclass
class Graph:
    n: int                    # |V|
    rowptr: torch.Tensor      # int64 [n+1]
    col: torch.Tensor         # int32 [nnz], each row ascending
    deg: torch.Tensor         # int32 [n], |N(v)| on the full graph
    block_ptr: torch.Tensor   # int64 [n_blocks+1] (CPU), blocks are contiguous id ranges

    @property
    def nnz(self) -> int:
        return int(self.col.numel())

    @property
    def n_blocks(self) -> int:
        return int(self.block_ptr.numel()) - 1

    def to(self, device):
        return Graph(self.n, self.rowptr.to(device), self.col.to(device),
                     self.deg.to(device), self.block_ptr)


def equal_block_ptr(n: int, n_blocks: int) -> torch.Tensor:
    """Contiguous blocks; the first n % n_blocks blocks get one extra node."""
    base, extra = divmod(n, n_blocks)
    sizes = torch.full((n_blocks,), base, dtype=torch.int64)
    sizes[:extra] += 1
    ptr = torch.zeros(n_blocks + 1, dtype=torch.int64)
    ptr[1:] = torch.cumsum(sizes, 0)
    return ptr


def _csr_from_unordered_pairs(n: int, key_u: torch.Tensor, block_ptr: torch.Tensor) -> Graph:
    """key_u: unique int64 keys lo*n+hi with lo < hi."""
    lo = key_u // n
    hi = key_u - lo * n
    key = torch.cat([key_u, hi * n + lo])
    del lo, hi
    key = torch.sort(key).values
    row = key // n
    col = (key - row * n).to(torch.int32)
    counts = torch.bincount(row, minlength=n)
    del row, key
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=col.device)
    rowptr[1:] = torch.cumsum(counts, 0)
    return Graph(n, rowptr, col, counts.to(torch.int32), block_ptr)


def _dedup_pairs(n: int, a: torch.Tensor, b: torch.Tensor) -> torch.Tensor:
    keep = a != b
    a, b = a[keep], b[keep]
    lo = torch.minimum(a, b)
    hi = torch.maximum(a, b)
    return torch.unique(lo * n + hi)


def sbm_bernoulli(n: int, n_blocks: int, p_in: float, p_out: float, seed: int,
                  device="cpu") -> Graph:
    """Every unordered pair is an edge with probability p_in (same block) or
    p_out (different blocks).  Quadratic in n: small graphs only."""
    block_ptr = equal_block_ptr(n, n_blocks)
    block_of = torch.repeat_interleave(torch.arange(n_blocks), block_ptr[1:] - block_ptr[:-1]).to(device)
    i, j = torch.triu_indices(n, n, offset=1, device=device)
    u = rng.uniform01(seed, 1, i * n + j)
    p = torch.where(block_of[i] == block_of[j], p_in, p_out)
    keep = u < p
    return _csr_from_unordered_pairs(n, (i[keep] * n + j[keep]), block_ptr)


def _poisson(seed: int, stream: int, idx: torch.Tensor, lam: float) -> torch.Tensor:
    """Poisson(lam) by inverse CDF (lam small)."""
    u = rng.uniform01(seed, stream, idx)
    k_max = int(lam + 12.0 * math.sqrt(lam + 1.0) + 12)
    out = torch.zeros_like(idx)
    p = math.exp(-lam)
    cdf = p
    for k in range(1, k_max + 1):
        out += (u >= cdf).to(out.dtype)
        p *= lam / k
        cdf += p
    return out


def sbm_partners(n: int, n_blocks: int, mean_degree: float, frac_intra: float, seed: int,
                 device="cpu") -> Graph:
    """Sparse block model for large n: every node draws Poisson(mean*frac/2)
    partners uniformly inside its block and Poisson(mean*(1-frac)/2) uniformly
    outside it; the union is symmetrised and deduplicated."""
    block_ptr = equal_block_ptr(n, n_blocks)
    sizes = (block_ptr[1:] - block_ptr[:-1])
    node = torch.arange(n, dtype=torch.int64, device=device)
    block_of = torch.repeat_interleave(torch.arange(n_blocks), sizes).to(device)
    bstart = block_ptr[:-1].to(device)[block_of]
    bsize = sizes.to(device)[block_of]
    k_in = _poisson(seed, 2, node, mean_degree * frac_intra / 2.0)
    k_out = _poisson(seed, 3, node, mean_degree * (1.0 - frac_intra) / 2.0)
    pairs = []
    for stream, cnt, intra in ((4, k_in, True), (5, k_out, False)):
        src = torch.repeat_interleave(node, cnt)
        first = torch.cumsum(cnt, 0) - cnt
        slot = torch.arange(src.numel(), dtype=torch.int64, device=device) - first[src]
        draw_idx = src * 64 + slot          # at most 64 draws per node and kind
        if intra:
            dst = bstart[src] + rng.randint(seed, stream, draw_idx, bsize[src])
        else:
            r = rng.randint(seed, stream, draw_idx, n - bsize[src])
            dst = torch.where(r >= bstart[src], r + bsize[src], r)
        pairs.append((src, dst))
    a = torch.cat([p[0] for p in pairs])
    b = torch.cat([p[1] for p in pairs])
    return _csr_from_unordered_pairs(n, _dedup_pairs(n, a, b), block_ptr)


def chung_lu_weights(n: int, exponent: float, mean_degree: float, max_degree: float) -> torch.Tensor:
    """Expected degrees w_i = min(cap, c * (i+1)^(-1/(exponent-1))), with c
    chosen by bisection so that the mean is `mean_degree` (float64, CPU)."""
    base = torch.arange(1, n + 1, dtype=torch.float64).pow(-1.0 / (exponent - 1.0))
    lo, hi = 0.0, float(max_degree) * float(n)
    for _ in range(200):
        c = 0.5 * (lo + hi)
        m = torch.clamp(base * c, max=max_degree).mean().item()
        if m < mean_degree:
            lo = c
        else:
            hi = c
    return torch.clamp(base * (0.5 * (lo + hi)), max=max_degree)


def chung_lu(n: int, exponent: float, mean_degree: float, max_degree: int, seed: int,
             device="cpu", chunk: int = 1 << 25) -> Graph:
    """Draw round(sum(w)/2) undirected edges with both endpoints chosen with
    probability proportional to w, then drop self-loops and duplicates.  The
    sampling is all-integer (weights scaled by 2^20) so CPU and GPU agree."""
    w = chung_lu_weights(n, exponent, mean_degree, max_degree)
    m_draws = int(round(w.sum().item() / 2.0))
    wi = torch.clamp((w * float(1 << 20)).round().to(torch.int64), min=1)
    cdf = torch.cumsum(wi, 0).to(device)
    total = int(cdf[-1].item())
    keys = []
    for s in range(0, m_draws, chunk):
        e = min(m_draws, s + chunk)
        idx = torch.arange(s, e, dtype=torch.int64, device=device)
        a = torch.searchsorted(cdf, rng.randint(seed, 6, idx, total), right=True)
        b = torch.searchsorted(cdf, rng.randint(seed, 7, idx, total), right=True)
        keys.append(_dedup_pairs(n, a, b))
        del a, b, idx
    key_u = torch.unique(torch.cat(keys)) if len(keys) > 1 else keys[0]
    del keys
    return _csr_from_unordered_pairs(n, key_u, equal_block_ptr(n, 1))


def bfs_order(g: Graph, seed: int) -> torch.Tensor:
    """Queue-order breadth-first numbering: start at a seeded node, visit each
    node's unvisited neighbours in ascending id, restart from the lowest
    unvisited id when a component is exhausted.  Returns `order` with
    order[new_id] = old_id.  Level-synchronous and vectorised; the result is
    the same as a sequential FIFO traversal."""
    n, dev = g.n, g.col.device
    visited = torch.zeros(n, dtype=torch.bool, device=dev)
    start = int(rng.randint(seed, 8, torch.zeros(1, dtype=torch.int64), n).item())
    out = []
    n_done = 0
    frontier = torch.tensor([start], dtype=torch.int64, device=dev)
    visited[start] = True
    big = torch.iinfo(torch.int64).max
    while True:
        out.append(frontier)
        n_done += frontier.numel()
        cnt = g.rowptr[frontier + 1] - g.rowptr[frontier]
        total = int(cnt.sum().item())
        nxt = None
        if total > 0:
            rank = torch.repeat_interleave(torch.arange(frontier.numel(), device=dev), cnt)
            first = torch.cumsum(cnt, 0) - cnt
            off = torch.arange(total, dtype=torch.int64, device=dev) - first[rank]
            child = g.col[g.rowptr[frontier][rank] + off].to(torch.int64)
            keep = ~visited[child]
            child, rank = child[keep], rank[keep]
            if child.numel() > 0:
                key = rank * n + child                    # discovery order: parent rank, then id
                best = torch.full((n,), big, dtype=torch.int64, device=dev)
                best.scatter_reduce_(0, child, key, reduce="amin")
                first_seen = key == best[child]
                nxt = torch.sort(key[first_seen]).values % n
                del best
        if nxt is None or nxt.numel() == 0:
            if n_done == n:
                break
            rest = torch.nonzero(~visited)[:1, 0]
            nxt = rest
        visited[nxt] = True
        frontier = nxt
    return torch.cat(out)


def relabel(g: Graph, order: torch.Tensor, block_ptr: torch.Tensor) -> Graph:
    """Renumber nodes so that new id i is old node order[i]."""
    n, dev = g.n, g.col.device
    new_of_old = torch.empty(n, dtype=torch.int64, device=dev)
    new_of_old[order] = torch.arange(n, dtype=torch.int64, device=dev)
    row_old = torch.repeat_interleave(torch.arange(n, dtype=torch.int64, device=dev),
                                      g.rowptr[1:] - g.rowptr[:-1])
    key = new_of_old[row_old] * n + new_of_old[g.col.to(torch.int64)]
    del row_old
    key = torch.sort(key).values
    row = key // n
    col = (key - row * n).to(torch.int32)
    counts = torch.bincount(row, minlength=n)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(counts, 0)
    return Graph(n, rowptr, col, counts.to(torch.int32), block_ptr)


def chung_lu_bfs_blocks(n: int, exponent: float, mean_degree: float, max_degree: int,
                        n_blocks: int, seed: int, device="cpu") -> Graph:
    g = chung_lu(n, exponent, mean_degree, max_degree, seed, device)
    order = bfs_order(g, seed)
    return relabel(g, order, equal_block_ptr(n, n_blocks))


def batch_with_outside_links(n_batch: int, n_outside: int, links: int, seed: int, device="cpu") -> Graph:
    """The paper's synthetic overhead workload (Section 6 "Experiments", runtime analysis): a mini-batch of `n_batch` nodes,
    each randomly linked to `links` other nodes of the batch, plus `n_outside` out-of-batch nodes each randomly
    linked to `links` nodes inside the batch.  Nodes 0..n_batch-1 are the batch (block 0), the rest block 1.
    "Linked to 60 other nodes" is read as an average degree of 60 inside the batch: every node draws links/2
    partners and the union is symmetrised; an outside node draws `links` distinct-or-not partners, deduplicated."""
    node = torch.arange(n_batch, dtype=torch.int64, device=device)
    half = max(1, links // 2)
    src = node.repeat_interleave(half)
    slot = torch.arange(src.numel(), dtype=torch.int64, device=device)
    dst = rng.randint(seed, 20, slot, n_batch - 1)
    dst = torch.where(dst >= src, dst + 1, dst)                     # anyone but oneself
    n = n_batch + n_outside
    pairs_a, pairs_b = [src], [dst]
    if n_outside > 0:
        out = n_batch + torch.arange(n_outside, dtype=torch.int64, device=device)
        osrc = out.repeat_interleave(links)
        oslot = torch.arange(osrc.numel(), dtype=torch.int64, device=device)
        pairs_a.append(osrc)
        pairs_b.append(rng.randint(seed, 21, oslot, n_batch))
    a, b = torch.cat(pairs_a), torch.cat(pairs_b)
    block_ptr = torch.tensor([0, n_batch, n], dtype=torch.int64)
    return _csr_from_unordered_pairs(n, _dedup_pairs(n, a, b), block_ptr)
