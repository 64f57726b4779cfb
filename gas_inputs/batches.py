"""Mini-batch selection and batch-subgraph index structures.

`split` is the paper's Split(G, B) step of Algorithm 1 with the clustering
replaced by the synthetic block structure: a seeded permutation of the blocks
is cut into consecutive groups.  `batch_subgraph` builds, for one batch, the
node list V_b = B ++ halo (the `n_id` assignment vector of the paper's
programming-interface appendix) and the sparsity pattern of the rows of G_b
that belong to in-batch nodes, as CSR and as a CSC copy.

Only index structure is built here.  Edge values (normalisation) are computed
separately by the library under test and by the oracle.
"""
from dataclasses import dataclass

import torch

from . import rng
from .graphs import Graph


def split(g: Graph, blocks_per_batch: int, seed: int):
    """List of int64 node-id tensors (ascending), one per batch."""
    perm = rng.permutation(seed, 9, g.n_blocks)
    batches = []
    for s in range(0, g.n_blocks, blocks_per_batch):
        ids = perm[s:s + blocks_per_batch]
        parts = [torch.arange(int(g.block_ptr[b]), int(g.block_ptr[b + 1]), dtype=torch.int64)
                 for b in sorted(ids.tolist())]
        batches.append(torch.cat(parts))
    return batches


@dataclass
class BatchSubgraph:
    nb: int                  # |B|
    nh: int                  # |V_b \ B|
    n_id: torch.Tensor       # int32 [nb+nh] global ids: batch ascending, then halo ascending
    rowptr: torch.Tensor     # int32 [nb+1]
    col: torch.Tensor        # int32 [nnz] local ids < nb+nh, each row ascending
    colptr: torch.Tensor     # int32 [nb+nh+1]   CSC copy of the same pattern
    row: torch.Tensor        # int32 [nnz] local row ids < nb, each column ascending
    csc_perm: torch.Tensor   # int32 [nnz] CSC entry k is CSR entry csc_perm[k]

    @property
    def nv(self) -> int:
        return self.nb + self.nh

    @property
    def nnz(self) -> int:
        return int(self.col.numel())

    def to(self, device):
        return BatchSubgraph(self.nb, self.nh, *[t.to(device) for t in (
            self.n_id, self.rowptr, self.col, self.colptr, self.row, self.csc_perm)])


def batch_subgraph(g: Graph, batch: torch.Tensor, self_loops: bool) -> BatchSubgraph:
    """Rows = in-batch nodes, columns = in-batch nodes followed by the 1-hop
    halo.  With `self_loops` every row also holds its own diagonal entry."""
    dev = g.col.device
    batch = batch.to(dev)
    nb = int(batch.numel())
    cnt = g.rowptr[batch + 1] - g.rowptr[batch]
    total = int(cnt.sum().item())
    lrow = torch.repeat_interleave(torch.arange(nb, dtype=torch.int64, device=dev), cnt)
    first = torch.cumsum(cnt, 0) - cnt
    off = torch.arange(total, dtype=torch.int64, device=dev) - first[lrow]
    gcol = g.col[g.rowptr[batch][lrow] + off].to(torch.int64)
    del off
    local = torch.full((g.n,), -1, dtype=torch.int64, device=dev)
    local[batch] = torch.arange(nb, dtype=torch.int64, device=dev)
    outside = local[gcol] < 0
    halo = torch.unique(gcol[outside])
    nh = int(halo.numel())
    local[halo] = nb + torch.arange(nh, dtype=torch.int64, device=dev)
    lcol = local[gcol]
    del gcol, local, outside
    if self_loops:
        diag = torch.arange(nb, dtype=torch.int64, device=dev)
        lrow = torch.cat([lrow, diag])
        lcol = torch.cat([lcol, diag])
    nv = nb + nh
    key = torch.sort(lrow * nv + lcol).values
    r = key // nv
    c = key - r * nv
    rowptr = torch.zeros(nb + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(torch.bincount(r, minlength=nb), 0)
    # CSC copy: sort the same entries by (column, row)
    tkey, perm = torch.sort(c * nb + r)
    colptr = torch.zeros(nv + 1, dtype=torch.int64, device=dev)
    colptr[1:] = torch.cumsum(torch.bincount(c, minlength=nv), 0)
    trow = tkey - (tkey // nb) * nb
    i32 = torch.int32
    return BatchSubgraph(nb, nh, torch.cat([batch, halo]).to(i32), rowptr.to(i32), c.to(i32),
                         colptr.to(i32), trow.to(i32), perm.to(i32))
