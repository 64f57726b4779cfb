"""Oracle for the GAS mini-batch execution (test infrastructure).

`gas_batch_forward` walks one mini-batch through all layers in the order of
the paper's Algorithm 1: compute layer l for the in-batch nodes from the
current mini-batch tensor, push the result to history l, pull the halo rows
from history l, go on to layer l+1; the last layer is computed and not pushed.
The out-of-batch neighbours therefore enter layer l+1 through their stored
historical embeddings, which is the approximation of the paper's Eq. (2).

`full_batch_forward` is the exact model of Eq. (1) on the whole graph in
float64 (scipy sparse product), without any storage rounding; it is what the
invariants in the tests pin the mini-batch executor to.  `dense_adjacency`
writes the aggregation matrix out densely for brute-force checks on tiny
graphs.

Operators (paper, operator appendix): GCN, GCNII (initial residual alpha,
identity map beta_l) and GIN (sum aggregation, (1+eps) self term, 2-layer MLP).
ReLU follows every layer but the last, and the value pushed is the activated
one, as in the paper's interface listing where the activation precedes
push_and_pull.
"""
from dataclasses import dataclass, field
import math

import numpy as np
import scipy.sparse as sp

from . import ops


@dataclass
class Model:
    op: str                      # "gcn" | "gcnii" | "gin"
    weights: list                # per message-passing layer: W, or (W1, W2) for gin
    w_in: np.ndarray = None      # gcnii: graph-agnostic input projection
    alpha: float = 0.0           # gcnii
    gin_eps: float = 0.0
    betas: list = field(default_factory=list)   # gcnii: beta_l per layer

    @property
    def n_layers(self) -> int:
        return len(self.weights)


def gcnii_betas(n_layers: int):
    return [math.log(0.5 / l + 1.0) for l in range(1, n_layers + 1)]


# ----------------------------------------------------------------------------
# batch subgraph, written out plainly from Algorithm 1 (V_b and the rows of G_b)
# ----------------------------------------------------------------------------
def batch_subgraph(rowptr, col, batch, self_loops):
    """n_id = batch ++ sorted halo; CSR with one row per in-batch node whose
    columns are local ids of N(v) (and v itself with self_loops), ascending."""
    batch = [int(v) for v in batch]
    in_batch = {v: i for i, v in enumerate(batch)}
    halo = set()
    for v in batch:
        for k in range(rowptr[v], rowptr[v + 1]):
            w = int(col[k])
            if w not in in_batch:
                halo.add(w)
    halo = sorted(halo)
    local = dict(in_batch)
    for i, w in enumerate(halo):
        local[w] = len(batch) + i
    lptr, lcol = [0], []
    for v in batch:
        cols = [local[int(col[k])] for k in range(rowptr[v], rowptr[v + 1])]
        if self_loops:
            cols.append(local[v])
        lcol.extend(sorted(cols))
        lptr.append(len(lcol))
    n_id = np.array(batch + halo, dtype=np.int32)
    return n_id, np.array(lptr, dtype=np.int32), np.array(lcol, dtype=np.int32)


# ----------------------------------------------------------------------------
# one mini-batch, all layers (Algorithm 1, inner loop)
# ----------------------------------------------------------------------------
def gas_batch_forward(model: Model, n_id, rowptr, col, nb, deg, x_feat, histories,
                      do_push=True, return_layers=False):
    """x_feat: [N, F_0] feature table; histories: list of [N, F] tables, updated
    in place.  Returns the last layer's output for the in-batch nodes (and,
    if asked, the mini-batch tensor after every layer)."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    nv = n_id.size
    val = ops.gcn_norm(rowptr, col, n_id, deg) if model.op in ("gcn", "gcnii") else None
    x = ops.pull(x_feat, n_id)                       # layer-0 embeddings are the exact features
    h0 = None
    if model.op == "gcnii":
        h0 = ops.linear(x, model.w_in, relu=True)    # graph-agnostic, exact for halo rows too
        x = h0
    L = model.n_layers
    layers = []
    for l in range(1, L + 1):
        last = l == L
        if model.op == "gcn":
            z = ops.spmm(rowptr, col, val, x)
            y = ops.linear(z, model.weights[l - 1], relu=not last)
        elif model.op == "gin":
            z = ops.spmm(rowptr, col, None, x, diag=1.0 + model.gin_eps)
            w1, w2 = model.weights[l - 1]
            y = ops.mlp2(z, w1, w2, relu_out=not last)
        elif model.op == "gcnii":
            z = ops.spmm(rowptr, col, val, x, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
            b = model.betas[l - 1]
            y = ops.linear(z, model.weights[l - 1], c_identity=1.0 - b, c_weight=b, relu=not last)
        else:
            raise ValueError(model.op)
        if last:
            layers.append(y)
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        x = np.empty((nv, y.shape[1]), dtype=y.dtype)
        x[:nb] = y
        x[nb:] = ops.pull(histories[l - 1], n_id[nb:])
        layers.append(x)
    return (y, layers) if return_layers else y


# ----------------------------------------------------------------------------
# exact full-batch model, float64, no rounding (Eq. 1 on the whole graph)
# ----------------------------------------------------------------------------
def _adjacency(rowptr, col, n):
    return sp.csr_matrix((np.ones(len(col)), np.asarray(col, dtype=np.int64),
                          np.asarray(rowptr, dtype=np.int64)), shape=(n, n))


def full_batch_forward(model: Model, rowptr, col, x_feat):
    """List of per-layer embeddings h^(1..L) as float64 [N, F] (post-ReLU for
    all but the last layer)."""
    n = len(rowptr) - 1
    a = _adjacency(rowptr, col, n)
    deg = np.asarray(a.sum(axis=1)).ravel()
    f64 = ops.to_f64
    if model.op in ("gcn", "gcnii"):
        dinv = 1.0 / np.sqrt(deg + 1.0)
        a_hat = sp.diags(dinv) @ (a + sp.identity(n)) @ sp.diags(dinv)
    h = f64(x_feat)
    h0 = None
    if model.op == "gcnii":
        h0 = np.maximum(h @ f64(model.w_in), 0.0)
        h = h0
    out = []
    L = model.n_layers
    for l in range(1, L + 1):
        if model.op == "gcn":
            y = (a_hat @ h) @ f64(model.weights[l - 1])
        elif model.op == "gin":
            w1, w2 = model.weights[l - 1]
            z = (1.0 + model.gin_eps) * h + a @ h
            y = np.maximum(z @ f64(w1), 0.0) @ f64(w2)
        else:
            z = (1.0 - model.alpha) * (a_hat @ h) + model.alpha * h0
            b = model.betas[l - 1]
            y = (1.0 - b) * z + b * (z @ f64(model.weights[l - 1]))
        if l < L:
            y = np.maximum(y, 0.0)
        out.append(y)
        h = y
    return out


def dense_adjacency(n_id, rowptr, col, val, nb):
    """The nb x nv aggregation matrix of a batch subgraph, written out densely."""
    nv = len(n_id)
    a = np.zeros((nb, nv), dtype=np.float64)
    for v in range(nb):
        for k in range(rowptr[v], rowptr[v + 1]):
            a[v, col[k]] += 1.0 if val is None else float(val[k])
    return a
