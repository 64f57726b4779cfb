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


# ----------------------------------------------------------------------------
# one mini-batch forward + backward (training step without the optimiser)
# ----------------------------------------------------------------------------
def gas_batch_forward_kept(model: Model, n_id, rowptr, col, nb, deg, x_feat, histories, do_push=True):
    """Forward as gas_batch_forward (GIN's MLP as two stored linears) with every activation the backward
    pass reads kept.  Returns (Y_L, kept) with kept = (val, x0, h0, saved), saved[l] = (Z, hidden or None, Y)."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    nv = n_id.size
    val = ops.gcn_norm(rowptr, col, n_id, deg) if model.op in ("gcn", "gcnii") else None
    x0 = ops.pull(x_feat, n_id)
    x = x0
    h0 = None
    if model.op == "gcnii":
        h0 = ops.linear(x0, model.w_in, relu=True)
        x = h0
    L = model.n_layers
    saved = []
    y = None
    for l in range(1, L + 1):
        last = l == L
        if model.op == "gcn":
            z = ops.spmm(rowptr, col, val, x)
            y = ops.linear(z, model.weights[l - 1], relu=not last)
            saved.append((z, None, y))
        elif model.op == "gin":
            z = ops.spmm(rowptr, col, None, x, diag=1.0 + model.gin_eps)
            w1, w2 = model.weights[l - 1]
            h = ops.linear(z, w1, relu=True)
            y = ops.linear(h, w2, relu=not last)
            saved.append((z, h, y))
        else:
            z = ops.spmm(rowptr, col, val, x, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
            b = model.betas[l - 1]
            y = ops.linear(z, model.weights[l - 1], c_identity=1.0 - b, c_weight=b, relu=not last)
            saved.append((z, None, y))
        if last:
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        xn = np.empty((nv, y.shape[1]), dtype=y.dtype)
        xn[:nb] = y
        xn[nb:] = ops.pull(histories[l - 1], n_id[nb:])
        x = xn
    return y, (val, x0, h0, saved)


def gas_batch_train(model: Model, n_id, rowptr, col, nb, deg, x_feat, histories, grad_out, do_push=True):
    """Forward with kept activations, then the chain rule backwards.

    Historical embeddings are constants: gradients flow through in-batch rows only, layer by layer
    (the pulled halo rows of layers >= 2 receive none).  GCNII's input projection is computed in-graph for
    halo rows too, so its weight gradient includes them.  `grad_out` is dLoss/dY_L [nb, F_L] in the storage
    dtype.  Returns (Y_L, grads) with grads[l] = dW_l (or (dW1, dW2) for GIN) as float32, and grads["w_in"]
    for GCNII."""
    y, (val, x0, h0, saved) = gas_batch_forward_kept(model, n_id, rowptr, col, nb, deg, x_feat, histories, do_push)
    return y, gas_batch_backward(model, n_id, rowptr, col, nb, val, x0, h0, saved, grad_out)


def _all_grads(model: Model, grads):
    """(weight, gradient) pairs in a fixed order: layer by layer (GIN: W1 then W2), GCNII's projection last."""
    out = []
    for l in range(model.n_layers):
        if model.op == "gin":
            out += list(zip(model.weights[l], grads[l]))
        else:
            out.append((model.weights[l], grads[l]))
    if model.op == "gcnii":
        out.append((model.w_in, grads["w_in"]))
    return out


def apply_sgd(model: Model, grads, lr, weight_decay=0.0, max_norm=None):
    """One gradient-descent update of every weight matrix, in place; with max_norm the gradients are first
    clipped by their global L2 norm (paper, Section 3)."""
    pairs = _all_grads(model, grads)
    scale = 1.0 if max_norm is None else ops.clip_scale([ops.sq_norm(dw) for _, dw in pairs], max_norm)
    for w, dw in pairs:
        if scale != 1.0:
            dw = (dw.astype(np.float64) * scale).astype(np.float32)
        ops.sgd_step(w, np.ascontiguousarray(dw), lr, weight_decay)


def layer_input(model: Model, l, n_id, nb, x0, h0, saved, histories):
    """The mini-batch tensor layer l read in a forward pass whose activations were kept: the features (GCNII: the
    projected features) for l = 1, else layer l-1's output for the in-batch rows and the halo rows as they stand in
    history table l-1 (this batch's pushes do not touch halo rows, so they are what the layer pulled)."""
    if l == 1:
        return h0 if model.op == "gcnii" else x0
    y = saved[l - 2][2]
    x = np.empty((n_id.size, y.shape[1]), dtype=y.dtype)
    x[:nb] = y
    x[nb:] = ops.pull(histories[l - 2], n_id[nb:])
    return x


def gas_train_step(model: Model, n_id, rowptr, col, nb, deg, x_feat, histories, labels, lr, weight_decay=0.0,
                   max_norm=None, reg_weight=0.0, reg_eps=None):
    """One optimisation step of Algorithm 1's loop body on one mini-batch: forward with Push/Pull per layer,
    softmax cross-entropy averaged over the labelled in-batch nodes (labels: one per node of the graph, < 0 =
    unlabelled), backward with the histories held constant, gradient-descent update.  The model's weights and
    the histories are updated in place.  reg_weight: the local Lipschitz regulariser of Eq. (3) is added for every
    layer, differentiated with respect to that layer's weights.  Returns the mean loss (without the regulariser)
    before the update."""
    y, (val, x0, h0, saved) = gas_batch_forward_kept(model, n_id, rowptr, col, nb, deg, x_feat, histories)
    lab = np.ascontiguousarray(np.asarray(labels)[np.asarray(n_id[:nb], dtype=np.int64)], dtype=np.int32)
    n_lab = int((lab >= 0).sum())
    _, loss_sum, g = ops.softmax_xent(y, lab, scale=1.0 / max(1, n_lab))
    grads = gas_batch_backward(model, n_id, rowptr, col, nb, val, x0, h0, saved, g)
    if reg_weight != 0.0:
        # loss + reg_weight * sum over the layers of Eq. (3); reg_eps[l-1] holds layer l's drawn perturbations
        n_id = np.ascontiguousarray(n_id, dtype=np.int32)
        for l in range(1, model.n_layers + 1):
            x = layer_input(model, l, n_id, nb, x0, h0, saved, histories)
            _, dw = lipschitz_reg_grad(model, l, x, reg_eps[l - 1], rowptr, col, val, nb, h0)
            if model.op == "gin":
                grads[l - 1] = tuple((a.astype(np.float64) + reg_weight * b).astype(np.float32)
                                     for a, b in zip(grads[l - 1], dw))
            else:
                grads[l - 1] = (grads[l - 1].astype(np.float64) + reg_weight * dw).astype(np.float32)
    apply_sgd(model, grads, lr, weight_decay, max_norm)
    return loss_sum / max(1, n_lab)


def gas_batch_backward(model: Model, n_id, rowptr, col, nb, val, x0, h0, saved, grad_out):
    """The chain rule backwards through the layers, from the activations a forward pass has kept:
    saved[l] = (Z, hidden or None, Y) of layer l+1, x0 = the pulled features, h0 = GCNII's initial embedding.
    The ReLU masks are read off these stored activations."""
    nv = len(n_id)
    L = model.n_layers
    grads = {}
    g = np.ascontiguousarray(grad_out)
    g_h0 = None           # GCNII: gradient w.r.t. the initial embedding, all nv rows, accumulated in float64
    for l in range(L, 0, -1):
        z, h, yl = saved[l - 1]
        if l != L:
            g = ops.relu_bwd(g, yl)
        if model.op == "gcn":
            grads[l - 1] = ops.linear_bwd_weight(z, g)
            gz = ops.linear_bwd_input(g, model.weights[l - 1])
        elif model.op == "gin":
            w1, w2 = model.weights[l - 1]
            dw2 = ops.linear_bwd_weight(h, g)
            gh = ops.linear_bwd_input(g, w2, mask=h)
            grads[l - 1] = (ops.linear_bwd_weight(z, gh), dw2)
            gz = ops.linear_bwd_input(gh, w1)
            # operator appendix, GIN: Z_v = (1 + eps) h_v + sum over N(v), eps trainable: dL/d eps = sum_v <GZ_v, h_v>
            x_in = x0 if l == 1 else saved[l - 2][2]
            grads.setdefault("eps", np.zeros(L, dtype=np.float64))[l - 1] = ops.row_dot(gz, x_in[:nb])[1]
        else:
            b = model.betas[l - 1]
            grads[l - 1] = ops.linear_bwd_weight(z, g, c_weight=b)
            gz = ops.linear_bwd_input(g, model.weights[l - 1], c_identity=1.0 - b, c_weight=b)
            if g_h0 is None:
                g_h0 = np.zeros((nv, gz.shape[1]), dtype=np.float64)
            g_h0[:nb] += model.alpha * ops.to_f64(gz)
        if l == 1:
            if model.op == "gcnii":
                # layer 1 aggregates h0 itself, for every column of the batch subgraph (halo rows included)
                gx = ops.spmm_t(rowptr, col, val, gz, nv, s_agg=1.0 - model.alpha)
                g_h0 += ops.to_f64(gx)
            break
        if model.op == "gin":
            g = ops.spmm_t(rowptr, col, None, gz, nb, diag=1.0 + model.gin_eps)
        elif model.op == "gcn":
            g = ops.spmm_t(rowptr, col, val, gz, nb)
        else:
            g = ops.spmm_t(rowptr, col, val, gz, nb, s_agg=1.0 - model.alpha)
    if model.op == "gcnii":
        gh0 = np.where(ops.to_f64(h0) > 0.0, g_h0, 0.0)
        grads["w_in"] = (ops.to_f64(x0).T @ gh0).astype(np.float32)
    return grads


# ----------------------------------------------------------------------------
# APPNP (paper, operator appendix): graph-agnostic prediction, then K propagation steps without weights
# ----------------------------------------------------------------------------
def appnp_batch_forward(w1, w2, alpha, n_steps, n_id, rowptr, col, nb, deg, x_feat, histories, do_push=True):
    """h^(0) = relu(x W1) W2 for every node of V_b (it depends on the node's own features only, so it is exact
    for halo rows too), then for l = 1..K:  h^(l)_v = alpha h^(0)_v + (1 - alpha) sum_w h^(l-1)_w / c_{w,v}
    over N(v) and v itself, with the GCN coefficients.  Steps 1..K-1 are pushed to histories[l-1] and their
    halo rows pulled back, as for any other operator of Algorithm 1.  Returns h^(K) of the in-batch nodes."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    nv = n_id.size
    val = ops.gcn_norm(rowptr, col, n_id, deg)
    h0 = ops.mlp2(ops.pull(x_feat, n_id), w1, w2, relu_out=False)
    x = h0
    y = None
    for l in range(1, n_steps + 1):
        y = ops.spmm(rowptr, col, val, x, s_agg=1.0 - alpha, r=h0, s_res=alpha)
        if l == n_steps:
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        x = np.empty((nv, y.shape[1]), dtype=y.dtype)
        x[:nb] = y
        x[nb:] = ops.pull(histories[l - 1], n_id[nb:])
    return y


def appnp_full_batch(w1, w2, alpha, n_steps, rowptr, col, x_feat):
    """The same model on the whole graph in float64 without storage rounding: list of h^(1..K)."""
    n = len(rowptr) - 1
    a = _adjacency(rowptr, col, n)
    deg = np.asarray(a.sum(axis=1)).ravel()
    dinv = 1.0 / np.sqrt(deg + 1.0)
    a_hat = sp.diags(dinv) @ (a + sp.identity(n)) @ sp.diags(dinv)
    f64 = ops.to_f64
    h0 = np.maximum(f64(x_feat) @ f64(w1), 0.0) @ f64(w2)
    h, out = h0, []
    for _ in range(n_steps):
        h = alpha * h0 + (1.0 - alpha) * (a_hat @ h)
        out.append(h)
    return out


# ----------------------------------------------------------------------------
# PNA (paper, operator appendix)
# ----------------------------------------------------------------------------
def pna_layer(x, nb, rowptr, col, w1, w2, delta, relu):
    """h'_v = W2 [h_v, (+)_w W1 [h_v, h_w]] for the in-batch rows.  W1 is [2F, F1] (rows 0..F-1 multiply the
    receiving node, rows F.. the neighbour), W2 is [F + 9 F1, F_out].  A message is W1a h_v + W1b h_w and its
    first part is the same for every neighbour, so it commutes with mean, min and max: the neighbour part is
    computed once per node of V_b, aggregated, and the receiving-node part added afterwards."""
    f = x.shape[1]
    w1a, w1b = np.ascontiguousarray(w1[:f]), np.ascontiguousarray(w1[f:])
    p = ops.linear(x, w1b)                          # every node of V_b as a neighbour
    q = ops.linear(np.ascontiguousarray(x[:nb]), w1a)
    a9 = ops.pna_aggregate(rowptr, col, p, delta, add=q)
    cat = np.concatenate([x[:nb], a9], axis=1)
    return ops.linear(cat, w2, relu=relu)


def pna_batch_forward(weights, delta, n_id, rowptr, col, nb, x_feat, histories, do_push=True):
    """All layers of a PNA model for one mini-batch in the order of Algorithm 1; weights[l] = (W1, W2)."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    nv = n_id.size
    x = ops.pull(x_feat, n_id)
    L = len(weights)
    y = None
    for l in range(1, L + 1):
        w1, w2 = weights[l - 1]
        y = pna_layer(x, nb, rowptr, col, w1, w2, delta, relu=l < L)
        if l == L:
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        x = np.empty((nv, y.shape[1]), dtype=y.dtype)
        x[:nb] = y
        x[nb:] = ops.pull(histories[l - 1], n_id[nb:])
    return y


# ----------------------------------------------------------------------------
# GAT (paper, operator appendix); several heads are independent copies of the operator on column blocks
# ----------------------------------------------------------------------------
def gat_batch_forward(weights, n_id, rowptr, col, nb, x_feat, histories, negative_slope=0.2, do_push=True, heads=1):
    """All layers of a GAT for one mini-batch in the order of Algorithm 1; weights[l] = (W, a_dst, a_src).
    rowptr/col: the batch subgraph WITH self-loops (the sums run over N(v) and v).  Per layer: P = X W for every
    node of V_b, attention-weighted aggregation for the in-batch rows, ReLU on all layers but the last.
    heads > 1 (the multi-head attention of the operator's source, which the paper's appendix states for one head):
    the columns of W, a_dst and a_src are `heads` equal blocks, each block an attention head of its own with its
    own coefficients alpha, and the layer's output is the heads side by side."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    nv = n_id.size
    x = ops.pull(x_feat, n_id)
    L = len(weights)
    y = None
    for l in range(1, L + 1):
        w, a_dst, a_src = weights[l - 1]
        p = ops.linear(x, w)
        fh = p.shape[1] // heads
        assert fh * heads == p.shape[1]
        y = np.concatenate([ops.gat_aggregate(rowptr, col, p[:, h * fh:(h + 1) * fh], a_dst[h * fh:(h + 1) * fh],
                                              a_src[h * fh:(h + 1) * fh], negative_slope, relu=l < L)
                            for h in range(heads)], axis=1)
        if l == L:
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        x = np.empty((nv, y.shape[1]), dtype=y.dtype)
        x[:nb] = y
        x[nb:] = ops.pull(histories[l - 1], n_id[nb:])
    return y


def _next_input(y, nb, n_id, history):
    x = np.empty((n_id.size, y.shape[1]), dtype=y.dtype)
    x[:nb] = y
    x[nb:] = ops.pull(history, n_id[nb:])
    return x


def pna_batch_forward_kept(weights, delta, n_id, rowptr, col, nb, x_feat, histories, do_push=True):
    """pna_batch_forward with what the backward pass reads kept: per layer (X, P, [X[:nb] | A9], Y)."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    x = ops.pull(x_feat, n_id)
    L = len(weights)
    kept = []
    y = None
    for l in range(1, L + 1):
        w1, w2 = weights[l - 1]
        f = x.shape[1]
        p = ops.linear(x, np.ascontiguousarray(w1[f:]))
        q = ops.linear(np.ascontiguousarray(x[:nb]), np.ascontiguousarray(w1[:f]))
        cat = np.concatenate([x[:nb], ops.pna_aggregate(rowptr, col, p, delta, add=q)], axis=1)
        y = ops.linear(cat, w2, relu=l < L)
        kept.append((x, p, cat, y))
        if l == L:
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        x = _next_input(y, nb, n_id, histories[l - 1])
    return y, kept


def pna_batch_backward(weights, delta, rowptr, col, nb, kept, grad_out):
    """The chain rule backwards through PNA layers from kept activations (operator appendix, PNA; histories are
    constants, so only in-batch rows pass gradient to the layer below).  A layer computed, for the mini-batch
    tensor X [nv, F]:  P = X W1b (every node as a neighbour),  Q = X[:nb] W1a (the receiving node's part),
    A9 = the nine scaled aggregations of P, each plus Q,  Y = act([X[:nb] | A9] W2).  P of a halo row depends on W1b
    although the row itself is a constant, so W1b's gradient sums over all nv rows.
    Returns grads[l] = (dW1 [2F, F1], dW2) as float32."""
    L = len(weights)
    grads = {}
    g = np.ascontiguousarray(grad_out)
    for l in range(L, 0, -1):
        w1, w2 = weights[l - 1]
        x, p, cat, yl = kept[l - 1]
        f, nv = x.shape[1], x.shape[0]
        w1a, w1b = np.ascontiguousarray(w1[:f]), np.ascontiguousarray(w1[f:])
        if l != L:
            g = ops.relu_bwd(g, yl)
        dw2 = ops.linear_bwd_weight(cat, g)
        gcat = ops.linear_bwd_input(g, w2)
        gp, gq = ops.pna_aggregate_bwd(rowptr, col, p, delta, np.ascontiguousarray(gcat[:, f:]), nv)
        xb = np.ascontiguousarray(x[:nb])
        grads[l - 1] = (np.concatenate([ops.linear_bwd_weight(xb, gq), ops.linear_bwd_weight(x, gp)], axis=0), dw2)
        if l == 1:
            break
        # dL/dX[:nb]: the copy of h_v in the concatenation, the neighbour part, the receiving-node part
        g = ops.axpy(np.ascontiguousarray(gcat[:, :f]), ops.linear_bwd_input(np.ascontiguousarray(gp[:nb]), w1b), 1.0)
        g = ops.axpy(g, ops.linear_bwd_input(gq, w1a), 1.0)
    return grads


def pna_batch_train(weights, delta, n_id, rowptr, col, nb, x_feat, histories, grad_out, do_push=True):
    """Forward with kept activations, then the backward pass: (Y_L, grads)."""
    y, kept = pna_batch_forward_kept(weights, delta, n_id, rowptr, col, nb, x_feat, histories, do_push)
    return y, pna_batch_backward(weights, delta, rowptr, col, nb, kept, grad_out)


def _head_blocks(width, heads):
    fh = width // heads
    assert fh * heads == width
    return [slice(h * fh, (h + 1) * fh) for h in range(heads)]


def gat_batch_forward_kept(weights, n_id, rowptr, col, nb, x_feat, histories, negative_slope=0.2, do_push=True, heads=1):
    """gat_batch_forward with what the backward pass reads kept: per layer (X, P, Y)."""
    n_id = np.ascontiguousarray(n_id, dtype=np.int32)
    x = ops.pull(x_feat, n_id)
    L = len(weights)
    kept = []
    y = None
    for l in range(1, L + 1):
        w, a_dst, a_src = weights[l - 1]
        p = ops.linear(x, w)
        y = np.concatenate([ops.gat_aggregate(rowptr, col, p[:, c], a_dst[c], a_src[c], negative_slope, relu=l < L)
                            for c in _head_blocks(p.shape[1], heads)], axis=1)
        kept.append((x, p, y))
        if l == L:
            break
        if do_push:
            ops.push(y, n_id[:nb], histories[l - 1])
        x = _next_input(y, nb, n_id, histories[l - 1])
    return y, kept


def gat_batch_backward(weights, rowptr, col, nb, kept, grad_out, negative_slope=0.2, heads=1):
    """The chain rule backwards through GAT layers from kept activations (operator appendix, GAT; histories are
    constants).  P = X W is computed for every node of V_b, so W's gradient sums over all nv rows of the gradient
    of P; only the in-batch rows pass gradient on to the layer below.
    Returns grads[l] = (dW, d a_dst, d a_src) as float32."""
    L = len(weights)
    grads = {}
    g = np.ascontiguousarray(grad_out)
    for l in range(L, 0, -1):
        w, a_dst, a_src = weights[l - 1]
        x, p, yl = kept[l - 1]
        nv = x.shape[0]
        if l != L:
            g = ops.relu_bwd(g, yl)
        parts = [ops.gat_aggregate_bwd(rowptr, col, np.ascontiguousarray(p[:, c]), a_dst[c], a_src[c],
                                       np.ascontiguousarray(g[:, c]), nv, negative_slope)
                 for c in _head_blocks(p.shape[1], heads)]
        gp = np.concatenate([t[0] for t in parts], axis=1)
        grads[l - 1] = (ops.linear_bwd_weight(x, gp), np.concatenate([t[1] for t in parts]),
                        np.concatenate([t[2] for t in parts]))
        if l == 1:
            break
        g = ops.linear_bwd_input(np.ascontiguousarray(gp[:nb]), w)
    return grads


def gat_batch_train(weights, n_id, rowptr, col, nb, x_feat, histories, grad_out, negative_slope=0.2, do_push=True,
                    heads=1):
    """Forward with kept activations, then the backward pass: (Y_L, grads)."""
    y, kept = gat_batch_forward_kept(weights, n_id, rowptr, col, nb, x_feat, histories, negative_slope, do_push, heads)
    return y, gat_batch_backward(weights, rowptr, col, nb, kept, grad_out, negative_slope, heads)


# ----------------------------------------------------------------------------
# local Lipschitz regulariser (paper, Eq. 3)
# ----------------------------------------------------------------------------
def layer_forward(model: Model, l, x, h0, rowptr, col, val, nb):
    """Layer l (1-based) of the model applied to a mini-batch tensor x [nv, F]: output for the in-batch rows."""
    last = l == model.n_layers
    if model.op == "gcn":
        return ops.linear(ops.spmm(rowptr, col, val, x), model.weights[l - 1], relu=not last)
    if model.op == "gin":
        w1, w2 = model.weights[l - 1]
        return ops.mlp2(ops.spmm(rowptr, col, None, x, diag=1.0 + model.gin_eps), w1, w2, relu_out=not last)
    if model.op == "gcnii":
        z = ops.spmm(rowptr, col, val, x, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
        b = model.betas[l - 1]
        return ops.linear(z, model.weights[l - 1], c_identity=1.0 - b, c_weight=b, relu=not last)
    raise ValueError(model.op)


def lipschitz_reg(model: Model, l, x, eps, rowptr, col, val, nb, h0=None):
    """Eq. (3) for layer l on one mini-batch: the mean over the in-batch nodes of || f(x)_v - f(x + eps)_v ||_2,
    where x is the mini-batch tensor the layer reads (in-batch rows and pulled halo rows alike are perturbed:
    the layer is a function of all of them) and eps holds one drawn perturbation per row."""
    y = layer_forward(model, l, x, h0, rowptr, col, val, nb)
    y2 = layer_forward(model, l, ops.axpy(x, eps, 1.0), h0, rowptr, col, val, nb)
    _, total = ops.row_distance(y, y2)
    return total / max(1, nb)


def lipschitz_reg_grad(model: Model, l, x, eps, rowptr, col, val, nb, h0=None):
    """Eq. (3) for layer l and its gradient with respect to that layer's weights, the layer's input held fixed:
    returns (loss, dW) with loss as in lipschitz_reg and dW of the layer's weight matrix (a pair for GIN).  Both
    evaluations of the layer are differentiated: with u_v = (y_v - y'_v) / (nb ||y_v - y'_v||) the output
    gradients are u and -u, and each passes back through its own evaluation's activations."""
    last = l == model.n_layers
    x2 = ops.axpy(x, eps, 1.0)
    grads = None
    outs = []
    for xx in (x, x2):
        if model.op == "gcn":
            z = ops.spmm(rowptr, col, val, xx)
            outs.append((z, None, ops.linear(z, model.weights[l - 1], relu=not last)))
        elif model.op == "gin":
            w1, w2 = model.weights[l - 1]
            z = ops.spmm(rowptr, col, None, xx, diag=1.0 + model.gin_eps)
            h = ops.linear(z, w1, relu=True)
            outs.append((z, h, ops.linear(h, w2, relu=not last)))
        else:
            b = model.betas[l - 1]
            z = ops.spmm(rowptr, col, val, xx, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
            outs.append((z, None, ops.linear(z, model.weights[l - 1], c_identity=1.0 - b, c_weight=b, relu=not last)))
    (_, _, y), (_, _, y2) = outs
    _, total = ops.row_distance(y, y2)
    u = ops.row_distance_bwd(y, y2, 1.0 / max(1, nb))
    for sign, (z, h, yy) in zip((1.0, -1.0), outs):
        g = u if last else ops.relu_bwd(u, yy)
        if model.op == "gin":
            w1, w2 = model.weights[l - 1]
            dw2 = ops.linear_bwd_weight(h, g, c_weight=sign)
            gh = ops.linear_bwd_input(g, w2, mask=h)
            part = (ops.linear_bwd_weight(z, gh, c_weight=sign), dw2)
            grads = part if grads is None else tuple((a.astype(np.float64) + b).astype(np.float32)
                                                     for a, b in zip(grads, part))
        else:
            c = model.betas[l - 1] if model.op == "gcnii" else 1.0
            part = ops.linear_bwd_weight(z, g, c_weight=sign * c)
            grads = part if grads is None else (grads.astype(np.float64) + part).astype(np.float32)
    return total / max(1, nb), grads

