"""Sequencing of the C-ABI calls for one mini-batch (paper, Algorithm 1).

Nothing is computed here: buffers are torch allocations and every step is a
gas_* call.  For layer l of a batch B with halo V_b \\ B:

    gas_spmm   Z      = aggregation of the mini-batch tensor X over the rows of G_b
    gas_linear Y      = transform(Z)            (gas_mlp2 for GIN), written into rows 0..nb-1 of the next X
    gas_push   H[l]   <- Y   for the in-batch nodes        (not for the last layer)
    gas_pull   X[nb:] <- H[l] for the halo nodes

The first layer's X is a gas_pull of all of V_b from the feature table (exact
inputs); GCNII first applies its graph-agnostic input projection to all rows.
"""
import math

import torch

from . import binding as B


class BatchGraph:
    """Device-side index structure of one batch subgraph plus its plans."""

    def __init__(self, nb, n_id, rowptr, col, deg=None, colptr=None, row=None, max_F=256, normalise=True, timed=False,
                 plan_options=None, csc_pos=None):
        """timed: wait for the device after each part of the per-batch set-up and keep its wall time in
        self.setup_ms (plans, coefficients, fused source indices); the benchmark reports it."""
        import time
        self.setup_ms = {}

        def part(name, fn):
            if not timed:
                return fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            out = fn()
            torch.cuda.synchronize()
            self.setup_ms[name] = round((time.perf_counter() - t0) * 1e3, 3)
            return out

        self.nb, self.nv = int(nb), int(n_id.numel())
        self.n_id, self.rowptr, self.col = n_id, rowptr, col
        self.nnz = int(col.numel())
        self.max_row = int((rowptr[1:] - rowptr[:-1]).max().item()) if self.nb > 0 else 0
        self.plan = part("plan_csr", lambda: B.gas_plan_create(rowptr, self.nnz, max_F, ind=col, options=plan_options))
        self.val = None
        if normalise:
            self.val = torch.empty(self.nnz, dtype=torch.float32, device=col.device)
            part("gcn_norm_csr", lambda: B.gas_gcn_norm(rowptr, col, n_id, deg, self.val))
        self._src = None
        self.csc_pos = csc_pos       # int32[nnz]: position of every CSC entry in the CSR arrays (PNA / GAT backward)
        self._n_id_host = None
        self._plan_t_all, self._max_F = None, max_F
        self.colptr, self.row, self.val_t, self.plan_t = colptr, row, None, None
        if colptr is not None:
            # backward over the in-batch columns only: histories are constants
            nnz_t = int(colptr[self.nb].item())
            self.plan_t = part("plan_csc", lambda: B.gas_plan_create(colptr[: self.nb + 1], nnz_t, max_F,
                                                                     n_rows=self.nb, ind=row, options=plan_options))
            if normalise:
                self.val_t = torch.empty(self.nnz, dtype=torch.float32, device=col.device)
                part("gcn_norm_csc", lambda: B.gas_gcn_norm(colptr, row, n_id, deg, self.val_t))
        if timed:
            part("fuse_sources", lambda: self.src)
            self.setup_ms["total"] = round(sum(self.setup_ms.values()), 3)

    @property
    def plan_t_all(self):
        """Plan of the backward aggregation over ALL columns, halo included (GCNII's first layer: the gradient of
        the projected features of every node of V_b); built on first use, once per batch."""
        if self._plan_t_all is None:
            self._plan_t_all = B.gas_plan_create(self.colptr, self.nnz, self._max_F, ind=self.row)
        return self._plan_t_all

    @property
    def n_id_host(self):
        """The node ids in host memory (index lists of tables on disk are read by host threads)."""
        if self._n_id_host is None:
            self._n_id_host = self.n_id.cpu()
        return self._n_id_host

    @property
    def src(self):
        """Source indices for gas_spmm_hist (built on first use, once per batch)."""
        if self._src is None:
            self._src = torch.empty_like(self.col)
            B.gas_fuse_sources(self.col, self.nb, self.n_id, self._src)
        return self._src


class Model:
    def __init__(self, op, weights, w_in=None, alpha=0.0, gin_eps=0.0):
        self.op, self.weights, self.w_in, self.alpha, self.gin_eps = op, weights, w_in, alpha, gin_eps

    @property
    def n_layers(self):
        return len(self.weights)

    def out_width(self, l):
        w = self.weights[l]
        return (w[1] if self.op == "gin" else w).shape[1]


# Rows longer than this keep the two-kernel form, whose plan splits them over wavefronts; the one-launch layer
# gives a row to one team of lanes.
ONE_LAUNCH_MAX_ROW = 512


def gcnii_beta(layer: int) -> float:
    return math.log(0.5 / layer + 1.0)


def forward_batch_fused(model: Model, bg: BatchGraph, x_feat, histories, do_push=True):
    """Same result as forward_batch, with the halo rows read in place by the
    aggregation (gas_spmm_hist) instead of being pulled into the mini-batch
    tensor, and the Push taken in the transform's epilogue: per layer
    aggregate(X_batch, H[l-1]) -> transform, rows stored to H[l] as well.
    Layer 1 reads its halo rows from the feature table the same way.  GCNII: its first layer aggregates the
    projected features of all of V_b, which no table holds, so that layer gathers from the mini-batch tensor; from
    layer 2 on the halo rows come from the history tables in place.  Narrow fp32 layers of GCN and GCNII (widths
    up to 128, no row above ONE_LAUNCH_MAX_ROW entries) take one launch each (gas_spmm_linear)."""
    dev, dt = x_feat.device, x_feat.dtype
    nb = bg.nb
    if model.op == "gcnii":
        return _forward_gcnii_fused(model, bg, x_feat, histories, do_push)
    x = torch.empty((nb, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id[:nb], x)
    L = model.n_layers
    y = None
    for l in range(1, L + 1):
        last = l == L
        table = x_feat if l == 1 else histories[l - 2]
        y = torch.empty((nb, model.out_width(l - 1)), dtype=dt, device=dev)
        push = not last and do_push          # the transform stores its rows to the next history table as well
        if model.op == "gcn" and B.spmm_linear_supported(x, y.shape[1]) and bg.max_row <= ONE_LAUNCH_MAX_ROW:
            # narrow layers: aggregation, transform and Push in one launch
            B.gas_spmm_linear(bg.rowptr, bg.src, bg.val, x, model.weights[l - 1], y, hist=table, relu=not last,
                              push_idx=bg.n_id[:nb] if push else None, push_hist=histories[l - 1] if push else None)
            x = y
            continue
        z = torch.empty((nb, x.shape[1]), dtype=dt, device=dev)
        if model.op == "gcn":
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, x, table, z)
            if push:
                B.gas_linear_push(z, model.weights[l - 1], y, bg.n_id[:nb], histories[l - 1], relu=True)
            else:
                B.gas_linear(z, model.weights[l - 1], y, relu=not last)
        else:
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, None, x, table, z, diag=1.0 + model.gin_eps)
            w1, w2 = model.weights[l - 1]
            if push:
                B.gas_mlp2_push(z, w1, w2, y, bg.n_id[:nb], histories[l - 1], relu_out=True)
            else:
                B.gas_mlp2(z, w1, w2, y, relu_out=not last)
        x = y
    return y


def _forward_gcnii_fused(model: Model, bg: BatchGraph, x_feat, histories, do_push):
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x0 = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x0)
    h0 = torch.empty((nv, model.w_in.shape[1]), dtype=dt, device=dev)
    B.gas_linear(x0, model.w_in, h0, relu=True)
    x, y = h0, None
    L = model.n_layers
    for l in range(1, L + 1):
        last = l == L
        y = torch.empty((nb, model.out_width(l - 1)), dtype=dt, device=dev)
        beta = gcnii_beta(l)
        push = not last and do_push
        if B.spmm_linear_supported(x, y.shape[1]) and bg.max_row <= ONE_LAUNCH_MAX_ROW:
            # narrow layers: aggregation, transform and Push in one launch
            B.gas_spmm_linear(bg.rowptr, bg.col if l == 1 else bg.src, bg.val, x, model.weights[l - 1], y,
                              hist=None if l == 1 else histories[l - 2], s_agg=1.0 - model.alpha, r=h0,
                              s_res=model.alpha, c_identity=1.0 - beta, c_weight=beta, relu=not last,
                              push_idx=bg.n_id[:nb] if push else None, push_hist=histories[l - 1] if push else None)
            x = y
            continue
        z = torch.empty((nb, h0.shape[1]), dtype=dt, device=dev)
        if l == 1:
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
        else:
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, x, histories[l - 2], z, s_agg=1.0 - model.alpha, r=h0,
                            s_res=model.alpha)
        if push:
            B.gas_linear_push(z, model.weights[l - 1], y, bg.n_id[:nb], histories[l - 1], c_identity=1.0 - beta,
                              c_weight=beta, relu=True)
        else:
            B.gas_linear(z, model.weights[l - 1], y, c_identity=1.0 - beta, c_weight=beta, relu=not last)
        x = y
    return y


def _aggregate_transform(model: Model, l, bg: BatchGraph, x, h0, z, y):
    """Layer l (1-based) on the mini-batch tensor x: aggregation into z, transform into y (ReLU unless last)."""
    last = l == model.n_layers
    if model.op == "gcn":
        B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z)
        B.gas_linear(z, model.weights[l - 1], y, relu=not last)
    elif model.op == "gin":
        B.gas_spmm(bg.plan, bg.rowptr, bg.col, None, x, z, diag=1.0 + model.gin_eps)
        w1, w2 = model.weights[l - 1]
        B.gas_mlp2(z, w1, w2, y, relu_out=not last)
    elif model.op == "gcnii":
        B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
        beta = gcnii_beta(l)
        B.gas_linear(z, model.weights[l - 1], y, c_identity=1.0 - beta, c_weight=beta, relu=not last)
    else:
        raise ValueError(model.op)


def forward_batch(model: Model, bg: BatchGraph, x_feat, histories, do_push=True, keep_layers=False):
    """Run all layers for one batch.  Returns the last layer's [nb, F] output
    (and the list of mini-batch tensors if keep_layers)."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    h0 = None
    if model.op == "gcnii":
        h0 = torch.empty((nv, model.w_in.shape[1]), dtype=dt, device=dev)
        B.gas_linear(x, model.w_in, h0, relu=True)
        x = h0
    layers = []
    L = model.n_layers
    y = None
    for l in range(1, L + 1):
        last = l == L
        f_in, f_out = x.shape[1], model.out_width(l - 1)
        z = torch.empty((nb, f_in), dtype=dt, device=dev)
        if last:
            y = torch.empty((nb, f_out), dtype=dt, device=dev)
        else:
            x_next = torch.empty((nv, f_out), dtype=dt, device=dev)
            y = x_next[:nb]
        _aggregate_transform(model, l, bg, x, h0, z, y)
        if last:
            break
        if do_push:
            B.gas_push(y, bg.n_id[:nb], histories[l - 1])
        if nv > nb:
            B.gas_pull(histories[l - 1], bg.n_id[nb:], x_next[nb:])
        x = x_next
        if keep_layers:
            layers.append(x)
    return (y, layers) if keep_layers else y


class HostPipeline:
    """Streams for histories kept in host memory (Section 5 "PyGAS" of the paper: history access runs beside the
    computation).  One stream carries the pulls, one the pushes, both at the default priority.  The mini-batch
    tensors the transfers touch belong to the pipeline: two sets, used by alternate batches, so that a batch can
    compute while the pushes of the one before still read its tensors.  Events: `table_pushed[l]`, the end of the
    last push into table l (a later pull from that table waits for it); `set_pushed[i]` / `set_read[i]`, the end
    of the pushes / of the computation that last read set i (the next writers of that set wait for them)."""

    def __init__(self, device):
        self.pull = torch.cuda.Stream(device)
        self.push = torch.cuda.Stream(device)
        self.turn = 0
        self.table_pushed = {}
        self.set_pushed = [None, None]
        self.set_read = [None, None]
        self._buffers = {}
        self._fresh = False

    def buffer(self, l, rows, width, dtype, device):
        """The mini-batch tensor of the current set that layer l writes and layer l + 1 reads; grown when a
        batch needs more rows."""
        key = (self.turn, l, width, dtype)
        t = self._buffers.get(key)
        if t is None or t.shape[0] < rows:
            if t is not None:                    # the transfer streams may still be using the old tensor
                t.record_stream(self.pull)
                t.record_stream(self.push)
            t = self._buffers[key] = torch.empty((rows, width), dtype=dtype, device=device)
            self._fresh = True                   # memory the compute stream may still be using
        return t[:rows]

    def join(self):
        """Make the current stream wait for every transfer issued so far."""
        cur = torch.cuda.current_stream()
        cur.wait_stream(self.pull)
        cur.wait_stream(self.push)


def forward_batch_host(model: Model, bg: BatchGraph, x_feat, histories, pipe: HostPipeline, do_push=True):
    """forward_batch for history tables in pinned host memory (binding.HostTable), with the transfers taken off
    the compute stream: the halo rows of every layer are pulled ahead on pipe.pull (they were pushed by earlier
    batches, so none depends on this batch's computation) and each layer's output is pushed on pipe.push while
    the next layer computes.  A layer waits only for its own halo rows, a pull only for the earlier pushes into
    its own table.  Same bits as forward_batch: in-batch and halo rows of a table are disjoint, so the order of
    this batch's pushes and pulls is immaterial (Algorithm 1).  The caller calls pipe.join() before it reads the
    tables or uses them outside this function."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    L = model.n_layers
    cur = torch.cuda.current_stream()
    turn = pipe.turn = pipe.turn ^ 1
    pipe._fresh = False
    xs = [None] + [pipe.buffer(l, nv, model.out_width(l - 1), dt, dev) for l in range(1, L)]
    pulled = [None] * L
    if nv > nb:
        with torch.cuda.stream(pipe.pull):
            if pipe._fresh or pipe.set_read[turn] is None:
                pipe.pull.wait_stream(cur)
            else:
                pipe.pull.wait_event(pipe.set_read[turn])
            for l in range(1, L):
                if l - 1 in pipe.table_pushed:
                    pipe.pull.wait_event(pipe.table_pushed[l - 1])
                B.gas_pull(histories[l - 1], bg.n_id[nb:], xs[l][nb:])
                pulled[l] = torch.cuda.Event()
                pulled[l].record(pipe.pull)
    if pipe.set_pushed[turn] is not None:
        cur.wait_event(pipe.set_pushed[turn])    # pushes that still read the rows the layers overwrite
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    h0 = None
    if model.op == "gcnii":
        h0 = torch.empty((nv, model.w_in.shape[1]), dtype=dt, device=dev)
        B.gas_linear(x, model.w_in, h0, relu=True)
        x = h0
    y = None
    for l in range(1, L + 1):
        last = l == L
        z = torch.empty((nb, x.shape[1]), dtype=dt, device=dev)
        y = torch.empty((nb, model.out_width(l - 1)), dtype=dt, device=dev) if last else xs[l][:nb]
        if l > 1 and pulled[l - 1] is not None:
            cur.wait_event(pulled[l - 1])
        _aggregate_transform(model, l, bg, x, h0, z, y)
        if last:
            break
        if do_push:
            done = torch.cuda.Event()
            done.record(cur)
            with torch.cuda.stream(pipe.push):
                pipe.push.wait_event(done)
                B.gas_push(y, bg.n_id[:nb], histories[l - 1])
                pipe.table_pushed[l - 1] = torch.cuda.Event()
                pipe.table_pushed[l - 1].record(pipe.push)
        x = xs[l]
    pipe.set_read[turn] = torch.cuda.Event()
    pipe.set_read[turn].record(cur)
    if do_push and L > 1:
        pipe.set_pushed[turn] = pipe.table_pushed[L - 2]
    return y


class DiskPipeline:
    """Mini-batch tensors for histories kept on disk (binding.DiskTable): two sets, used by alternate batches, so
    that a batch can compute while the pushes of the one before still read its tensors; `pushing[i]` lists the
    (table, ticket) pairs of the pushes that read set i."""

    def __init__(self):
        self.turn = 0
        self.pushing = [[], []]
        self._buffers = {}

    def buffer(self, l, rows, width, dtype, device):
        key = (self.turn, l, width, dtype)
        t = self._buffers.get(key)
        if t is None or t.shape[0] < rows:
            t = self._buffers[key] = torch.empty((rows, width), dtype=dtype, device=device)
        return t[:rows]

    def settle(self, turn):
        """Wait for the pushes that still read the tensors of set `turn`."""
        for table, ticket in self.pushing[turn]:
            table.wait(ticket)
        self.pushing[turn] = []

    def join(self):
        self.settle(0)
        self.settle(1)


def forward_batch_disk(model: Model, bg: BatchGraph, x_feat, tables, pipe: DiskPipeline, do_push=True):
    """forward_batch for history tables on disk (the tier the paper's "Conclusion and Future Work" names; transfer
    scheme of its Section 5 "PyGAS").  The halo rows of every layer are requested at the start of the batch (they
    were pushed by earlier batches; each table runs its transfers in the order queued, so a pull sees the pushes
    queued before it), a layer waits for its own halo rows only, and each layer's output goes to its table while
    the next layer computes.  Same bits as forward_batch.  The caller calls pipe.join() before it reads the tables."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    L = model.n_layers
    turn = pipe.turn = pipe.turn ^ 1
    pipe.settle(turn)
    ids = bg.n_id_host
    xs = [None] + [pipe.buffer(l, nv, model.out_width(l - 1), dt, dev) for l in range(1, L)]
    pulled = [None] * L
    if nv > nb:
        # the transfer starts after the work queued so far, which includes the last readers of this set
        for l in range(1, L):
            pulled[l] = tables[l - 1].pull(ids[nb:], xs[l][nb:])
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    h0 = None
    if model.op == "gcnii":
        h0 = torch.empty((nv, model.w_in.shape[1]), dtype=dt, device=dev)
        B.gas_linear(x, model.w_in, h0, relu=True)
        x = h0
    y = None
    for l in range(1, L + 1):
        last = l == L
        z = torch.empty((nb, x.shape[1]), dtype=dt, device=dev)
        y = torch.empty((nb, model.out_width(l - 1)), dtype=dt, device=dev) if last else xs[l][:nb]
        if l > 1 and pulled[l - 1] is not None:
            tables[l - 2].wait(pulled[l - 1])
        _aggregate_transform(model, l, bg, x, h0, z, y)
        if last:
            break
        if do_push:
            pipe.pushing[turn].append((tables[l - 1], tables[l - 1].push(y, ids[:nb])))
        x = xs[l]
    return y


def train_batch(model: Model, bg: BatchGraph, x_feat, histories, grad_out, do_push=True, fused=False):
    """Forward with the activations kept, then the backward pass through all layers (no optimiser step).
    Historical embeddings are constants, so gradients travel along in-batch rows only; GCNII's input projection
    is computed in-graph for the halo rows too and its gradient includes them.  GIN's MLP stores its hidden
    activation here (gas_mlp2_keep: the backward pass reads it again).  Returns (Y_L, grads, kept) with
    grads[l] = dW_l (float32; a pair for GIN), grads["w_in"] for GCNII, and kept = the stored activations the
    backward pass read (x0, h0, per layer (Z, hidden, Y)).  grad_out is dLoss/dY_L [nb, F_L], or a function
    that returns it given Y_L.  fused: the forward aggregations read their halo rows from the feature table / the
    history tables in place (gas_spmm_hist) and nothing is pulled; same bits.  GCNII's first layer gathers the
    projected features from the mini-batch tensor, its later layers from the histories.  Narrow fp32 layers of
    GCN and GCNII then take one launch each (gas_spmm_linear with Z kept; the row sums are taken in another order,
    so these agree with the other form to rounding, not bit for bit).  Every step is a gas_* call."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    all_rows = not fused or model.op == "gcnii"      # GCNII projects the features of every node of V_b
    x0 = torch.empty((nv if all_rows else nb, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id if all_rows else bg.n_id[:nb], x0)
    x, h0 = x0, None
    if model.op == "gcnii":
        h0 = torch.empty((nv, model.w_in.shape[1]), dtype=dt, device=dev)
        B.gas_linear(x0, model.w_in, h0, relu=True)
        x = h0
    L = model.n_layers
    saved = []
    y = None
    for l in range(1, L + 1):
        last = l == L
        f_in, f_out = x.shape[1], model.out_width(l - 1)
        z = torch.empty((nb, f_in), dtype=dt, device=dev)
        x_next = torch.empty((nb if (last or fused) else nv, f_out), dtype=dt, device=dev)
        y = x_next[:nb]
        h, pushed = None, False
        table = (x_feat if l == 1 else histories[l - 2]) if fused else None
        if fused and model.op == "gcnii" and l == 1:
            table = None                                  # layer 1 gathers the projected features from h0 itself
        one_launch = (fused and model.op in ("gcn", "gcnii") and B.spmm_linear_supported(x, f_out)
                      and bg.max_row <= ONE_LAUNCH_MAX_ROW)
        if one_launch:
            # narrow layers: aggregation, transform and Push in one launch; Z is kept for the weight gradient
            push = not last and do_push
            beta = gcnii_beta(l) if model.op == "gcnii" else 1.0
            kw = dict(s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha, c_identity=1.0 - beta,
                      c_weight=beta) if model.op == "gcnii" else {}
            B.gas_spmm_linear(bg.rowptr, bg.col if table is None else bg.src, bg.val, x, model.weights[l - 1], y,
                              hist=table, relu=not last, z_out=z, push_idx=bg.n_id[:nb] if push else None,
                              push_hist=histories[l - 1] if push else None, **kw)
            saved.append((z, h, y))
            if last:
                break
            x = x_next
            continue
        if model.op == "gcn":
            if fused:
                B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, x, table, z)
            else:
                B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z)
            B.gas_linear(z, model.weights[l - 1], y, relu=not last)
        elif model.op == "gin":
            if fused:
                B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, None, x, table, z, diag=1.0 + model.gin_eps)
            else:
                B.gas_spmm(bg.plan, bg.rowptr, bg.col, None, x, z, diag=1.0 + model.gin_eps)
            w1, w2 = model.weights[l - 1]
            h = torch.empty((nb, w1.shape[1]), dtype=dt, device=dev)
            # both products in one call, the hidden activation stored for the backward pass, the Push in its epilogue
            push = not last and do_push
            B.gas_mlp2_keep(z, w1, w2, y, h, idx=bg.n_id[:nb] if push else None,
                            hist=histories[l - 1] if push else None, relu_out=not last)
            pushed = push
        else:
            if table is not None:
                B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, x, table, z, s_agg=1.0 - model.alpha, r=h0,
                                s_res=model.alpha)
            else:
                B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
            beta = gcnii_beta(l)
            B.gas_linear(z, model.weights[l - 1], y, c_identity=1.0 - beta, c_weight=beta, relu=not last)
        saved.append((z, h, y))
        if last:
            break
        if do_push and not pushed:
            B.gas_push(y, bg.n_id[:nb], histories[l - 1])
        if nv > nb and not fused:
            B.gas_pull(histories[l - 1], bg.n_id[nb:], x_next[nb:])
        x = x_next
    # ---- backward
    def weight_grad(zz, gg, c=1.0):
        dw = torch.empty((zz.shape[1], gg.shape[1]), dtype=torch.float32, device=dev)
        ws = torch.empty(max(1, B.gas_linear_bwd_weight_workspace(zz.shape[0], zz.shape[1], gg.shape[1])),
                         dtype=torch.uint8, device=dev)
        B.gas_linear_bwd_weight(zz, gg, dw, ws, c_weight=c)
        return dw

    grads = {}
    g = grad_out(y) if callable(grad_out) else grad_out     # a loss: gradient at the output, from the output
    g_h0 = None
    for l in range(L, 0, -1):
        z, h, yl = saved[l - 1]
        if l != L:
            gp = torch.empty_like(g)
            B.gas_relu_bwd(g, yl, gp)
            g = gp
        gz = torch.empty_like(z)
        if model.op == "gcn":
            grads[l - 1] = weight_grad(z, g)
            B.gas_linear_bwd_input(g, model.weights[l - 1], gz)
        elif model.op == "gin":
            w1, w2 = model.weights[l - 1]
            dw2 = weight_grad(h, g)
            gh = torch.empty_like(h)
            B.gas_linear_bwd_input(g, w2, gh, mask=h)
            grads[l - 1] = (weight_grad(z, gh), dw2)
            B.gas_linear_bwd_input(gh, w1, gz)
            # gradient of this layer's eps: sum over the in-batch nodes of <dL/dZ_v, h_v> (h = the layer's input)
            if "eps" not in grads:
                grads["eps"] = torch.zeros(L, dtype=torch.float32, device=dev)
            x_in = x0 if l == 1 else saved[l - 2][2]
            B.gas_row_dot(gz, x_in[:nb], torch.empty(nb, dtype=torch.float32, device=dev), grads["eps"][l - 1:l])
        else:
            beta = gcnii_beta(l)
            grads[l - 1] = weight_grad(z, g, beta)
            B.gas_linear_bwd_input(g, model.weights[l - 1], gz, c_identity=1.0 - beta, c_weight=beta)
            if g_h0 is None:
                g_h0 = torch.zeros((nv, gz.shape[1]), dtype=dt, device=dev)
            B.gas_axpy(g_h0[:nb], gz, g_h0[:nb], model.alpha)      # the initial residual's share: g_h0 += alpha * gz
        if l == 1:
            if model.op == "gcnii":
                gx = torch.empty((nv, gz.shape[1]), dtype=dt, device=dev)
                B.gas_spmm_t(bg.plan_t_all, bg.colptr, bg.row, bg.val_t, gz, gx, s_agg=1.0 - model.alpha)
                B.gas_axpy(g_h0, gx, g_h0, 1.0)
            break
        gx = torch.empty((nb, gz.shape[1]), dtype=dt, device=dev)
        if model.op == "gin":
            B.gas_spmm_t(bg.plan_t, bg.colptr, bg.row, None, gz, gx, diag=1.0 + model.gin_eps)
        elif model.op == "gcn":
            B.gas_spmm_t(bg.plan_t, bg.colptr, bg.row, bg.val_t, gz, gx)
        else:
            B.gas_spmm_t(bg.plan_t, bg.colptr, bg.row, bg.val_t, gz, gx, s_agg=1.0 - model.alpha)
        g = gx
    if model.op == "gcnii":
        gp = torch.empty_like(g_h0)
        B.gas_relu_bwd(g_h0, h0, gp)
        grads["w_in"] = weight_grad(x0, gp)
    return y, grads, {"x0": x0, "h0": h0, "layers": saved}


def apply_sgd(model: Model, grads, lr, weight_decay=0.0, max_norm=None):
    """One gradient-descent update of every weight matrix, in place (gas_sgd_step per matrix).  max_norm: the
    gradients are first clipped by their global L2 norm (paper, Section 3): one gas_sq_norm per gradient, then
    gas_sgd_step_clipped, which forms the common factor on the device."""
    pairs = []
    for l in range(model.n_layers):
        if model.op == "gin":
            pairs += list(zip(model.weights[l], grads[l]))
        else:
            pairs.append((model.weights[l], grads[l]))
    if model.op == "gcnii":
        pairs.append((model.w_in, grads["w_in"]))
    if max_norm is None:
        for w, dw in pairs:
            B.gas_sgd_step(w, dw, lr, weight_decay)
        return
    sq = torch.empty(len(pairs), dtype=torch.float32, device=pairs[0][0].device)
    for k, (_, dw) in enumerate(pairs):
        B.gas_sq_norm(dw, sq[k:k + 1])
    for w, dw in pairs:
        B.gas_sgd_step_clipped(w, dw, lr, sq, max_norm, weight_decay)


def layer_input(model: Model, l, bg: BatchGraph, kept, histories):
    """The mini-batch tensor [nv, F] layer l read in a pass whose activations were kept (train_batch, not fused):
    the features (GCNII: the projected features) for l = 1, else layer l-1's output for the in-batch rows and the
    halo rows as they stand in history table l-1 (this batch's pushes do not touch them)."""
    if l == 1:
        return kept["h0"] if model.op == "gcnii" else kept["x0"]
    y = kept["layers"][l - 2][2]
    x = torch.empty((bg.nv, y.shape[1]), dtype=y.dtype, device=y.device)
    B.gas_pull(y, None, x[:bg.nb], base=0, n=bg.nb)
    if bg.nv > bg.nb:
        B.gas_pull(histories[l - 2], bg.n_id[bg.nb:], x[bg.nb:])
    return x


def train_step(model: Model, bg: BatchGraph, x_feat, histories, labels_batch, lr, weight_decay=0.0, n_labelled=None,
               fused=False, max_norm=None, reg_weight=0.0, reg_eps=None):
    """One optimisation step of Algorithm 1's loop body on one mini-batch: forward with Push/Pull per layer,
    softmax cross-entropy averaged over the labelled in-batch nodes, backward with the histories held constant,
    gradient-descent update of the weights (in place).  labels_batch: int32 [nb], the labels of the in-batch
    nodes in batch order, < 0 = unlabelled; n_labelled: their count if the caller knows it (saves a device
    read-back).  reg_weight: the local Lipschitz regulariser of Eq. (3) is added for every layer (lipschitz_reg_grad
    on the layer's kept input).  Returns (loss_sum as a 1-element float32 device tensor, n_labelled, logits, grads)."""
    if n_labelled is None:
        n_labelled = int((labels_batch >= 0).sum().item())
    dev = x_feat.device
    loss_rows = torch.empty(bg.nb, dtype=torch.float32, device=dev)
    loss_sum = torch.empty(1, dtype=torch.float32, device=dev)

    def loss_grad(y):
        g = torch.empty_like(y)
        B.gas_softmax_xent(y, labels_batch, g, loss_rows, loss_sum, scale=1.0 / max(1, n_labelled))
        return g
    y, grads, kept = train_batch(model, bg, x_feat, histories, loss_grad, fused=fused)
    if reg_weight != 0.0:
        # loss + reg_weight * sum over the layers of Eq. (3), each differentiated with respect to its layer's
        # weights; reg_eps[l-1]: layer l's drawn perturbations [nv, F_in]
        if fused:
            raise ValueError("the regulariser perturbs the whole mini-batch tensor of every layer: fused=False")
        for l in range(1, model.n_layers + 1):
            _, _, dw = lipschitz_reg_grad(model, l, bg, layer_input(model, l, bg, kept, histories), reg_eps[l - 1],
                                          kept["h0"])
            for a, b in zip(grads[l - 1] if model.op == "gin" else (grads[l - 1],), dw if model.op == "gin" else (dw,)):
                B.gas_axpy(a, b, a, reg_weight)
    apply_sgd(model, grads, lr, weight_decay, max_norm)
    return loss_sum, n_labelled, y, grads


def appnp_forward_batch(w1, w2, alpha, n_steps, bg: BatchGraph, x_feat, histories, do_push=True, fused=False):
    """APPNP (paper, operator appendix) on one mini-batch: h0 = relu(x W1) W2 for every row of the mini-batch
    tensor (graph-agnostic, so exact for halo rows), then n_steps propagation steps
    h <- alpha h0 + (1 - alpha) A_hat h, each one aggregation call with the residual in its epilogue; steps
    1..K-1 are pushed to histories[l-1] and their halo rows pulled back.  fused: from step 2 on the aggregation
    reads the halo rows from the history table in place (no pull).  Returns h^(K) of the in-batch rows."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x0 = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x0)
    h0 = torch.empty((nv, w2.shape[1]), dtype=dt, device=dev)
    B.gas_mlp2(x0, w1, w2, h0, relu_out=False)
    x, y = h0, None
    for l in range(1, n_steps + 1):
        last = l == n_steps
        x_next = torch.empty((nb if (last or fused) else nv, h0.shape[1]), dtype=dt, device=dev)
        y = x_next[:nb]
        if fused and l > 1:
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, x, histories[l - 2], y, s_agg=1.0 - alpha, r=h0,
                            s_res=alpha)
        else:
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, y, s_agg=1.0 - alpha, r=h0, s_res=alpha)
        if last:
            break
        if do_push:
            B.gas_push(y, bg.n_id[:nb], histories[l - 1])
        if not fused and nv > nb:
            B.gas_pull(histories[l - 1], bg.n_id[nb:], x_next[nb:])
        x = x_next
    return y


def pna_layer(x, nb, rowptr, col, w1, w2, delta, relu, y=None):
    """One PNA layer (paper, operator appendix) for the in-batch rows: h'_v = W2 [h_v, (+)_w W1 [h_v, h_w]].
    x: mini-batch tensor [nv, F]; w1 [2F, F1] (rows 0..F-1 multiply the receiving node, rows F.. the neighbour),
    w2 [F + 9 F1, F_out].  The neighbour part of a message is computed once per node (gas_linear over all of
    V_b), aggregated by mean, min and max in one pass with the degree scalers (gas_pna_aggregate), the
    receiving-node part is added inside that call, and the concatenation with h_v is laid out in one buffer
    that the second gas_linear reads."""
    dev, dt = x.device, x.dtype
    f, f1 = x.shape[1], w1.shape[1]
    p = torch.empty((x.shape[0], f1), dtype=dt, device=dev)
    B.gas_linear(x, w1[f:], p)
    q = torch.empty((nb, f1), dtype=dt, device=dev)
    B.gas_linear(x[:nb], w1[:f], q)
    cat = torch.empty((nb, f + 9 * f1), dtype=dt, device=dev)
    B.gas_pull(x, None, cat[:, :f], base=0, n=nb)                 # h_v into the first F columns (a strided row copy)
    B.gas_pna_aggregate(rowptr, col, p, cat[:, f:], delta, add=q)
    if y is None:
        y = torch.empty((nb, w2.shape[1]), dtype=dt, device=dev)
    B.gas_linear(cat, w2, y, relu=relu)
    return y


def pna_forward_batch(weights, delta, bg: BatchGraph, x_feat, histories, do_push=True):
    """All layers of a PNA model for one mini-batch in the order of Algorithm 1; weights[l] = (W1, W2)."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    L = len(weights)
    y = None
    for l in range(1, L + 1):
        w1, w2 = weights[l - 1]
        last = l == L
        x_next = torch.empty((nb if last else nv, w2.shape[1]), dtype=dt, device=dev)
        y = pna_layer(x, nb, bg.rowptr, bg.col, w1, w2, delta, relu=not last, y=x_next[:nb])
        if last:
            break
        if do_push:
            B.gas_push(y, bg.n_id[:nb], histories[l - 1])
        if nv > nb:
            B.gas_pull(histories[l - 1], bg.n_id[nb:], x_next[nb:])
        x = x_next
    return y


def gat_forward_batch(weights, bg: BatchGraph, x_feat, histories, negative_slope=0.2, do_push=True, heads=1):
    """All layers of a GAT (paper, operator appendix) for one mini-batch in the order of Algorithm 1;
    weights[l] = (W, a_dst, a_src); bg: the batch subgraph with self-loops.  Per layer: P = X W for every row of
    the mini-batch tensor (gas_linear), then scores, softmax and weighted sum in one pass (gas_gat_aggregate,
    ReLU in its epilogue on all layers but the last), push, pull.  heads > 1: the columns of W, a_dst and a_src are
    `heads` equal blocks; one gas_gat_aggregate call per head on its block of columns of P (a strided view),
    writing its block of the output."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    L = len(weights)
    y = None
    for l in range(1, L + 1):
        w, a_dst, a_src = weights[l - 1]
        last = l == L
        p = torch.empty((nv, w.shape[1]), dtype=dt, device=dev)
        B.gas_linear(x, w, p)
        x_next = torch.empty((nb if last else nv, w.shape[1]), dtype=dt, device=dev)
        y = x_next[:nb]
        fh = w.shape[1] // heads
        if fh * heads != w.shape[1]:
            raise ValueError("gat_forward_batch: the layer width is not a multiple of the number of heads")
        for h in range(heads):
            cols = slice(h * fh, (h + 1) * fh)
            B.gas_gat_aggregate(bg.rowptr, bg.col, p[:, cols], a_dst[cols], a_src[cols], y[:, cols], negative_slope,
                                relu=not last)
        if last:
            break
        if do_push:
            B.gas_push(y, bg.n_id[:nb], histories[l - 1])
        if nv > nb:
            B.gas_pull(histories[l - 1], bg.n_id[nb:], x_next[nb:])
        x = x_next
    return y


def _weight_grad(zz, gg, dw=None):
    if dw is None:
        dw = torch.empty((zz.shape[1], gg.shape[1]), dtype=torch.float32, device=zz.device)
    ws = torch.empty(max(1, B.gas_linear_bwd_weight_workspace(zz.shape[0], zz.shape[1], gg.shape[1])),
                     dtype=torch.uint8, device=zz.device)
    B.gas_linear_bwd_weight(zz, gg, dw, ws)
    return dw


def _next_input(y_rows, bg: BatchGraph, history, do_push):
    """Push the in-batch rows (already in rows 0..nb-1 of the next mini-batch tensor) and pull its halo rows."""
    if do_push:
        B.gas_push(y_rows[:bg.nb], bg.n_id[:bg.nb], history)
    if bg.nv > bg.nb:
        B.gas_pull(history, bg.n_id[bg.nb:], y_rows[bg.nb:])


def pna_train_batch(weights, delta, bg: BatchGraph, x_feat, histories, grad_out, do_push=True):
    """pna_forward_batch with the activations kept, then the backward pass (operator appendix, PNA; histories are
    constants, so only in-batch rows pass gradient to the layer below, while the neighbour half of W1 takes gradient
    through every row of V_b).  bg needs the CSC copy with csc_pos.  grad_out: dLoss/dY_L [nb, F_L] or a function of
    Y_L.  Returns (Y_L, grads, kept) with grads[l] = (dW1 [2F, F1], dW2), float32, and kept[l] = the stored
    activations (X, P, [X[:nb] | A9], Y) the backward pass read.  Every step is a gas_* call."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    L = len(weights)
    kept = []
    y = None
    for l in range(1, L + 1):
        w1, w2 = weights[l - 1]
        last = l == L
        f, f1 = x.shape[1], w1.shape[1]
        p = torch.empty((nv, f1), dtype=dt, device=dev)
        B.gas_linear(x, w1[f:], p)
        q = torch.empty((nb, f1), dtype=dt, device=dev)
        B.gas_linear(x[:nb], w1[:f], q)
        cat = torch.empty((nb, f + 9 * f1), dtype=dt, device=dev)
        B.gas_pull(x, None, cat[:, :f], base=0, n=nb)
        B.gas_pna_aggregate(bg.rowptr, bg.col, p, cat[:, f:], delta, add=q)
        x_next = torch.empty((nb if last else nv, w2.shape[1]), dtype=dt, device=dev)
        y = x_next[:nb]
        B.gas_linear(cat, w2, y, relu=not last)
        kept.append((x, p, cat, y))
        if last:
            break
        _next_input(x_next, bg, histories[l - 1], do_push)
        x = x_next
    grads = {}
    g = grad_out(y) if callable(grad_out) else grad_out
    for l in range(L, 0, -1):
        w1, w2 = weights[l - 1]
        x, p, cat, yl = kept[l - 1]
        f, f1 = x.shape[1], w1.shape[1]
        if l != L:
            gm = torch.empty_like(g)
            B.gas_relu_bwd(g, yl, gm)
            g = gm
        dw2 = _weight_grad(cat, g)
        gcat = torch.empty_like(cat)
        B.gas_linear_bwd_input(g, w2, gcat)
        gp = torch.empty((nv, f1), dtype=dt, device=dev)
        gq = torch.empty((nb, f1), dtype=dt, device=dev)
        B.gas_pna_aggregate_bwd(bg.rowptr, bg.col, bg.colptr, bg.row, bg.csc_pos, p, gcat[:, f:], gp, delta, gadd=gq,
                                plan_t=bg.plan_t_all)
        dw1 = torch.empty((2 * f, f1), dtype=torch.float32, device=dev)
        _weight_grad(x[:nb], gq, dw1[:f])
        _weight_grad(x, gp, dw1[f:])
        grads[l - 1] = (dw1, dw2)
        if l == 1:
            break
        # dL/dX[:nb] = the copy of h_v in the concatenation + the neighbour part + the receiving-node part
        gx = torch.empty((nb, f), dtype=dt, device=dev)
        B.gas_linear_bwd_input(gp[:nb], w1[f:], gx)
        B.gas_axpy(gcat[:, :f], gx, gx, 1.0)
        t = torch.empty((nb, f), dtype=dt, device=dev)
        B.gas_linear_bwd_input(gq, w1[:f], t)
        B.gas_axpy(gx, t, gx, 1.0)
        g = gx
    return y, grads, kept


def gat_train_batch(weights, bg: BatchGraph, x_feat, histories, grad_out, negative_slope=0.2, do_push=True, heads=1):
    """gat_forward_batch with the activations kept, then the backward pass (operator appendix, GAT).  P = X W is
    computed for every node of V_b, so W takes gradient through all nv rows of P's gradient; only in-batch rows pass
    gradient to the layer below.  bg: the batch subgraph with self-loops and the CSC copy with csc_pos.
    Returns (Y_L, grads, kept) with grads[l] = (dW, d a_dst, d a_src), float32, and kept[l] = (X, P, Y).  Every
    step is a gas_* call."""
    dev, dt = x_feat.device, x_feat.dtype
    nb, nv = bg.nb, bg.nv
    x = torch.empty((nv, x_feat.shape[1]), dtype=dt, device=dev)
    B.gas_pull(x_feat, bg.n_id, x)
    L = len(weights)
    kept = []
    y = None

    def blocks(width):
        fh = width // heads
        if fh * heads != width:
            raise ValueError("gat_train_batch: the layer width is not a multiple of the number of heads")
        return [slice(h * fh, (h + 1) * fh) for h in range(heads)]
    for l in range(1, L + 1):
        w, a_dst, a_src = weights[l - 1]
        last = l == L
        p = torch.empty((nv, w.shape[1]), dtype=dt, device=dev)
        B.gas_linear(x, w, p)
        x_next = torch.empty((nb if last else nv, w.shape[1]), dtype=dt, device=dev)
        y = x_next[:nb]
        for c in blocks(w.shape[1]):
            B.gas_gat_aggregate(bg.rowptr, bg.col, p[:, c], a_dst[c], a_src[c], y[:, c], negative_slope, relu=not last)
        kept.append((x, p, y))
        if last:
            break
        _next_input(x_next, bg, histories[l - 1], do_push)
        x = x_next
    grads = {}
    g = grad_out(y) if callable(grad_out) else grad_out
    for l in range(L, 0, -1):
        w, a_dst, a_src = weights[l - 1]
        x, p, yl = kept[l - 1]
        if l != L:
            gm = torch.empty_like(g)
            B.gas_relu_bwd(g, yl, gm)
            g = gm
        gp = torch.empty_like(p)
        gd = torch.empty(w.shape[1], dtype=torch.float32, device=dev)
        gs = torch.empty(w.shape[1], dtype=torch.float32, device=dev)
        for c in blocks(w.shape[1]):
            B.gas_gat_aggregate_bwd(bg.rowptr, bg.col, bg.colptr, bg.row, bg.csc_pos, p[:, c], a_dst[c], a_src[c],
                                    g[:, c], gp[:, c], gd[c], gs[c], negative_slope, plan_t=bg.plan_t_all)
        grads[l - 1] = (_weight_grad(x, gp), gd, gs)
        if l == 1:
            break
        gx = torch.empty((nb, w.shape[0]), dtype=dt, device=dev)
        B.gas_linear_bwd_input(gp[:nb], w, gx)
        g = gx
    return y, grads, kept


def sgd_update(weights, grads, lr, weight_decay=0.0):
    """gas_sgd_step on every tensor of a list of per-layer weight tuples (PNA, GAT) with the matching gradients."""
    for l, ws in enumerate(weights):
        for w, dw in zip(ws, grads[l]):
            B.gas_sgd_step(w, dw, lr, weight_decay)


def layer_forward(model: Model, l, bg: BatchGraph, x, h0=None, y=None):
    """Layer l (1-based) of the model applied to a mini-batch tensor x [nv, F]: output for the in-batch rows."""
    dev, dt = x.device, x.dtype
    nb = bg.nb
    last = l == model.n_layers
    z = torch.empty((nb, x.shape[1]), dtype=dt, device=dev)
    if y is None:
        y = torch.empty((nb, model.out_width(l - 1)), dtype=dt, device=dev)
    if model.op == "gcn":
        B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z)
        B.gas_linear(z, model.weights[l - 1], y, relu=not last)
    elif model.op == "gin":
        B.gas_spmm(bg.plan, bg.rowptr, bg.col, None, x, z, diag=1.0 + model.gin_eps)
        w1, w2 = model.weights[l - 1]
        B.gas_mlp2(z, w1, w2, y, relu_out=not last)
    elif model.op == "gcnii":
        B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, x, z, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
        beta = gcnii_beta(l)
        B.gas_linear(z, model.weights[l - 1], y, c_identity=1.0 - beta, c_weight=beta, relu=not last)
    else:
        raise ValueError(model.op)
    return y


def lipschitz_reg(model: Model, l, bg: BatchGraph, x, eps, h0=None):
    """Eq. (3) for layer l on one mini-batch: the layer applied to the mini-batch tensor x and to x + eps (one
    drawn perturbation per row, in-batch and halo rows alike), and the mean over the in-batch nodes of the
    distance between the two output rows.  Returns (sum of distances as a 1-element device tensor, nb)."""
    dev = x.device
    y = layer_forward(model, l, bg, x, h0)
    xp = torch.empty_like(x)
    B.gas_axpy(x, eps, xp, 1.0)
    y2 = layer_forward(model, l, bg, xp, h0)
    dist = torch.empty(bg.nb, dtype=torch.float32, device=dev)
    total = torch.empty(1, dtype=torch.float32, device=dev)
    B.gas_row_distance(y, y2, dist, total)
    return total, bg.nb


def lipschitz_reg_grad(model: Model, l, bg: BatchGraph, x, eps, h0=None):
    """Eq. (3) for layer l and its gradient with respect to that layer's weights (the layer's input held fixed).
    Both evaluations of the layer are differentiated: with u_v = (y_v - y'_v) / (nb ||y_v - y'_v||)
    (gas_row_distance_bwd) the output gradients are u and -u; each goes back through its own evaluation's stored
    activations (gas_relu_bwd, gas_linear_bwd_input for GIN's hidden layer, gas_linear_bwd_weight), and the two
    weight gradients are added.  Returns (sum of distances as a 1-element device tensor, nb, dW) with dW float32
    (a pair for GIN), scaled for the MEAN over the in-batch nodes."""
    dev, dt = x.device, x.dtype
    nb = bg.nb
    last = l == model.n_layers
    xp = torch.empty_like(x)
    B.gas_axpy(x, eps, xp, 1.0)
    outs = []
    for xx in (x, xp):
        z = torch.empty((nb, x.shape[1]), dtype=dt, device=dev)
        y = torch.empty((nb, model.out_width(l - 1)), dtype=dt, device=dev)
        h = None
        if model.op == "gcn":
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, xx, z)
            B.gas_linear(z, model.weights[l - 1], y, relu=not last)
        elif model.op == "gin":
            w1, w2 = model.weights[l - 1]
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, None, xx, z, diag=1.0 + model.gin_eps)
            h = torch.empty((nb, w1.shape[1]), dtype=dt, device=dev)
            B.gas_linear(z, w1, h, relu=True)            # stored: the backward pass reads the hidden activation
            B.gas_linear(h, w2, y, relu=not last)
        else:
            beta = gcnii_beta(l)
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, xx, z, s_agg=1.0 - model.alpha, r=h0, s_res=model.alpha)
            B.gas_linear(z, model.weights[l - 1], y, c_identity=1.0 - beta, c_weight=beta, relu=not last)
        outs.append((z, h, y))
    y, y2 = outs[0][2], outs[1][2]
    dist = torch.empty(nb, dtype=torch.float32, device=dev)
    total = torch.empty(1, dtype=torch.float32, device=dev)
    B.gas_row_distance(y, y2, dist, total)
    u = torch.empty_like(y)
    B.gas_row_distance_bwd(y, y2, u, 1.0 / max(1, nb))

    def weight_grad(zz, gg, c):
        dw = torch.empty((zz.shape[1], gg.shape[1]), dtype=torch.float32, device=dev)
        ws = torch.empty(max(1, B.gas_linear_bwd_weight_workspace(zz.shape[0], zz.shape[1], gg.shape[1])),
                         dtype=torch.uint8, device=dev)
        B.gas_linear_bwd_weight(zz, gg, dw, ws, c_weight=c)
        return dw

    def add(a, b):
        B.gas_axpy(a, b, a, 1.0)                         # float32 matrices, in place
        return a

    grads = None
    for sign, (z, h, yy) in zip((1.0, -1.0), outs):
        g = u
        if not last:
            g = torch.empty_like(u)
            B.gas_relu_bwd(u, yy, g)
        if model.op == "gin":
            w1, w2 = model.weights[l - 1]
            dw2 = weight_grad(h, g, sign)
            gh = torch.empty_like(h)
            B.gas_linear_bwd_input(g, w2, gh, mask=h)
            part = (weight_grad(z, gh, sign), dw2)
            grads = part if grads is None else tuple(add(a, b) for a, b in zip(grads, part))
        else:
            c = gcnii_beta(l) if model.op == "gcnii" else 1.0
            part = weight_grad(z, g, sign * c)
            grads = part if grads is None else add(grads, part)
    return total, nb, grads
