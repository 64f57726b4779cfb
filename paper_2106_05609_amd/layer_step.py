"""One GAS layer step on one mini-batch, as the benchmark times it and the
full-size parity tests check it: buffers are torch allocations, every
operation is a C-ABI call.

    gas_pull    halo rows of the mini-batch tensor <- history table l
    gas_spmm    aggregation over the batch subgraph
    gas_linear  dense transform + ReLU              (gas_mlp2 for GIN)
    gas_push    in-batch rows -> history table l+1
    gas_spmm_t  backward aggregation over the CSC copy (in-batch columns)

The in-place form of the same step is three calls: gas_spmm_hist (halo rows
read from the history table by the aggregation itself), gas_linear_push /
gas_mlp2_push (the transform stores each output row to its history slot as
well), gas_spmm_t.

Three kinds of layer (Algorithm 1 treats them differently):
  "first"   the input is exact for every node of V_b: ALL rows of the
            mini-batch tensor are gathered from the feature table (no history
            is read); the output is pushed; no backward aggregation (features
            take no gradient).  In place: only the in-batch rows are gathered,
            the aggregation reads the other rows from the feature table.
  "middle"  hidden width in and out, pull + push, backward aggregation.
  "last"    no ReLU, nothing is pushed; backward aggregation.
"""
import torch

from . import binding as B
from . import executor

NAMES = ["pull", "spmm", "linear", "push", "spmm_t"]
KINDS = ("first", "middle", "last")


class LayerStep:
    def __init__(self, cfg, g, sg, rng, device, kind="middle", bg=None, plan_options=None, tables_in=None, table_out=None,
                 pools=None):
        """cfg: benchmark configuration, g: graph, sg: batch subgraph (index tensors on `device`),
        rng: the seeded generator module for the synthetic tensors, bg: the batch's plans if already built.
        tables_in: tensors [N, F_in] allocated by the caller beforehand, every one of which is filled with the table
        the layer gathers from (place_table then keeps the one the gathers run fastest on); table_out: likewise a
        caller-allocated [N, F_out] tensor for the table the layer pushes to; pools: two caller-allocated byte
        buffers the two mini-batch tensors are carved from (same reason: memory allocated early)."""
        assert kind in KINDS
        self.cfg, self.sg, self.kind = cfg, sg, kind
        self.nb, self.nh, self.nv, self.nnz = sg.nb, sg.nh, sg.nv, sg.nnz
        self.nnz_t = int(sg.colptr[sg.nb].item())
        hidden = cfg.widths[-2]
        self.F_in = cfg.widths[0] if kind == "first" else hidden
        self.F_out = cfg.widths[-1] if kind == "last" else hidden
        self.F = self.F_in
        self.does_push = kind != "last"
        self.does_spmm_t = kind != "first"
        self.relu = kind != "last"
        dt = self.dt = cfg.dtype
        self.gin = cfg.op == "gin"
        if bg is None:
            bg = executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, sg.colptr, sg.row, max_F=max(cfg.widths),
                                     normalise=not self.gin, timed=True, plan_options=plan_options)
        self.bg = bg
        nb, nv, Fi, Fo = self.nb, self.nv, self.F_in, self.F_out
        # the table the rows outside the batch come from: the feature table for the first layer, else history l
        self.hist_in = rng.normal_matrix(cfg.seed, 10 if kind == "first" else 200, cfg.n, Fi, device, dt)
        self.candidates = []
        if tables_in:
            for t in tables_in:
                assert t.shape == self.hist_in.shape and t.dtype == dt
                B.gas_pull(self.hist_in, None, t, base=0, n=t.shape[0])       # the library's own contiguous copy
            self.candidates = list(tables_in)
            self.hist_in = tables_in[0]
        self.hist_out = None
        if self.does_push:
            self.hist_out = table_out.zero_() if table_out is not None else torch.zeros((cfg.n, Fo), dtype=dt, device=device)
        def carve(pool, rows, cols):
            if pool is None:
                return torch.empty((rows, cols), dtype=dt, device=device)
            nbytes = rows * cols * (4 if dt == torch.float32 else 2)
            assert pool.numel() >= nbytes, "pool too small for the mini-batch tensor"
            return pool[:nbytes].view(dt).view(rows, cols)

        px, pxn = pools if pools else (None, None)
        self.x = carve(px, nv, Fi)
        if kind == "first":
            self.x.zero_()                                               # every row arrives through gas_pull
        else:
            fresh = rng.normal_matrix(cfg.seed, 210, nb, Fi, device, dt)
            self.x[:nb] = fresh                                          # rows 0..nb-1: fresh in-batch embeddings
            self.x[nb:] = 0                                              # halo rows arrive through gas_pull
            del fresh
        self.z = torch.empty((nb, Fi), dtype=dt, device=device)
        self.x_next = carve(pxn, nv if self.does_push else nb, Fo)
        if self.does_spmm_t:
            self.gz = rng.normal_matrix(cfg.seed, 211, nb, Fi, device, dt)   # upstream gradient for the backward aggregation
            self.gx = torch.empty((nb, Fi), dtype=dt, device=device)
        else:
            self.gz = self.gx = None
        if self.gin:
            self.w1 = rng.glorot_uniform(cfg.seed, 102, Fi, cfg.gin_hidden, device, dt)
            self.w2 = rng.glorot_uniform(cfg.seed, 103, cfg.gin_hidden, Fo, device, dt)
        else:
            self.w = rng.glorot_uniform(cfg.seed, 101, Fi, Fo, device, dt)
        self.h0 = rng.normal_matrix(cfg.seed, 212, nb, Fi, device, dt) if cfg.op == "gcnii" else None
        self.beta = executor.gcnii_beta(2)
        self.diag = (1.0 + cfg.gin_eps) if self.gin else 0.0

    def place_table(self, candidates=3, reps=3):
        """Where the driver puts a table of tens of gigabytes changes the time of the random gathers from it by up to
        10 % (same data, same process, same box; see profiles/): a training run allocates its history tables once,
        so it can afford to try a few allocations and keep the best.  Times the in-place aggregation on every
        candidate table (the ones the caller allocated beforehand, else `candidates - 1` further copies allocated
        here), keeps the fastest and drops the others.  Returns the per-candidate times in ms (the kept one first)."""
        bg, nb = self.bg, self.nb

        def time_on(table):
            self.hist_in = table
            for _ in range(2):
                self._aggregate_in_place()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record()
            for _ in range(reps):
                self._aggregate_in_place()
            ev[1].record()
            torch.cuda.synchronize()
            return ev[0].elapsed_time(ev[1]) / reps

        if self.kind == "first":
            B.gas_pull(self.hist_in, bg.n_id[:nb], self.x[:nb])
        tables = list(self.candidates) if self.candidates else [self.hist_in]
        while len(tables) < candidates:
            t = torch.empty_like(self.hist_in)
            B.gas_pull(self.hist_in, None, t, base=0, n=t.shape[0])
            tables.append(t)
        times = [time_on(t) for t in tables]
        best = min(range(len(tables)), key=lambda i: times[i])
        self.hist_in = tables[best]
        self.candidates = [tables[best]]
        del tables
        torch.cuda.empty_cache()
        return [round(times[best], 4)] + [round(t, 4) for i, t in enumerate(times) if i != best]

    def _aggregate_in_place(self):
        cfg, bg, xb = self.cfg, self.bg, self.x[:self.nb]
        if self.gin:
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, None, xb, self.hist_in, self.z, diag=self.diag)
        elif cfg.op == "gcnii":
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, xb, self.hist_in, self.z, s_agg=1.0 - cfg.alpha,
                            r=self.h0, s_res=cfg.alpha)
        else:
            B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, xb, self.hist_in, self.z)

    def run(self, mark=None, skip_spmm_t=False, fused=False, only_spmm_t=False):
        """fused: the aggregation reads the rows outside the batch from their table itself
        (gas_spmm_hist) and the transform pushes its output rows (gas_linear_push /
        gas_mlp2_push); the push launch disappears, and the pull launch too (for the
        first layer it shrinks to the in-batch rows)."""
        cfg, bg, nb = self.cfg, self.bg, self.nb
        mark = mark or (lambda i: None)
        if only_spmm_t:                                  # profiling aid: the backward aggregation alone
            for i in range(5):
                mark(i)
            if self.does_spmm_t:
                B.gas_spmm_t(bg.plan_t, bg.colptr, bg.row, bg.val_t, self.gz, self.gx, diag=self.diag)
            mark(5)
            return
        mark(0)
        if self.kind == "first":
            n_pull = nb if fused else self.nv
            B.gas_pull(self.hist_in, bg.n_id[:n_pull], self.x[:n_pull])
        elif not fused:
            B.gas_pull(self.hist_in, bg.n_id[nb:], self.x[nb:])
        mark(1)
        if fused:
            self._aggregate_in_place()
        elif self.gin:
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, None, self.x, self.z, diag=self.diag)
        elif cfg.op == "gcnii":
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, self.x, self.z, s_agg=1.0 - cfg.alpha, r=self.h0,
                       s_res=cfg.alpha)
        else:
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, self.x, self.z)
        mark(2)
        self.transform(push=fused and self.does_push)
        mark(3)
        if not fused and self.does_push:
            B.gas_push(self.x_next[:nb], bg.n_id[:nb], self.hist_out)
        mark(4)
        if self.does_spmm_t and not skip_spmm_t:
            B.gas_spmm_t(bg.plan_t, bg.colptr, bg.row, bg.val_t, self.gz, self.gx, diag=self.diag)
        mark(5)

    def transform(self, push):
        """Dense transform of the aggregated rows into the next mini-batch tensor; with push, each row
        also goes to its slot of the next history table in the same call."""
        cfg, nb = self.cfg, self.nb
        y, idx = self.x_next[:nb], self.bg.n_id[:nb]
        if self.gin:
            if push:
                B.gas_mlp2_push(self.z, self.w1, self.w2, y, idx, self.hist_out, relu_out=self.relu)
            else:
                B.gas_mlp2(self.z, self.w1, self.w2, y, relu_out=self.relu)
            return
        gcnii = cfg.op == "gcnii" and self.F_in == self.F_out
        c_id, c_w = (1.0 - self.beta, self.beta) if gcnii else (0.0, 1.0)
        if push:
            B.gas_linear_push(self.z, self.w, y, idx, self.hist_out, c_identity=c_id, c_weight=c_w, relu=self.relu)
        else:
            B.gas_linear(self.z, self.w, y, c_identity=c_id, c_weight=c_w, relu=self.relu)

    def algorithmic_bytes(self):
        """Bytes each call must move at least once (indices and values once, every
        needed feature row once, every output row once)."""
        Fi, Fo, s = self.F_in, self.F_out, (4 if self.dt == torch.float32 else 2)
        nb, nh, nv, nnz, nnz_t = self.nb, self.nh, self.nv, self.nnz, self.nnz_t
        vb = 0 if self.gin else 4
        hid = self.cfg.gin_hidden
        n_pull = nv if self.kind == "first" else nh
        return {
            "pull": n_pull * (2 * Fi * s + 4),
            "pull_in_place": nb * (2 * Fi * s + 4) if self.kind == "first" else 0,
            "spmm": nnz * (4 + vb) + (nb + 1) * 4 + nv * Fi * s + nb * Fi * s,
            "linear": nb * (Fi + Fo) * s + ((Fi * hid + hid * Fo) if self.gin else Fi * Fo) * s,
            "push": nb * (2 * Fo * s + 4) if self.does_push else 0,
            "push_in_epilogue": nb * (Fo * s + 4) if self.does_push else 0,   # the transform holds the row: only the store is left
            "spmm_t": (nnz_t * (4 + vb) + (nb + 1) * 4 + nb * Fi * s + nb * Fi * s) if self.does_spmm_t else 0,
            "spmm_no_reuse": nnz * (4 + vb) + (nb + 1) * 4 + nnz * Fi * s + nb * Fi * s,
        }

    def flops(self):
        Fi, Fo, hid = self.F_in, self.F_out, self.cfg.gin_hidden
        return 2.0 * self.nb * ((Fi * hid + hid * Fo) if self.gin else Fi * Fo)
