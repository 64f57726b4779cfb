"""One middle-layer GAS step on one mini-batch, as the benchmark times it and
the full-size parity tests check it: buffers are torch allocations, every
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
"""
import torch

from . import binding as B
from . import executor

NAMES = ["pull", "spmm", "linear", "push", "spmm_t"]


class LayerStep:
    def __init__(self, cfg, g, sg, rng, device):
        """cfg: benchmark configuration, g: graph, sg: batch subgraph (index tensors on `device`),
        rng: the seeded generator module for the synthetic tensors."""
        self.cfg, self.sg = cfg, sg
        self.nb, self.nh, self.nv, self.nnz = sg.nb, sg.nh, sg.nv, sg.nnz
        self.nnz_t = int(sg.colptr[sg.nb].item())
        F = self.F = cfg.widths[-2]
        dt = self.dt = cfg.dtype
        self.gin = cfg.op == "gin"
        self.bg = executor.BatchGraph(sg.nb, sg.n_id, sg.rowptr, sg.col, g.deg, sg.colptr, sg.row, max_F=F,
                                      normalise=not self.gin)
        nb, nv = self.nb, self.nv
        self.hist_in = rng.normal_matrix(cfg.seed, 200, cfg.n, F, device, dt)
        self.hist_out = torch.zeros((cfg.n, F), dtype=dt, device=device)
        self.x = rng.normal_matrix(cfg.seed, 210, nv, F, device, dt)     # rows 0..nb-1: fresh in-batch embeddings
        self.x[nb:] = 0                                                  # halo rows arrive through gas_pull
        self.z = torch.empty((nb, F), dtype=dt, device=device)
        self.x_next = torch.empty((nv, F), dtype=dt, device=device)
        self.gz = rng.normal_matrix(cfg.seed, 211, nb, F, device, dt)    # upstream gradient for the backward aggregation
        self.gx = torch.empty((nb, F), dtype=dt, device=device)
        if self.gin:
            self.w1 = rng.glorot_uniform(cfg.seed, 102, F, cfg.gin_hidden, device, dt)
            self.w2 = rng.glorot_uniform(cfg.seed, 103, cfg.gin_hidden, F, device, dt)
        else:
            self.w = rng.glorot_uniform(cfg.seed, 101, F, F, device, dt)
        self.h0 = rng.normal_matrix(cfg.seed, 212, nb, F, device, dt) if cfg.op == "gcnii" else None
        self.beta = executor.gcnii_beta(2)
        self.diag = (1.0 + cfg.gin_eps) if self.gin else 0.0

    def run(self, mark=None, skip_spmm_t=False, fused=False):
        """fused: the aggregation reads the halo rows from the history table itself
        (gas_spmm_hist) and the transform pushes its output rows (gas_linear_push /
        gas_mlp2_push); the pull and push launches disappear."""
        cfg, bg, nb = self.cfg, self.bg, self.nb
        mark = mark or (lambda i: None)
        mark(0)
        if not fused:
            B.gas_pull(self.hist_in, bg.n_id[nb:], self.x[nb:])
        mark(1)
        if fused:
            xb = self.x[:nb]
            if self.gin:
                B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, None, xb, self.hist_in, self.z, diag=self.diag)
            elif cfg.op == "gcnii":
                B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, xb, self.hist_in, self.z, s_agg=1.0 - cfg.alpha,
                                r=self.h0, s_res=cfg.alpha)
            else:
                B.gas_spmm_hist(bg.plan, bg.rowptr, bg.src, bg.val, xb, self.hist_in, self.z)
        elif self.gin:
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, None, self.x, self.z, diag=self.diag)
        elif cfg.op == "gcnii":
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, self.x, self.z, s_agg=1.0 - cfg.alpha, r=self.h0,
                       s_res=cfg.alpha)
        else:
            B.gas_spmm(bg.plan, bg.rowptr, bg.col, bg.val, self.x, self.z)
        mark(2)
        self.transform(push=fused)
        mark(3)
        if not fused:
            B.gas_push(self.x_next[:nb], bg.n_id[:nb], self.hist_out)
        mark(4)
        if not skip_spmm_t:
            B.gas_spmm_t(bg.plan_t, bg.colptr, bg.row, bg.val_t, self.gz, self.gx, diag=self.diag)
        mark(5)

    def transform(self, push):
        """Dense transform of the aggregated rows into the next mini-batch tensor; with push, each row
        also goes to its slot of the next history table in the same call."""
        cfg, nb = self.cfg, self.nb
        y, idx = self.x_next[:nb], self.bg.n_id[:nb]
        if self.gin:
            if push:
                B.gas_mlp2_push(self.z, self.w1, self.w2, y, idx, self.hist_out, relu_out=True)
            else:
                B.gas_mlp2(self.z, self.w1, self.w2, y, relu_out=True)
            return
        c_id, c_w = (1.0 - self.beta, self.beta) if cfg.op == "gcnii" else (0.0, 1.0)
        if push:
            B.gas_linear_push(self.z, self.w, y, idx, self.hist_out, c_identity=c_id, c_weight=c_w, relu=True)
        else:
            B.gas_linear(self.z, self.w, y, c_identity=c_id, c_weight=c_w, relu=True)

    def algorithmic_bytes(self):
        """Bytes each call must move at least once (indices and values once, every
        needed feature row once, every output row once)."""
        F, s = self.F, (4 if self.dt == torch.float32 else 2)
        nb, nh, nv, nnz, nnz_t = self.nb, self.nh, self.nv, self.nnz, self.nnz_t
        vb = 0 if self.gin else 4
        return {
            "pull": nh * (2 * F * s + 4),
            "spmm": nnz * (4 + vb) + (nb + 1) * 4 + nv * F * s + nb * F * s,
            "linear": nb * 2 * F * s + F * F * s * (2 if self.gin else 1),
            "push": nb * (2 * F * s + 4),
            "push_in_epilogue": nb * (F * s + 4),       # the transform already holds the row: only the store is left
            "spmm_t": nnz_t * (4 + vb) + (nb + 1) * 4 + nb * F * s + nb * F * s,
            "spmm_no_reuse": nnz * (4 + vb) + (nb + 1) * 4 + nnz * F * s + nb * F * s,
        }

    def fused_algorithmic_bytes(self):
        """The fused aggregation reads the same rows once (in-batch from X, halo
        from the history table) and writes Z; no halo copy is written or re-read."""
        return self.algorithmic_bytes()["spmm"]
