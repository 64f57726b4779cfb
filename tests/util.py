"""Helpers shared by the tests: torch <-> numpy views and the error measure."""
import numpy as np
import torch

from oracle import model as omodel
from oracle import ops as oops


def to_np(t: torch.Tensor) -> np.ndarray:
    """CPU numpy view; bf16 tensors become uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def f64(a) -> np.ndarray:
    if isinstance(a, torch.Tensor):
        a = to_np(a)
    return oops.to_f64(a) if a.dtype in (np.uint16, np.float32) else np.asarray(a, dtype=np.float64)


def max_rel_err(a, b) -> float:
    """max|a-b| / max|b| over a whole tensor, b the reference."""
    a, b = f64(a), f64(b)
    if a.size == 0:
        return 0.0
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / (den if den > 0 else 1.0))


def row_rel_err(a, b, floor: float = 1e-3, scale=None) -> float:
    """Worst row of a node-by-feature matrix, each row measured on its own scale:
    max_v  max_j|a_vj - b_vj| / max(max_j|b_vj|, floor * max|b|),  b the reference.
    A pooled maximum lets the rows of a few hub nodes set the scale for everybody; on a
    power-law batch with sum aggregation a light row could then lose a whole neighbour
    unnoticed.  The floor keeps rows that are (nearly) all zero, e.g. after a ReLU, from
    dividing rounding noise by nothing.  `scale` (one positive number per row) replaces the row's own
    maximum where that is a poor yardstick: a narrow transform output after a ReLU can be far smaller
    than the products that were summed for it, and rounding errors are relative to those."""
    a, b = f64(a), f64(b)
    if a.size == 0:
        return 0.0
    if a.ndim != 2:
        return max_rel_err(a, b)
    den = np.abs(b).max()
    den = den if den > 0 else 1.0
    own = np.abs(b).max(axis=1) if scale is None else np.maximum(np.abs(b).max(axis=1), np.asarray(scale, dtype=np.float64))
    scale = np.maximum(own, floor * den)
    return float((np.abs(a - b).max(axis=1) / scale).max())


WORST_ROW_ERR = {}      # test id -> worst per-row error it saw (printed at the end of a pytest session)


def node_rel_err(a, b, scale=None) -> float:
    """The gate for every matrix with one row per node (aggregations, transforms, model outputs,
    histories): the larger of the pooled error and the worst row's own relative error."""
    import os
    pooled, rows = max_rel_err(a, b), row_rel_err(a, b, scale=scale)
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0]
    WORST_ROW_ERR[test] = max(WORST_ROW_ERR.get(test, 0.0), rows)
    return max(pooled, rows)


def oracle_model(wl) -> omodel.Model:
    cfg = wl.cfg
    if cfg.op == "gin":
        ws = [(to_np(a), to_np(b)) for a, b in wl.weights]
    else:
        ws = [to_np(w) for w in wl.weights]
    return omodel.Model(cfg.op, ws, None if wl.w_in is None else to_np(wl.w_in), cfg.alpha, cfg.gin_eps,
                        omodel.gcnii_betas(len(ws)) if cfg.op == "gcnii" else [])
