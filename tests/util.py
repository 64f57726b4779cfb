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
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / (den if den > 0 else 1.0))


def oracle_model(wl) -> omodel.Model:
    cfg = wl.cfg
    if cfg.op == "gin":
        ws = [(to_np(a), to_np(b)) for a, b in wl.weights]
    else:
        ws = [to_np(w) for w in wl.weights]
    return omodel.Model(cfg.op, ws, None if wl.w_in is None else to_np(wl.w_in), cfg.alpha, cfg.gin_eps,
                        omodel.gcnii_betas(len(ws)) if cfg.op == "gcnii" else [])
