"""Pins for the oracle's whole-model backward passes of PNA and GAT (CPU only): every weight gradient of a
three-layer model on a proper mini-batch (halo rows read from constant histories) against float64 autograd on a
dense re-statement of the same layers, written with masked matrices instead of index lists."""
import numpy as np
import pytest
import torch

from gas_inputs import rng
from oracle import model as omodel
from tests.util import to_np, f64
from tests.test_oracle_gas import _workload, _sub

T = lambda a: torch.from_numpy(f64(a))


def _mask(rp, cl, nb, nv):
    m = torch.zeros((nb, nv), dtype=torch.bool)
    for v in range(nb):
        m[v, cl[rp[v]:rp[v + 1]]] = True
    return m


def _close(got, want, tol, floor=0.0):
    return np.abs(f64(got) - want).max() <= tol * max(np.abs(want).max(), floor)


def test_pna_model_gradients_match_float64_autograd():
    wl = _workload("gin", n=300, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[1])
    nb, nv = sg.nb, sg.nv
    assert sg.nh > 0
    f, f1, L = 6, 5, 3
    x = to_np(rng.normal_matrix(61, 1100, g.n, f))
    ws = [(to_np(rng.glorot_uniform(61, 1101 + 2 * l, 2 * f, f1)), to_np(rng.glorot_uniform(61, 1102 + 2 * l, f + 9 * f1, f)))
          for l in range(L)]
    hist = [to_np(rng.normal_matrix(61, 1110 + l, g.n, f)) for l in range(L - 1)]
    gout = to_np(rng.normal_matrix(61, 1120, nb, f))
    delta = float(np.log(to_np(g.deg).astype(np.float64) + 1.0).mean())
    y, grads = omodel.pna_batch_train(ws, delta, n_id, rp, cl, nb, x, [h.copy() for h in hist], gout, do_push=False)
    assert np.array_equal(y, omodel.pna_batch_forward(ws, delta, n_id, rp, cl, nb, x, [h.copy() for h in hist], do_push=False))
    # dense float64 model
    a = _mask(rp, cl, nb, nv)
    d = a.sum(dim=1).double()
    has = (d > 0)[:, None]
    s = (torch.log(d + 1.0) / delta)[:, None]
    tw = [(T(w1).requires_grad_(), T(w2).requires_grad_()) for w1, w2 in ws]
    xt = T(x)[torch.from_numpy(n_id.astype(np.int64))]
    yt = None
    for l in range(L):
        w1, w2 = tw[l]
        p, q = xt @ w1[f:], xt[:nb] @ w1[:f]
        inf = torch.tensor(float("inf"), dtype=torch.float64)
        three = [(a.double() @ p) / d.clamp(min=1)[:, None],
                 torch.where(a[:, :, None], p[None], inf).amin(dim=1), torch.where(a[:, :, None], p[None], -inf).amax(dim=1)]
        agg = [torch.where(has, t + q, torch.zeros_like(q)) for t in three]
        a9 = torch.cat(agg + [s * t for t in agg] + [torch.where(has, t / s.clamp(min=1e-30), torch.zeros_like(t)) for t in agg],
                       dim=1)
        yt = torch.cat([xt[:nb], a9], dim=1) @ w2
        if l < L - 1:
            yt = torch.relu(yt)
            xt = torch.cat([yt, T(hist[l])[torch.from_numpy(n_id[nb:].astype(np.int64))]], dim=0)
    assert _close(y, yt.detach().numpy(), 5e-6)
    (yt * T(gout)).sum().backward()
    for l in range(L):
        assert _close(grads[l][0], tw[l][0].grad.numpy(), 1e-5), l
        assert _close(grads[l][1], tw[l][1].grad.numpy(), 1e-5), l
    # the neighbour half of W1 takes gradient through the halo rows too: without them the result differs
    assert np.abs(tw[0][0].grad.numpy()[f:]).max() > 0


@pytest.mark.parametrize("heads", [1, 3])
def test_gat_model_gradients_match_float64_autograd(heads):
    wl = _workload("gcn", n=300, layers=2, f=8)
    g = wl.graph
    sg, n_id, rp, cl = _sub(wl, wl.batches[2])
    nb, nv = sg.nb, sg.nv
    assert sg.nh > 0
    f, L, slope = 6, 3, 0.2
    x = to_np(rng.normal_matrix(62, 1200, g.n, f))
    ws = [(to_np(rng.glorot_uniform(62, 1201 + 3 * l, f, f)), to_np(rng.normal(62, 1202 + 3 * l, 0, f)) * 0.3,
           to_np(rng.normal(62, 1203 + 3 * l, 0, f)) * 0.3) for l in range(L)]
    hist = [to_np(rng.normal_matrix(62, 1210 + l, g.n, f)) for l in range(L - 1)]
    gout = to_np(rng.normal_matrix(62, 1220, nb, f))
    y, grads = omodel.gat_batch_train(ws, n_id, rp, cl, nb, x, [h.copy() for h in hist], gout, slope, do_push=False,
                                      heads=heads)
    assert np.array_equal(y, omodel.gat_batch_forward(ws, n_id, rp, cl, nb, x, [h.copy() for h in hist], slope,
                                                      do_push=False, heads=heads))
    mask = _mask(rp, cl, nb, nv)
    tw = [tuple(T(t).requires_grad_() for t in w) for w in ws]
    xt = T(x)[torch.from_numpy(n_id.astype(np.int64))]
    fh = f // heads
    yt = None
    for l in range(L):
        w, ad, asr = tw[l]
        p = xt @ w
        outs = []
        for h in range(heads):
            c = slice(h * fh, (h + 1) * fh)
            e = torch.nn.functional.leaky_relu((p[:nb, c] @ ad[c])[:, None] + (p[:, c] @ asr[c])[None, :], slope)
            outs.append(torch.softmax(e.masked_fill(~mask, float("-inf")), dim=1) @ p[:, c])
        yt = torch.cat(outs, dim=1)
        if l < L - 1:
            yt = torch.relu(yt)
            xt = torch.cat([yt, T(hist[l])[torch.from_numpy(n_id[nb:].astype(np.int64))]], dim=0)
    assert _close(y, yt.detach().numpy(), 5e-6)
    (yt * T(gout)).sum().backward()
    for l in range(L):
        scale = max(np.abs(tw[l][1].grad.numpy()).max(), np.abs(tw[l][2].grad.numpy()).max())
        assert _close(grads[l][0], tw[l][0].grad.numpy(), 1e-5), l
        assert _close(grads[l][1], tw[l][1].grad.numpy(), 1e-5, floor=scale), l
        assert _close(grads[l][2], tw[l][2].grad.numpy(), 1e-5, floor=scale), l
