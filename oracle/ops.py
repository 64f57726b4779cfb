"""ctypes wrappers around the oracle's C functions (test infrastructure).

Arrays are numpy: float32 for fp32 buffers, uint16 bit patterns for bf16
buffers, int32 for indices.  Each wrapper allocates its output and returns it;
`push` updates the history in place.  See gas_oracle.c for the definitions and
the passages of the paper they follow.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None

F32, BF16 = 0, 1


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.oracle_round_bf16.restype = C.c_uint16
        _lib.oracle_round_bf16.argtypes = [C.c_double]
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle buffers are float32 or uint16 (bf16 bits), got {a.dtype}")


def _np_dtype(dt: int):
    return np.float32 if dt == F32 else np.uint16


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _rows(a: np.ndarray):
    """(array, leading dimension in elements) of a 2-D row-major array."""
    assert a.ndim == 2 and a.strides[1] == a.itemsize, "need row-major 2-D"
    return a, a.strides[0] // a.itemsize


def _i32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int32
    return a


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def round_bf16(x: float) -> int:
    return int(lib().oracle_round_bf16(float(x)))


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def pull(hist: np.ndarray, idx: np.ndarray) -> np.ndarray:
    hist, ld = _rows(hist)
    idx = _i32(idx)
    out = np.empty((idx.size, hist.shape[1]), dtype=hist.dtype)
    lib().oracle_pull(_p(hist), C.c_int64(ld), _p(idx), C.c_int64(idx.size), C.c_int32(hist.shape[1]),
                      C.c_int32(hist.itemsize), _p(out), C.c_int64(hist.shape[1]))
    return out


def push(src: np.ndarray, idx: np.ndarray, hist: np.ndarray) -> None:
    src, lds = _rows(src)
    hist, ldh = _rows(hist)
    idx = _i32(idx)
    assert src.dtype == hist.dtype and src.shape == (idx.size, hist.shape[1])
    lib().oracle_push(_p(src), C.c_int64(lds), _p(idx), C.c_int64(idx.size), C.c_int32(hist.shape[1]),
                      C.c_int32(hist.itemsize), _p(hist), C.c_int64(ldh))


def gcn_norm(ptr, ind, n_id, deg) -> np.ndarray:
    ptr, ind, n_id, deg = _i32(ptr), _i32(ind), _i32(n_id), _i32(deg)
    val = np.empty(ind.size, dtype=np.float32)
    lib().oracle_gcn_norm(_p(ptr), _p(ind), C.c_int64(ptr.size - 1), _p(n_id), _p(deg), _p(val))
    return val


def spmm(rowptr, col, val, x, diag=0.0, s_agg=1.0, r=None, s_res=0.0, out_dt=None) -> np.ndarray:
    rowptr, col = _i32(rowptr), _i32(col)
    x, ldx = _rows(x)
    n_rows, f = rowptr.size - 1, x.shape[1]
    if val is not None:
        val = np.ascontiguousarray(val)
        assert val.dtype == np.float32 and val.size == col.size
    ldr = 0
    if r is not None:
        r, ldr = _rows(r)
        assert r.dtype == x.dtype and r.shape[1] == f and r.shape[0] >= n_rows
    out_dt = _dt(x) if out_dt is None else out_dt
    z = np.empty((n_rows, f), dtype=_np_dtype(out_dt))
    lib().oracle_spmm(_p(rowptr), _p(col), _p(val), C.c_double(diag), _p(x), C.c_int64(ldx), C.c_int(_dt(x)),
                      C.c_int32(f), C.c_double(s_agg), _p(r), C.c_int64(ldr), C.c_double(s_res),
                      _p(z), C.c_int64(f), C.c_int(out_dt), C.c_int64(n_rows))
    return z


def spmm_t(rowptr, col, val, g, n_out, diag=0.0, out_dt=None, s_agg=1.0) -> np.ndarray:
    rowptr, col = _i32(rowptr), _i32(col)
    g, ldg = _rows(g)
    n_rows, f = rowptr.size - 1, g.shape[1]
    assert g.shape[0] == n_rows
    if val is not None:
        val = np.ascontiguousarray(val)
        assert val.dtype == np.float32
    out_dt = _dt(g) if out_dt is None else out_dt
    gx = np.empty((n_out, f), dtype=_np_dtype(out_dt))
    lib().oracle_spmm_t(_p(rowptr), _p(col), _p(val), C.c_double(diag), C.c_double(s_agg), _p(g), C.c_int64(ldg), C.c_int(_dt(g)),
                        C.c_int32(f), C.c_int64(n_rows), C.c_int64(n_out), _p(gx), C.c_int64(f), C.c_int(out_dt))
    return gx


def linear(z, w, bias=None, c_identity=0.0, c_weight=1.0, relu=False, out_dt=None) -> np.ndarray:
    z, ldz = _rows(z)
    w = np.ascontiguousarray(w)
    assert w.dtype == z.dtype and w.shape[0] == z.shape[1]
    if c_identity != 0.0:
        assert w.shape[0] == w.shape[1]
    out_dt = _dt(z) if out_dt is None else out_dt
    y = np.empty((z.shape[0], w.shape[1]), dtype=_np_dtype(out_dt))
    lib().oracle_linear(_p(z), C.c_int64(ldz), C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _p(w),
                        C.c_int32(w.shape[1]), _p(bias), C.c_int(_dt(z)), C.c_double(c_identity),
                        C.c_double(c_weight), C.c_int(int(relu)), _p(y), C.c_int64(w.shape[1]), C.c_int(out_dt))
    return y


def mlp2(z, w1, w2, b1=None, b2=None, relu_out=False, out_dt=None) -> np.ndarray:
    z, ldz = _rows(z)
    w1, w2 = np.ascontiguousarray(w1), np.ascontiguousarray(w2)
    assert w1.dtype == z.dtype == w2.dtype and w1.shape[0] == z.shape[1] and w2.shape[0] == w1.shape[1]
    out_dt = _dt(z) if out_dt is None else out_dt
    y = np.empty((z.shape[0], w2.shape[1]), dtype=_np_dtype(out_dt))
    lib().oracle_mlp2(_p(z), C.c_int64(ldz), C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _p(w1),
                      C.c_int32(w1.shape[1]), _p(b1), _p(w2), C.c_int32(w2.shape[1]), _p(b2), C.c_int(_dt(z)),
                      C.c_int(int(relu_out)), _p(y), C.c_int64(w2.shape[1]), C.c_int(out_dt))
    return y


def relu_bwd(gy, y) -> np.ndarray:
    gy, ldgy = _rows(gy)
    y, ldy = _rows(y)
    assert gy.shape == y.shape and gy.dtype == y.dtype
    gp = np.empty(gy.shape, dtype=gy.dtype)
    lib().oracle_relu_bwd(_p(gy), C.c_int64(ldgy), _p(y), C.c_int64(ldy), C.c_int64(gy.shape[0]), C.c_int32(gy.shape[1]),
                          C.c_int(_dt(gy)), _p(gp), C.c_int64(gy.shape[1]))
    return gp


def linear_bwd_input(gp, w, c_identity=0.0, c_weight=1.0, mask=None) -> np.ndarray:
    """gp [n, F_out], w [F_in, F_out] -> gz [n, F_in]."""
    gp, ldgp = _rows(gp)
    w = np.ascontiguousarray(w)
    assert w.dtype == gp.dtype and w.shape[1] == gp.shape[1]
    ldm = 0
    if mask is not None:
        mask, ldm = _rows(mask)
        assert mask.dtype == gp.dtype and mask.shape == (gp.shape[0], w.shape[0])
    gz = np.empty((gp.shape[0], w.shape[0]), dtype=gp.dtype)
    lib().oracle_linear_bwd_input(_p(gp), C.c_int64(ldgp), C.c_int64(gp.shape[0]), C.c_int32(gp.shape[1]), _p(w),
                                  C.c_int32(w.shape[0]), C.c_int(_dt(gp)), C.c_double(c_identity), C.c_double(c_weight),
                                  _p(mask), C.c_int64(ldm), _p(gz), C.c_int64(w.shape[0]))
    return gz


def linear_bwd_weight(z, gp, c_weight=1.0) -> np.ndarray:
    """z [n, F_in], gp [n, F_out] -> dW [F_in, F_out] float32."""
    z, ldz = _rows(z)
    gp, ldgp = _rows(gp)
    assert z.dtype == gp.dtype and z.shape[0] == gp.shape[0]
    dw = np.empty((z.shape[1], gp.shape[1]), dtype=np.float32)
    lib().oracle_linear_bwd_weight(_p(z), C.c_int64(ldz), _p(gp), C.c_int64(ldgp), C.c_int64(z.shape[0]),
                                   C.c_int32(z.shape[1]), C.c_int32(gp.shape[1]), C.c_int(_dt(z)), C.c_double(c_weight),
                                   _p(dw))
    return dw


def softmax_xent(a, labels, scale=1.0):
    """a [n, C] logits, labels int32[n] (< 0: row ignored) -> (loss_rows float32[n], loss_sum float, grad [n, C])."""
    a, lda = _rows(a)
    labels = _i32(labels)
    assert labels.size == a.shape[0]
    loss_rows = np.empty(a.shape[0], dtype=np.float32)
    total = C.c_double(0.0)
    g = np.empty(a.shape, dtype=a.dtype)
    lib().oracle_softmax_xent(_p(a), C.c_int64(lda), C.c_int64(a.shape[0]), C.c_int32(a.shape[1]), C.c_int(_dt(a)),
                              _p(labels), C.c_double(scale), _p(loss_rows), C.byref(total), _p(g),
                              C.c_int64(a.shape[1]))
    return loss_rows, float(total.value), g


def sgd_step(w, dw, lr, weight_decay=0.0) -> None:
    """In place: w <- w - lr * (dw + weight_decay * w); w contiguous in its storage type, dw float32."""
    assert w.flags.c_contiguous and dw.flags.c_contiguous and dw.dtype == np.float32 and dw.size == w.size
    lib().oracle_sgd_step(_p(w), C.c_int64(w.size), C.c_int(_dt(w)), _p(dw), C.c_double(lr), C.c_double(weight_decay))


def sq_norm(dw) -> float:
    """Sum of the squares of a gradient (plain definition, float64)."""
    return float(np.sum(np.asarray(dw, dtype=np.float64) ** 2))


def clip_scale(sq_norms, max_norm) -> float:
    """Gradient clipping by the global L2 norm (paper, Section 3: clipping keeps the parameters, and with them the
    histories, from changing too fast): every gradient is multiplied by min(1, max_norm / (||g|| + 1e-6)), where
    ||g|| is the norm of all gradients taken together."""
    total = float(np.sqrt(np.sum(np.asarray(sq_norms, dtype=np.float64))))
    return min(1.0, max_norm / (total + 1e-6))


def pna_aggregate(rowptr, col, x, delta, add=None) -> np.ndarray:
    """[n_rows, 9F]: scalers [1, s, 1/s] (x) aggregators [mean, min, max] over the neighbours, s = log(d+1)/delta."""
    rowptr, col = _i32(rowptr), _i32(col)
    x, ldx = _rows(x)
    n_rows, f = rowptr.size - 1, x.shape[1]
    ldadd = 0
    if add is not None:
        add, ldadd = _rows(add)
        assert add.dtype == x.dtype and add.shape == (n_rows, f)
    out = np.empty((n_rows, 9 * f), dtype=x.dtype)
    lib().oracle_pna_aggregate(_p(rowptr), _p(col), C.c_int64(n_rows), _p(x), C.c_int64(ldx), C.c_int(_dt(x)),
                               C.c_int32(f), _p(add), C.c_int64(ldadd), C.c_double(delta), _p(out), C.c_int64(9 * f))
    return out


def pna_aggregate_bwd(rowptr, col, x, delta, g, n_out, want_add=True):
    """Backward of pna_aggregate: (GX [n_out, F], Gadd [n_rows, F] or None) from G [n_rows, 9F]."""
    rowptr, col = _i32(rowptr), _i32(col)
    x, ldx = _rows(x)
    g, ldg = _rows(g)
    n_rows, f = rowptr.size - 1, x.shape[1]
    assert g.dtype == x.dtype and g.shape == (n_rows, 9 * f)
    gx = np.empty((n_out, f), dtype=x.dtype)
    gadd = np.empty((n_rows, f), dtype=x.dtype) if want_add else None
    lib().oracle_pna_aggregate_bwd(_p(rowptr), _p(col), C.c_int64(n_rows), C.c_int64(n_out), _p(x), C.c_int64(ldx),
                                   C.c_int(_dt(x)), C.c_int32(f), C.c_double(delta), _p(g), C.c_int64(ldg), _p(gx),
                                   C.c_int64(f), _p(gadd), C.c_int64(f))
    return gx, gadd


def gat_aggregate_bwd(rowptr, col, p, a_dst, a_src, gz, n_out, negative_slope=0.2):
    """Backward of gat_aggregate (gz: gradient at the weighted sum before any activation):
    (GP [n_out, F] in p's type, Ga_dst float32[F], Ga_src float32[F])."""
    rowptr, col = _i32(rowptr), _i32(col)
    p, ldp = _rows(p)
    gz, ldgz = _rows(gz)
    n_rows, f = rowptr.size - 1, p.shape[1]
    a_dst, a_src = np.ascontiguousarray(a_dst), np.ascontiguousarray(a_src)
    assert a_dst.dtype == p.dtype == a_src.dtype == gz.dtype and gz.shape == (n_rows, f)
    gp = np.empty((n_out, f), dtype=p.dtype)
    gd, gs = np.empty(f, dtype=np.float32), np.empty(f, dtype=np.float32)
    lib().oracle_gat_aggregate_bwd(_p(rowptr), _p(col), C.c_int64(n_rows), C.c_int64(n_out), _p(p), C.c_int64(ldp),
                                   C.c_int(_dt(p)), C.c_int32(f), _p(a_dst), _p(a_src), C.c_double(negative_slope),
                                   _p(gz), C.c_int64(ldgz), _p(gp), C.c_int64(f), _p(gd), _p(gs))
    return gp, gd, gs


def gat_aggregate(rowptr, col, p, a_dst, a_src, negative_slope=0.2, relu=False) -> np.ndarray:
    """Z[v] = sum_k softmax_k(LeakyReLU(a_dst.P[v] + a_src.P[col k])) P[col k] over the entries of row v."""
    rowptr, col = _i32(rowptr), _i32(col)
    p, ldp = _rows(p)
    n_rows, f = rowptr.size - 1, p.shape[1]
    a_dst, a_src = np.ascontiguousarray(a_dst), np.ascontiguousarray(a_src)
    assert a_dst.dtype == p.dtype == a_src.dtype and a_dst.size == f == a_src.size
    z = np.empty((n_rows, f), dtype=p.dtype)
    lib().oracle_gat_aggregate(_p(rowptr), _p(col), C.c_int64(n_rows), _p(p), C.c_int64(ldp), C.c_int(_dt(p)),
                               C.c_int32(f), _p(a_dst), _p(a_src), C.c_double(negative_slope), C.c_int(int(relu)), _p(z), C.c_int64(f))
    return z


def axpy(x, e, alpha) -> np.ndarray:
    """x + alpha * e, row-major [n, F], rounded once to the storage type."""
    x, ldx = _rows(x)
    e, lde = _rows(e)
    assert x.shape == e.shape and x.dtype == e.dtype
    y = np.empty(x.shape, dtype=x.dtype)
    lib().oracle_axpy(_p(x), C.c_int64(ldx), _p(e), C.c_int64(lde), C.c_int64(x.shape[0]), C.c_int32(x.shape[1]),
                      C.c_int(_dt(x)), C.c_double(alpha), _p(y), C.c_int64(x.shape[1]))
    return y


def row_distance(a, b):
    """(dist float32[n], sum of dist): dist[i] = ||a[i] - b[i]||_2."""
    a, lda = _rows(a)
    b, ldb = _rows(b)
    assert a.shape == b.shape and a.dtype == b.dtype
    dist = np.empty(a.shape[0], dtype=np.float32)
    total = C.c_double(0.0)
    lib().oracle_row_distance(_p(a), C.c_int64(lda), _p(b), C.c_int64(ldb), C.c_int64(a.shape[0]), C.c_int32(a.shape[1]),
                              C.c_int(_dt(a)), _p(dist), C.byref(total))
    return dist, float(total.value)


def row_dot(a, b):
    """(dot float32[n], their sum): dot[i] = sum_f a[i, f] * b[i, f], in float64."""
    a64, b64 = to_f64(np.asarray(a)), to_f64(np.asarray(b))
    assert a64.shape == b64.shape
    rows = (a64 * b64).sum(axis=1)
    return rows.astype(np.float32), float(rows.sum())


def row_distance_bwd(a, b, scale=1.0) -> np.ndarray:
    """Gradient of scale * sum_i ||a[i] - b[i]||_2 with respect to a (that with respect to b is its negative):
    row i is scale * (a[i] - b[i]) / ||a[i] - b[i]||_2, and zero where the two rows are equal.  In a's type."""
    a, lda = _rows(a)
    b, ldb = _rows(b)
    assert a.shape == b.shape and a.dtype == b.dtype
    g = np.empty(a.shape, dtype=a.dtype)
    lib().oracle_row_distance_bwd(_p(a), C.c_int64(lda), _p(b), C.c_int64(ldb), C.c_int64(a.shape[0]),
                                  C.c_int32(a.shape[1]), C.c_int(_dt(a)), C.c_double(scale), _p(g), C.c_int64(a.shape[1]))
    return g
