"""Thin ctypes binding of libgas.so: same names as the C ABI (include/gas.h),
argument marshalling only.  Tensors are torch tensors on the GPU; every step
runs in the library's kernels on torch's current stream."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgas.so")

F32, BF16 = 0, 1
OK = 0

EXPORTS = [
    "gas_last_error", "gas_version", "gas_validate_indices",
    "gas_pull", "gas_push", "gas_host_table_pointer", "gas_pull_host", "gas_push_host",
    "gas_gcn_norm", "gas_plan_create", "gas_plan_create_opt", "gas_plan_destroy", "gas_plan_describe", "gas_plan_copy_lists", "gas_spmm", "gas_spmm_hist", "gas_fuse_sources", "gas_spmm_t",
    "gas_linear", "gas_mlp2", "gas_linear_push", "gas_mlp2_push", "gas_mlp2_keep", "gas_spmm_linear",
    "gas_relu_bwd", "gas_linear_bwd_input", "gas_linear_bwd_weight", "gas_linear_bwd_weight_workspace", "gas_linear_bwd_weight_static",
    "gas_softmax_xent", "gas_sgd_step", "gas_sq_norm", "gas_sgd_step_clipped", "gas_axpy", "gas_row_distance", "gas_row_distance_bwd", "gas_row_dot",
    "gas_pna_aggregate", "gas_gat_aggregate", "gas_pna_aggregate_bwd", "gas_gat_aggregate_bwd",
    "gas_pna_aggregate_bwd_workspace", "gas_gat_aggregate_bwd_workspace",
    "gas_disk_open", "gas_disk_close", "gas_disk_pull", "gas_disk_push", "gas_disk_wait", "gas_disk_read_rows",
    "gas_disk_write_rows", "gas_disk_sync",
]

_lib = None


class GasError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"gas status {status}: {message}")
        self.status = status


def lib():
    """Load libgas.so.  There is no fallback: without the HIP library nothing runs."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2106_05609_amd._build` "
                              "(or __graft_entry__.build())")
        L = C.CDLL(LIB_PATH)
        L.gas_last_error.restype = C.c_char_p
        L.gas_version.restype = C.c_int
        L.gas_plan_destroy.restype = None
        L.gas_linear_bwd_weight_workspace.restype = C.c_int64
        L.gas_pna_aggregate_bwd_workspace.restype = C.c_int64
        L.gas_gat_aggregate_bwd_workspace.restype = C.c_int64
        for name in EXPORTS:
            if name not in ("gas_last_error", "gas_version", "gas_plan_destroy") and not name.endswith("_workspace"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(st):
    if st != OK:
        raise GasError(st, lib().gas_last_error().decode())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"feature tensors are float32 or bfloat16, got {t.dtype}")


def _mat(t: torch.Tensor):
    """(pointer, leading dimension in elements) of a 2-D row-major tensor or view."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("need a 2-D tensor with contiguous rows")
    return C.c_void_p(t.data_ptr()), C.c_int64(t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("need a contiguous tensor")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def gas_version() -> int:
    return int(lib().gas_version())


def gas_pull(hist, idx, dst, base=0, n=None):
    """dst[i] = hist[idx[i]] (idx int32 tensor) or hist[base+i] (idx None)."""
    n = (idx.numel() if idx is not None else dst.shape[0]) if n is None else n
    hp, ldh = _mat(hist)
    dp, ldd = _mat(dst)
    if dst.dtype != hist.dtype or dst.shape[1] != hist.shape[1] or dst.shape[0] < n:
        raise ValueError("gas_pull: dst does not match")
    fn = lib().gas_pull_host if isinstance(hist, HostTable) else lib().gas_pull
    _check(fn(hp, C.c_int64(hist.shape[0]), ldh, _ptr(idx, torch.int32), C.c_int64(base), C.c_int64(n),
              C.c_int32(hist.shape[1]), C.c_int(_dt(hist)), dp, ldd, _stream()))


def gas_push(src, idx, hist, base=0, n=None):
    """hist[idx[i]] = src[i] (idx int32 tensor, distinct) or hist[base+i] = src[i] (idx None)."""
    n = (idx.numel() if idx is not None else src.shape[0]) if n is None else n
    hp, ldh = _mat(hist)
    sp, lds = _mat(src)
    if src.dtype != hist.dtype or src.shape[1] != hist.shape[1] or src.shape[0] < n:
        raise ValueError("gas_push: src does not match")
    fn = lib().gas_push_host if isinstance(hist, HostTable) else lib().gas_push
    _check(fn(sp, lds, _ptr(idx, torch.int32), C.c_int64(base), C.c_int64(n), C.c_int32(hist.shape[1]),
              C.c_int(_dt(hist)), hp, C.c_int64(hist.shape[0]), ldh, _stream()))


def gas_gcn_norm(ptr, ind, n_id, deg, val):
    _check(lib().gas_gcn_norm(_ptr(ptr, torch.int32), _ptr(ind, torch.int32), C.c_int64(ptr.numel() - 1),
                              _ptr(n_id, torch.int32), _ptr(deg, torch.int32), _ptr(val, torch.float32), _stream()))


class PlanOptions(C.Structure):
    """gas_plan_options of the C ABI; a zero field means the default."""
    _fields_ = [("heavy_threshold", C.c_int32), ("chunk", C.c_int32), ("min_chunk", C.c_int32),
                ("window_rows", C.c_int32), ("xcd_ranges", C.c_int32), ("host_builder", C.c_int32)]


class Plan:
    """Owner of a gas_plan handle."""

    def __init__(self, ptr: torch.Tensor, nnz: int, max_F: int, n_rows=None, ind=None, options=None):
        """options: dict with any of heavy_threshold, chunk, min_chunk, window_rows, xcd_ranges (gas_plan_options)."""
        self.n_rows = ptr.numel() - 1 if n_rows is None else n_rows
        self.handle = C.c_void_p(0)
        if ind is not None and ind.numel() < nnz:
            raise ValueError("gas_plan_create: ind is shorter than nnz")
        opt = None
        if options:
            opt = PlanOptions(**options)
        _check(lib().gas_plan_create_opt(_ptr(ptr, torch.int32), _ptr(ind, torch.int32), C.c_int64(self.n_rows),
                                         C.c_int64(nnz), C.c_int32(max_F), None if opt is None else C.byref(opt),
                                         _stream(), C.byref(self.handle)))

    def describe(self) -> dict:
        info = (C.c_int64 * 16)()
        _check(lib().gas_plan_describe(self.handle, info))
        keys = ["n_rows", "nnz", "n_groups", "n_heavy", "n_chunks", "xcd_ranges", "max_F"]
        d = {k: int(info[i]) for i, k in enumerate(keys)}
        d["xcd_start"] = [int(info[7 + x]) for x in range(9)]
        return d

    def lists(self):
        """(group, heavy, chunk) as numpy int32 arrays on the host."""
        import numpy as np
        d = self.describe()
        group = np.zeros(2 * d["n_groups"], dtype=np.int32)
        heavy = np.zeros(2 * d["n_heavy"] + 1 if d["n_heavy"] else 0, dtype=np.int32)
        chunk = np.zeros(3 * d["n_chunks"], dtype=np.int32)
        as_p = lambda a: a.ctypes.data_as(C.c_void_p) if a.size else None
        _check(lib().gas_plan_copy_lists(self.handle, as_p(group), as_p(heavy), as_p(chunk), _stream()))
        return group, heavy, chunk

    def close(self):
        if self.handle:
            lib().gas_plan_destroy(self.handle)
            self.handle = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gas_plan_create(ptr, nnz, max_F, n_rows=None, ind=None, options=None) -> Plan:
    return Plan(ptr, nnz, max_F, n_rows, ind, options)


def gas_plan_destroy(plan: Plan):
    plan.close()


def gas_spmm(plan, rowptr, col, val, x, z, diag=0.0, s_agg=1.0, r=None, s_res=0.0):
    xp, ldx = _mat(x)
    zp, ldz = _mat(z)
    rp, ldr = (C.c_void_p(0), C.c_int64(0)) if r is None else _mat(r)
    if r is not None and r.dtype != x.dtype:
        raise TypeError("gas_spmm: R must have X's dtype")
    if z.shape[1] != x.shape[1] or z.shape[0] < plan.n_rows:
        raise ValueError("gas_spmm: Z does not match")
    _check(lib().gas_spmm(plan.handle, _ptr(rowptr, torch.int32), _ptr(col, torch.int32), _ptr(val, torch.float32),
                          C.c_float(diag), xp, ldx, C.c_int(_dt(x)), C.c_int32(x.shape[1]), C.c_float(s_agg), rp, ldr,
                          C.c_float(s_res), zp, ldz, C.c_int(_dt(z)), _stream()))


def gas_fuse_sources(col, nb, n_id, src):
    _check(lib().gas_fuse_sources(_ptr(col, torch.int32), C.c_int64(col.numel()), C.c_int64(nb), _ptr(n_id, torch.int32),
                                  _ptr(src, torch.int32), _stream()))


def gas_spmm_hist(plan, rowptr, src, val, x, hist, z, diag=0.0, s_agg=1.0, r=None, s_res=0.0):
    """x: the in-batch rows [n_rows, F]; hist: the history table the halo rows are read from."""
    xp, ldx = _mat(x)
    hp, ldh = _mat(hist)
    zp, ldz = _mat(z)
    rp, ldr = (C.c_void_p(0), C.c_int64(0)) if r is None else _mat(r)
    if hist.dtype != x.dtype or hist.shape[1] != x.shape[1] or (r is not None and r.dtype != x.dtype):
        raise TypeError("gas_spmm_hist: hist and R must match X")
    if z.shape[1] != x.shape[1] or z.shape[0] < plan.n_rows or x.shape[0] < plan.n_rows:
        raise ValueError("gas_spmm_hist: shapes do not match")
    _check(lib().gas_spmm_hist(plan.handle, _ptr(rowptr, torch.int32), _ptr(src, torch.int32), _ptr(val, torch.float32),
                               C.c_float(diag), xp, ldx, hp, C.c_int64(hist.shape[0]), ldh, C.c_int(_dt(x)),
                               C.c_int32(x.shape[1]), C.c_float(s_agg), rp, ldr, C.c_float(s_res), zp, ldz,
                               C.c_int(_dt(z)), _stream()))


def gas_spmm_t(plan, colptr, row, val, g, gx, diag=0.0, s_agg=1.0):
    gp, ldg = _mat(g)
    op, ldo = _mat(gx)
    if gx.shape[1] != g.shape[1] or gx.shape[0] < plan.n_rows:
        raise ValueError("gas_spmm_t: GX does not match")
    _check(lib().gas_spmm_t(plan.handle, _ptr(colptr, torch.int32), _ptr(row, torch.int32), _ptr(val, torch.float32),
                            C.c_float(diag), C.c_float(s_agg), C.c_int64(g.shape[0]), gp, ldg, C.c_int(_dt(g)), C.c_int32(g.shape[1]),
                            op, ldo, C.c_int(_dt(gx)), _stream()))


def gas_linear(z, w, y, bias=None, c_identity=0.0, c_weight=1.0, relu=False):
    zp, ldz = _mat(z)
    yp, ldy = _mat(y)
    if w.dtype != z.dtype or y.dtype != z.dtype or w.shape[0] != z.shape[1] or y.shape != (z.shape[0], w.shape[1]):
        raise ValueError("gas_linear: shapes or dtypes do not match")
    _check(lib().gas_linear(zp, ldz, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _ptr(w), C.c_int32(w.shape[1]),
                            _ptr(bias), C.c_int(_dt(z)), C.c_float(c_identity), C.c_float(c_weight),
                            C.c_int(int(relu)), yp, ldy, _stream()))


def gas_mlp2(z, w1, w2, y, b1=None, b2=None, relu_out=False):
    zp, ldz = _mat(z)
    yp, ldy = _mat(y)
    if not (w1.dtype == w2.dtype == z.dtype == y.dtype) or w1.shape[0] != z.shape[1] or w2.shape[0] != w1.shape[1] \
            or y.shape != (z.shape[0], w2.shape[1]):
        raise ValueError("gas_mlp2: shapes or dtypes do not match")
    _check(lib().gas_mlp2(zp, ldz, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _ptr(w1), C.c_int32(w1.shape[1]),
                          _ptr(b1), _ptr(w2), C.c_int32(w2.shape[1]), _ptr(b2), C.c_int(_dt(z)),
                          C.c_int(int(relu_out)), yp, ldy, _stream()))


def gas_validate_indices(idx, limit) -> bool:
    st = lib().gas_validate_indices(_ptr(idx, torch.int32), C.c_int64(idx.numel()), C.c_int64(limit), _stream())
    if st == -4:
        return False
    _check(st)
    return True


def gas_relu_bwd(gy, y, gp):
    """gp = gy where y > 0 else 0 (gp may be gy itself)."""
    a, lda = _mat(gy)
    b, ldb = _mat(y)
    c, ldc = _mat(gp)
    if not (gy.shape == y.shape == gp.shape and gy.dtype == y.dtype == gp.dtype):
        raise ValueError("gas_relu_bwd: shapes or dtypes do not match")
    _check(lib().gas_relu_bwd(a, lda, b, ldb, C.c_int64(gy.shape[0]), C.c_int32(gy.shape[1]), C.c_int(_dt(gy)), c, ldc,
                              _stream()))


def gas_linear_bwd_input(gp, w, gz, c_identity=0.0, c_weight=1.0, mask=None):
    """gz [n, F_in] = c_identity * gp + c_weight * gp @ w.T, zeroed where mask <= 0; w is [F_in, F_out]."""
    a, lda = _mat(gp)
    c, ldc = _mat(gz)
    mp, ldm = (C.c_void_p(0), C.c_int64(0)) if mask is None else _mat(mask)
    if w.dtype != gp.dtype or gz.dtype != gp.dtype or w.shape[1] != gp.shape[1] or gz.shape != (gp.shape[0], w.shape[0]) \
            or (mask is not None and (mask.shape != gz.shape or mask.dtype != gp.dtype)):
        raise ValueError("gas_linear_bwd_input: shapes or dtypes do not match")
    _check(lib().gas_linear_bwd_input(a, lda, C.c_int64(gp.shape[0]), C.c_int32(gp.shape[1]), _ptr(w),
                                      C.c_int32(w.shape[0]), C.c_int(_dt(gp)), C.c_float(c_identity),
                                      C.c_float(c_weight), mp, ldm, c, ldc, _stream()))


def gas_linear_bwd_weight_workspace(n_rows, f_in, f_out) -> int:
    return int(lib().gas_linear_bwd_weight_workspace(C.c_int64(n_rows), C.c_int32(f_in), C.c_int32(f_out)))


def gas_linear_bwd_weight(z, gp, dw, workspace, c_weight=1.0):
    """dw [F_in, F_out] float32 = c_weight * z.T @ gp; workspace: a uint8 tensor of at least
    gas_linear_bwd_weight_workspace(...) bytes."""
    a, lda = _mat(z)
    b, ldb = _mat(gp)
    if z.dtype != gp.dtype or z.shape[0] != gp.shape[0] or dw.dtype != torch.float32 or \
            dw.shape != (z.shape[1], gp.shape[1]) or not dw.is_contiguous():
        raise ValueError("gas_linear_bwd_weight: shapes or dtypes do not match")
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().gas_linear_bwd_weight(a, lda, b, ldb, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]),
                                       C.c_int32(gp.shape[1]), C.c_int(_dt(z)), C.c_float(c_weight), _ptr(dw),
                                       _ptr(workspace), C.c_int64(nbytes), _stream()))


def gas_linear_bwd_weight_static(z, gp, dw, c_weight=1.0):
    """gas_linear_bwd_weight with the slab partials in the library's static scratch array (no workspace)."""
    a, lda = _mat(z)
    b, ldb = _mat(gp)
    if z.dtype != gp.dtype or z.shape[0] != gp.shape[0] or dw.dtype != torch.float32 or \
            dw.shape != (z.shape[1], gp.shape[1]) or not dw.is_contiguous():
        raise ValueError("gas_linear_bwd_weight_static: shapes or dtypes do not match")
    _check(lib().gas_linear_bwd_weight_static(a, lda, b, ldb, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]),
                                              C.c_int32(gp.shape[1]), C.c_int(_dt(z)), C.c_float(c_weight),
                                              _ptr(dw), _stream()))


def gas_linear_push(z, w, y, idx, hist, bias=None, c_identity=0.0, c_weight=1.0, relu=False):
    """gas_linear, and y[i] is also stored to hist[idx[i]] (Push fused into the epilogue)."""
    zp, ldz = _mat(z)
    yp, ldy = _mat(y)
    hp, ldh = _mat(hist)
    if w.dtype != z.dtype or y.dtype != z.dtype or hist.dtype != z.dtype or w.shape[0] != z.shape[1] or \
            y.shape != (z.shape[0], w.shape[1]) or hist.shape[1] != w.shape[1] or idx.numel() != z.shape[0]:
        raise ValueError("gas_linear_push: shapes or dtypes do not match")
    _check(lib().gas_linear_push(zp, ldz, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _ptr(w), C.c_int32(w.shape[1]),
                                 _ptr(bias), C.c_int(_dt(z)), C.c_float(c_identity), C.c_float(c_weight),
                                 C.c_int(int(relu)), yp, ldy, _ptr(idx, torch.int32), hp, C.c_int64(hist.shape[0]), ldh,
                                 _stream()))


def gas_mlp2_keep(z, w1, w2, y, h_out, idx=None, hist=None, b1=None, b2=None, relu_out=False):
    """gas_mlp2 that also stores the hidden activation relu(z w1 + b1) to h_out, and (idx, hist given) pushes y."""
    zp, ldz = _mat(z)
    yp, ldy = _mat(y)
    hp, ldh = _mat(h_out)
    tp, ldt = (C.c_void_p(0), C.c_int64(0)) if hist is None else _mat(hist)
    if not (w1.dtype == w2.dtype == z.dtype == y.dtype == h_out.dtype) or w1.shape[0] != z.shape[1] or \
            w2.shape[0] != w1.shape[1] or y.shape != (z.shape[0], w2.shape[1]) or \
            h_out.shape != (z.shape[0], w1.shape[1]) or (hist is None) != (idx is None) or \
            (hist is not None and (hist.dtype != z.dtype or hist.shape[1] != w2.shape[1] or idx.numel() != z.shape[0])):
        raise ValueError("gas_mlp2_keep: shapes or dtypes do not match")
    _check(lib().gas_mlp2_keep(zp, ldz, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _ptr(w1), C.c_int32(w1.shape[1]),
                               _ptr(b1), _ptr(w2), C.c_int32(w2.shape[1]), _ptr(b2), C.c_int(_dt(z)),
                               C.c_int(int(relu_out)), yp, ldy, hp, ldh, _ptr(idx, torch.int32), tp,
                               C.c_int64(0 if hist is None else hist.shape[0]), ldt, _stream()))


def spmm_linear_supported(x, f_out) -> bool:
    """Whether gas_spmm_linear takes this layer (fp32, widths multiples of 4 up to 128)."""
    f_in = x.shape[1]
    return x.dtype == torch.float32 and f_in % 4 == 0 and f_out % 4 == 0 and max(f_in, f_out) <= 128


def gas_spmm_linear(rowptr, src, val, x, w, y, hist=None, diag=0.0, s_agg=1.0, r=None, s_res=0.0, bias=None,
                    c_identity=0.0, c_weight=1.0, relu=False, push_idx=None, push_hist=None, z_out=None):
    """One layer in one launch: aggregation of the rows of y (sources: rows of x, or rows of hist for negative
    indices), transform by w, optional store of every output row to push_hist[push_idx[i]]."""
    n_rows = y.shape[0]
    xp, ldx = _mat(x)
    yp, ldy = _mat(y)
    hp, ldh = (C.c_void_p(0), C.c_int64(0)) if hist is None else _mat(hist)
    rp, ldr = (C.c_void_p(0), C.c_int64(0)) if r is None else _mat(r)
    pp, ldp = (C.c_void_p(0), C.c_int64(0)) if push_hist is None else _mat(push_hist)
    zp, ldzo = (C.c_void_p(0), C.c_int64(0)) if z_out is None else _mat(z_out)
    if z_out is not None and (z_out.dtype != x.dtype or z_out.shape[1] != x.shape[1] or z_out.shape[0] < n_rows):
        raise ValueError("gas_spmm_linear: z_out does not match")
    if w.dtype != x.dtype or y.dtype != x.dtype or w.shape[0] != x.shape[1] or y.shape[1] != w.shape[1] or \
            rowptr.numel() != n_rows + 1 or (hist is not None and (hist.dtype != x.dtype or hist.shape[1] != x.shape[1])) or \
            (r is not None and (r.dtype != x.dtype or r.shape[1] != x.shape[1] or r.shape[0] < n_rows)) or \
            (push_hist is not None and (push_hist.dtype != x.dtype or push_hist.shape[1] != w.shape[1] or
                                        push_idx is None or push_idx.numel() != n_rows)):
        raise ValueError("gas_spmm_linear: shapes or dtypes do not match")
    _check(lib().gas_spmm_linear(
        _ptr(rowptr, torch.int32), _ptr(src, torch.int32), _ptr(val, torch.float32), C.c_int64(n_rows), xp, ldx, hp,
        C.c_int64(0 if hist is None else hist.shape[0]), ldh, C.c_int(_dt(x)), C.c_int32(x.shape[1]), C.c_float(diag),
        C.c_float(s_agg), rp, ldr, C.c_float(s_res), _ptr(w), C.c_int32(w.shape[1]), _ptr(bias), C.c_float(c_identity),
        C.c_float(c_weight), C.c_int(int(relu)), yp, ldy, zp, ldzo, _ptr(push_idx, torch.int32), pp,
        C.c_int64(0 if push_hist is None else push_hist.shape[0]), ldp, _stream()))


def gas_mlp2_push(z, w1, w2, y, idx, hist, b1=None, b2=None, relu_out=False):
    """gas_mlp2, and y[i] is also stored to hist[idx[i]]."""
    zp, ldz = _mat(z)
    yp, ldy = _mat(y)
    hp, ldh = _mat(hist)
    if not (w1.dtype == w2.dtype == z.dtype == y.dtype == hist.dtype) or w1.shape[0] != z.shape[1] or \
            w2.shape[0] != w1.shape[1] or y.shape != (z.shape[0], w2.shape[1]) or hist.shape[1] != w2.shape[1] or \
            idx.numel() != z.shape[0]:
        raise ValueError("gas_mlp2_push: shapes or dtypes do not match")
    _check(lib().gas_mlp2_push(zp, ldz, C.c_int64(z.shape[0]), C.c_int32(z.shape[1]), _ptr(w1), C.c_int32(w1.shape[1]),
                               _ptr(b1), _ptr(w2), C.c_int32(w2.shape[1]), _ptr(b2), C.c_int(_dt(z)),
                               C.c_int(int(relu_out)), yp, ldy, _ptr(idx, torch.int32), hp, C.c_int64(hist.shape[0]),
                               ldh, _stream()))


def gas_softmax_xent(a, labels, grad, loss_rows, loss_sum=None, scale=1.0):
    """Softmax cross-entropy per row and its gradient (scaled); rows with a label outside [0, C) are skipped."""
    ap, lda = _mat(a)
    gp, ldg = _mat(grad)
    if grad.dtype != a.dtype or grad.shape != a.shape or labels.numel() != a.shape[0] or \
            loss_rows.dtype != torch.float32 or loss_rows.numel() != a.shape[0] or not loss_rows.is_contiguous():
        raise ValueError("gas_softmax_xent: shapes or dtypes do not match")
    _check(lib().gas_softmax_xent(ap, lda, C.c_int64(a.shape[0]), C.c_int32(a.shape[1]), C.c_int(_dt(a)),
                                  _ptr(labels, torch.int32), C.c_float(scale), _ptr(loss_rows, torch.float32),
                                  _ptr(loss_sum, torch.float32), gp, ldg, _stream()))


def gas_sgd_step(w, dw, lr, weight_decay=0.0):
    """In place: w <- w - lr * (dw + weight_decay * w); dw float32 of the same shape."""
    if not w.is_contiguous() or not dw.is_contiguous() or dw.dtype != torch.float32 or dw.numel() != w.numel():
        raise ValueError("gas_sgd_step: w and dw must be contiguous and of equal size, dw float32")
    _check(lib().gas_sgd_step(_ptr(w), C.c_int64(w.numel()), C.c_int(_dt(w)), _ptr(dw, torch.float32),
                              C.c_float(lr), C.c_float(weight_decay), _stream()))


def gas_sq_norm(x, out):
    """out[0] = sum of the squares of x (float32, contiguous); out: a 1-element float32 view."""
    if not x.is_contiguous() or x.dtype != torch.float32 or out.dtype != torch.float32 or out.numel() < 1:
        raise ValueError("gas_sq_norm: x float32 contiguous, out float32")
    _check(lib().gas_sq_norm(_ptr(x, torch.float32), C.c_int64(x.numel()), _ptr(out, torch.float32), _stream()))


def gas_sgd_step_clipped(w, dw, lr, sq_norms, max_norm, weight_decay=0.0):
    """gas_sgd_step with dw scaled by min(1, max_norm / (sqrt(sum(sq_norms)) + 1e-6)), formed on the device."""
    if not w.is_contiguous() or not dw.is_contiguous() or dw.dtype != torch.float32 or dw.numel() != w.numel():
        raise ValueError("gas_sgd_step_clipped: w and dw must be contiguous and of equal size, dw float32")
    if sq_norms.dtype != torch.float32 or not sq_norms.is_contiguous():
        raise ValueError("gas_sgd_step_clipped: sq_norms float32 contiguous")
    _check(lib().gas_sgd_step_clipped(_ptr(w), C.c_int64(w.numel()), C.c_int(_dt(w)), _ptr(dw, torch.float32),
                                      C.c_float(lr), C.c_float(weight_decay), _ptr(sq_norms, torch.float32),
                                      C.c_int32(sq_norms.numel()), C.c_float(max_norm), _stream()))


def gas_pna_aggregate(rowptr, col, x, out, delta, add=None):
    """out [n_rows, 9F] = scalers [1, s, 1/s] (x) aggregators [mean, min, max] over the neighbours (+ add)."""
    xp, ldx = _mat(x)
    op, ldo = _mat(out)
    ap, lda = (C.c_void_p(0), C.c_int64(0)) if add is None else _mat(add)
    n_rows = rowptr.numel() - 1
    if out.dtype != x.dtype or out.shape[0] < n_rows or out.shape[1] != 9 * x.shape[1] or \
            (add is not None and (add.dtype != x.dtype or add.shape[1] != x.shape[1] or add.shape[0] < n_rows)):
        raise ValueError("gas_pna_aggregate: shapes or dtypes do not match")
    _check(lib().gas_pna_aggregate(_ptr(rowptr, torch.int32), _ptr(col, torch.int32), C.c_int64(n_rows), xp, ldx,
                                   C.c_int(_dt(x)), C.c_int32(x.shape[1]), ap, lda, C.c_float(delta), op, ldo,
                                   _stream()))


def gas_gat_aggregate(rowptr, col, p, a_dst, a_src, z, negative_slope=0.2, relu=False):
    """z[v] = sum_k softmax_k(LeakyReLU(a_dst.p[v] + a_src.p[col k])) p[col k] over the entries of row v."""
    pp, ldp = _mat(p)
    zp, ldz = _mat(z)
    n_rows = rowptr.numel() - 1
    if z.dtype != p.dtype or a_dst.dtype != p.dtype or a_src.dtype != p.dtype or z.shape[1] != p.shape[1] or \
            z.shape[0] < n_rows or a_dst.numel() != p.shape[1] or a_src.numel() != p.shape[1]:
        raise ValueError("gas_gat_aggregate: shapes or dtypes do not match")
    _check(lib().gas_gat_aggregate(_ptr(rowptr, torch.int32), _ptr(col, torch.int32), C.c_int64(n_rows), pp, ldp,
                                   C.c_int(_dt(p)), C.c_int32(p.shape[1]), _ptr(a_dst), _ptr(a_src),
                                   C.c_float(negative_slope), C.c_int(int(relu)), zp, ldz, _stream()))


def gas_axpy(x, e, y, alpha=1.0):
    """y = x + alpha * e over [n, F] (y may be x)."""
    xp, ldx = _mat(x)
    ep, lde = _mat(e)
    yp, ldy = _mat(y)
    if x.shape != e.shape or x.shape != y.shape or x.dtype != e.dtype or x.dtype != y.dtype:
        raise ValueError("gas_axpy: shapes or dtypes do not match")
    _check(lib().gas_axpy(xp, ldx, ep, lde, C.c_int64(x.shape[0]), C.c_int32(x.shape[1]), C.c_int(_dt(x)),
                          C.c_float(alpha), yp, ldy, _stream()))


def gas_row_dot(a, b, dot, dot_sum=None):
    """dot[i] = <a[i], b[i]> (float32 [n]); dot_sum (float32 [1]) receives their sum in a fixed order."""
    ap, lda = _mat(a)
    bp, ldb = _mat(b)
    if a.shape != b.shape or a.dtype != b.dtype or dot.dtype != torch.float32 or dot.numel() < a.shape[0]:
        raise ValueError("gas_row_dot: shapes or dtypes do not match")
    _check(lib().gas_row_dot(ap, lda, bp, ldb, C.c_int64(a.shape[0]), C.c_int32(a.shape[1]), C.c_int(_dt(a)),
                             _ptr(dot), _ptr(dot_sum), _stream()))


def gas_row_distance(a, b, dist, dist_sum=None):
    """dist[i] = ||a[i] - b[i]||_2 (float32 [n]); dist_sum (float32 [1]) receives their sum."""
    ap, lda = _mat(a)
    bp, ldb = _mat(b)
    if a.shape != b.shape or a.dtype != b.dtype or dist.dtype != torch.float32 or dist.numel() != a.shape[0] or \
            not dist.is_contiguous():
        raise ValueError("gas_row_distance: shapes or dtypes do not match")
    _check(lib().gas_row_distance(ap, lda, bp, ldb, C.c_int64(a.shape[0]), C.c_int32(a.shape[1]), C.c_int(_dt(a)),
                                  _ptr(dist, torch.float32), _ptr(dist_sum, torch.float32), _stream()))


def gas_row_distance_bwd(a, b, g, scale=1.0):
    """g[i] = scale * (a[i] - b[i]) / ||a[i] - b[i]||_2 (zero where the rows are equal)."""
    ap, lda = _mat(a)
    bp, ldb = _mat(b)
    gp, ldg = _mat(g)
    if a.shape != b.shape or g.shape != a.shape or not (a.dtype == b.dtype == g.dtype):
        raise ValueError("gas_row_distance_bwd: shapes or dtypes do not match")
    _check(lib().gas_row_distance_bwd(ap, lda, bp, ldb, C.c_int64(a.shape[0]), C.c_int32(a.shape[1]), C.c_int(_dt(a)),
                                      C.c_float(scale), gp, ldg, _stream()))


class HostTable:
    """A history table in pinned host memory, usable as the `hist` argument of gas_pull / gas_push: it carries
    the device-side address of the allocation and looks like a 2-D tensor to the marshalling code."""

    def __init__(self, t: torch.Tensor):
        if t.is_cuda or not t.is_pinned() or t.dim() != 2 or not t.is_contiguous():
            raise ValueError("HostTable: need a contiguous 2-D tensor in pinned host memory")
        dev = C.c_void_p(0)
        _check(lib().gas_host_table_pointer(C.c_void_p(t.data_ptr()), C.byref(dev)))
        self.tensor, self._dev = t, dev.value
        self.shape, self.dtype = t.shape, t.dtype

    def data_ptr(self):
        return self._dev

    def dim(self):
        return 2

    def stride(self, i):
        return self.tensor.stride(i)


class DiskTable:
    """A history table in a file (gas_disk_* of the C ABI).  Index lists are int32 tensors or arrays in HOST memory;
    pull and push return a ticket and run beside the caller, wait(ticket) blocks until that transfer is complete.
    The tensors of a transfer are kept alive here until it has been waited for."""

    def __init__(self, path, n_rows, width, dtype, create=True, io_threads=0, staging_bytes=0, calls=False):
        self.shape, self.dtype, self.path = (int(n_rows), int(width)), dtype, path
        self._code = _dt(torch.empty(0, dtype=dtype))
        self._h = C.c_void_p(0)
        self._held = {}
        _check(lib().gas_disk_open(os.fsencode(path), C.c_int64(n_rows), C.c_int32(width), C.c_int(self._code),
                                   C.c_int32((1 if create else 0) | (2 if calls else 0)), C.c_int32(io_threads),
                                   C.c_int64(staging_bytes),
                                   C.byref(self._h)))

    def _idx(self, idx):
        if idx is None:
            return None, C.c_void_p(0)
        t = torch.as_tensor(idx)
        if t.is_cuda or t.dtype != torch.int32 or t.dim() != 1 or not t.is_contiguous():
            raise ValueError("DiskTable: idx must be a contiguous 1-D int32 tensor in host memory")
        return t, C.c_void_p(t.data_ptr())

    def _rows(self, t, n, device):
        if t.dtype != self.dtype or t.dim() != 2 or t.shape[1] != self.shape[1] or t.shape[0] < n \
                or t.is_cuda != device:
            raise ValueError("DiskTable: rows do not match the table")
        return _mat(t)

    def _transfer(self, fn, idx, base, n, rows):
        it, ip = self._idx(idx)
        n = (it.numel() if it is not None else rows.shape[0]) if n is None else n
        rp, ld = self._rows(rows, n, True)
        ticket = C.c_int64(0)
        _check(fn(self._h, ip, C.c_int64(base), C.c_int64(n), rp, ld, _stream(), C.byref(ticket)))
        self._held[ticket.value] = rows
        return ticket.value

    def pull(self, idx, dst, base=0, n=None) -> int:
        """dst[i] = table[idx[i]] (or table[base + i]); starts after the current stream's work so far."""
        return self._transfer(lib().gas_disk_pull, idx, base, n, dst)

    def push(self, src, idx, base=0, n=None) -> int:
        """table[idx[i]] = src[i] (or table[base + i]); reads src after the current stream's work so far."""
        return self._transfer(lib().gas_disk_push, idx, base, n, src)

    def wait(self, ticket=0):
        try:
            _check(lib().gas_disk_wait(self._h, C.c_int64(ticket)))
        finally:
            for k in [k for k in self._held if ticket <= 0 or k <= ticket]:
                del self._held[k]

    def read_rows(self, dst, idx=None, base=0, n=None):
        it, ip = self._idx(idx)
        n = (it.numel() if it is not None else dst.shape[0]) if n is None else n
        rp, ld = self._rows(dst, n, False)
        _check(lib().gas_disk_read_rows(self._h, ip, C.c_int64(base), C.c_int64(n), rp, ld))
        self._held.clear()

    def write_rows(self, src, idx=None, base=0, n=None):
        it, ip = self._idx(idx)
        n = (it.numel() if it is not None else src.shape[0]) if n is None else n
        rp, ld = self._rows(src, n, False)
        _check(lib().gas_disk_write_rows(self._h, ip, C.c_int64(base), C.c_int64(n), rp, ld))
        self._held.clear()

    def sync(self):
        _check(lib().gas_disk_sync(self._h))
        self._held.clear()

    def close(self):
        if self._h:
            h, self._h = self._h, C.c_void_p(0)
            self._held.clear()
            _check(lib().gas_disk_close(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gas_pna_aggregate_bwd(rowptr, col, colptr, row, csc_pos, x, g, gx, delta, gadd=None, plan_t=None):
    """Backward of gas_pna_aggregate: gx [n_out, F] (n_out = gx.shape[0] columns of the pattern), gadd [n_rows, F].
    plan_t: a Plan of the CSC copy for those n_out columns (fast path), or None (plain kernels)."""
    xp, ldx = _mat(x)
    gp, ldg = _mat(g)
    op, ldo = _mat(gx)
    ap, lda = (C.c_void_p(0), C.c_int64(0)) if gadd is None else _mat(gadd)
    n_rows, F = rowptr.numel() - 1, x.shape[1]
    if g.shape != (n_rows, 9 * F) or gx.shape[1] != F or g.dtype != x.dtype or gx.dtype != x.dtype:
        raise ValueError("gas_pna_aggregate_bwd: shapes or dtypes do not match")
    nnz = col.numel()
    nbytes = int(lib().gas_pna_aggregate_bwd_workspace(C.c_int64(n_rows), C.c_int64(nnz), C.c_int32(F)))
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=x.device)
    _check(lib().gas_pna_aggregate_bwd(plan_t.handle if plan_t is not None else C.c_void_p(0),
                                       _ptr(rowptr, torch.int32), _ptr(col, torch.int32), C.c_int64(n_rows),
                                       C.c_int64(nnz), _ptr(colptr, torch.int32), _ptr(row, torch.int32), _ptr(csc_pos, torch.int32),
                                       C.c_int64(gx.shape[0]), xp, ldx, C.c_int(_dt(x)), C.c_int32(F), C.c_float(delta),
                                       gp, ldg, op, ldo, ap, lda, _ptr(ws), C.c_int64(nbytes), _stream()))


def gas_gat_aggregate_bwd(rowptr, col, colptr, row, csc_pos, p, a_dst, a_src, gz, gp_out, ga_dst, ga_src,
                          negative_slope=0.2, plan_t=None):
    """Backward of gas_gat_aggregate (gz: gradient before any activation): gp_out [n_out, F] rows of P's gradient,
    ga_dst / ga_src float32 [F].  plan_t: a Plan of the CSC copy for those n_out columns (fast path), or None."""
    pp, ldp = _mat(p)
    zp, ldz = _mat(gz)
    op, ldo = _mat(gp_out)
    n_rows, n_cols, F, nnz = rowptr.numel() - 1, p.shape[0], p.shape[1], col.numel()
    if gz.shape != (n_rows, F) or gp_out.shape[1] != F or colptr.numel() != n_cols + 1 or gz.dtype != p.dtype or \
            gp_out.dtype != p.dtype or ga_dst.dtype != torch.float32 or ga_src.dtype != torch.float32:
        raise ValueError("gas_gat_aggregate_bwd: shapes or dtypes do not match")
    nbytes = int(lib().gas_gat_aggregate_bwd_workspace(C.c_int64(n_rows), C.c_int64(n_cols), C.c_int64(nnz), C.c_int32(F)))
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=p.device)
    _check(lib().gas_gat_aggregate_bwd(plan_t.handle if plan_t is not None else C.c_void_p(0),
                                       _ptr(rowptr, torch.int32), _ptr(col, torch.int32), C.c_int64(n_rows),
                                       _ptr(colptr, torch.int32), _ptr(row, torch.int32), _ptr(csc_pos, torch.int32),
                                       C.c_int64(n_cols), C.c_int64(gp_out.shape[0]), C.c_int64(nnz), pp, ldp,
                                       C.c_int(_dt(p)), C.c_int32(F), _ptr(a_dst), _ptr(a_src), C.c_float(negative_slope),
                                       zp, ldz, op, ldo, _ptr(ga_dst), _ptr(ga_src), _ptr(ws), C.c_int64(nbytes), _stream()))
