"""MI355X-native hot path of the preconditioned Nystrom kernel ridge solver (arXiv 2006.10350).

Thin ctypes binding over ``libknm.so`` (hand-written HIP for gfx950).  The functions
here have the names of the C entry points declared in ``include/knm.h`` and only
marshal arguments: PyTorch supplies device memory and the stream, every step of the
computation runs in the library's kernels.  There is no CPU fallback: importing works
without a GPU (so the library's symbols can be checked), any compute call needs one.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libknm.so")

KNM_OK = 0
KNM_INVALID_ARG, KNM_UNSUPPORTED, KNM_ALLOC, KNM_HIP_ERROR, KNM_NOT_PD = -1, -2, -3, -4, -5
STATUS_NAMES = {0: "KNM_OK", -1: "KNM_INVALID_ARG", -2: "KNM_UNSUPPORTED", -3: "KNM_ALLOC",
                -4: "KNM_HIP_ERROR", -5: "KNM_NOT_PD"}

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_int = ctypes.c_int
_f32 = ctypes.c_float
_f64 = ctypes.c_double

_PTS = [_vp, _i64, _int, _i64, _vp, _i64, _i64, _f32]  # X n d ldx C M ldc sigma

SIGNATURES = {
    "knm_create": (_int, [ctypes.POINTER(_vp), _int, _vp]),
    "knm_destroy": (_int, [_vp]),
    "knm_strerror": (ctypes.c_char_p, [_int]),
    "knm_last_error": (ctypes.c_char_p, [_vp]),
    "knm_max_d": (_int, []),
    "knm_max_t": (_int, []),
    "knm_workspace_bytes": (ctypes.c_size_t, [_i64, _i64, _int, _int]),
    "knm_v": (_int, [_vp] + _PTS + [_vp, _int, _vp]),
    "knm_prod": (_int, [_vp] + _PTS + [_vp, _int, _vp, _vp]),
    "knm_prod_weighted": (_int, [_vp] + _PTS + [_vp, _vp, _int, _vp]),
    "knm_prod_static": (_int, [_vp] + _PTS + [_vp, _int, _vp, _vp]),
    "knm_static_scratch_bytes": (ctypes.c_size_t, []),
    "knm_t_y": (_int, [_vp] + _PTS + [_vp, _int, _vp]),
    "precond_build": (_int, [_vp, _vp, _i64, _int, _i64, _f32, _f64, _f64, ctypes.POINTER(_vp),
                             ctypes.POINTER(_i64)]),
    "precond_free": (_int, [_vp]),
    "precond_get_factors": (_int, [_vp, _vp, _vp, _vp]),
    "falkon_linop": (_int, [_vp, _vp] + _PTS + [_f64, _vp, _int, _vp]),
    "falkon_linop_weighted": (_int, [_vp, _vp] + _PTS + [_f64, _vp, _vp, _int, _vp]),
    "precond_reweight": (_int, [_vp, _vp, _f64, _vp, ctypes.POINTER(_i64)]),
    "precond_solve": (_int, [_vp, _vp, _int, _vp, _int, _vp]),
    "knm_prod_csr": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _i64, _f32, _vp, _int, _vp, _vp]),
    "knm_v_csr": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _i64, _f32, _vp, _int, _vp]),
    "precond_build_csr": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _f32, _f64, _f64, ctypes.POINTER(_vp),
                                 ctypes.POINTER(_i64)]),
    "falkon_fit_csr": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _int, _vp, _vp, _vp, _i64, _i64, _f32, _f64, _f64, _int,
                              _vp, _vp]),
    "precond_block_product": (_int, [_vp, _int, _i64, _i64, _i64, _f64, _vp, _i64, _vp, _i64, _f64, _vp, _i64]),
    "precond_get_block": (_int, [_vp, _vp, _int, _i64, _i64, _i64, _i64, _vp]),
    "precond_rank_k_update": (_int, [_vp, _int, _i64, _i64, _f64, _vp, _i64, _vp, _int, _f64, _f64, _vp, _i64]),
    "falkon_fit": (_int, [_vp, _vp, _i64, _int, _i64, _vp, _int, _vp, _i64, _i64, _f32, _f64, _f64, _int,
                          _vp, _vp]),
    "logfalkon_fit": (_int, [_vp, _vp, _i64, _int, _i64, _vp, _vp, _i64, _i64, _vp, _f32, _vp, _vp, _int, _f64,
                             _vp, _vp]),
    "logfalkon_fit_csr": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _i64, _i64, _vp, _f32, _vp, _vp, _int,
                                 _f64, _vp, _vp]),
    "knm_get_fit_timing": (_int, [_vp, ctypes.POINTER(_f64)]),
    "falkon_predict": (_int, [_vp] + _PTS + [_vp, _int, _vp]),
    "knm_set_cross_term": (_int, [_vp, _int]),
    "knm_get_cross_term": (_int, [_vp]),
    "knm_set_kernel": (_int, [_vp, _int]),
    "knm_set_sparse_head_limit": (_int, [_vp, _int]),
    "knm_workspace_held": (ctypes.c_size_t, [_vp]),
    "knm_set_pack_limit": (_int, [_vp, ctypes.c_size_t]),
    "knm_set_timing": (_int, [_vp, _int]),
    "knm_range_exceeded": (_int, [_vp, ctypes.POINTER(_i64), _int]),
    "knm_probe_rates": (_int, [_vp, ctypes.POINTER(_f64), _int]),
    "knm_get_timing": (_int, [_vp, ctypes.POINTER(_f32)]),
}

_lib = None


class KnmError(RuntimeError):
    def __init__(self, status: int, detail: str = ""):
        self.status = status
        name = STATUS_NAMES.get(status, str(status))
        super().__init__(f"{name}: {detail}" if detail else name)


def load_library() -> ctypes.CDLL:
    """Load libknm.so and declare every entry point; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with __graft_entry__.build() "
                              "(python paper_2006_10350_amd/build.py); there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _dev_f32(x: torch.Tensor, what: str) -> torch.Tensor:
    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32):
        raise TypeError(f"{what} must be a float32 tensor on the GPU")
    return x


def _points(x: torch.Tensor, what: str):
    _dev_f32(x, what)
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError(f"{what} must be 2-D with unit stride along features")
    return x, x.shape[0], x.shape[1], (x.stride(0) if x.shape[0] > 1 else x.shape[1])


def _cols(x: torch.Tensor, rows: int, what: str):
    _dev_f32(x, what)
    sq = x.dim() == 1
    x2 = x.reshape(rows, -1)
    if not x2.is_contiguous():
        x2 = x2.contiguous()
    return x2, x2.shape[1], sq


class Context:
    """A library context bound to a device and to the torch stream current at creation."""

    def __init__(self, device: Optional[int] = None):
        lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: libknm has no CPU path")
        self.device = torch.cuda.current_device() if device is None else int(device)
        with torch.cuda.device(self.device):
            self.stream = torch.cuda.current_stream()
        h = _vp()
        st = lib.knm_create(ctypes.byref(h), self.device, _vp(self.stream.cuda_stream))
        if st != KNM_OK:
            raise KnmError(st, "knm_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            load_library().knm_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st: int):
        if st != KNM_OK:
            raise KnmError(st, load_library().knm_last_error(self._h).decode())

    def set_cross_term(self, mode):
        """'f16x3' (split-fp16 products on the f16 matrix cores, default) or 'f32' (fp32 MFMA)."""
        code = {"f32": 0, "f16x3": 1}[mode] if isinstance(mode, str) else int(mode)
        self.check(load_library().knm_set_cross_term(self._h, code))

    @property
    def cross_term(self) -> str:
        return {0: "f32", 1: "f16x3"}[load_library().knm_get_cross_term(self._h)]

    def set_kernel(self, kind):
        """'gaussian' (default), 'laplacian', 'matern32' or 'matern52' (dense entry points only)."""
        code = {"gaussian": 0, "laplacian": 1, "matern32": 2, "matern52": 3}[kind] if isinstance(kind, str) else int(kind)
        self.check(load_library().knm_set_kernel(self._h, code))

    def probe_rates(self) -> dict:
        """Sustained instruction rates of this device (knm_probe_rates)."""
        names = ("mfma_f32_tflops", "mfma_f16_const_tflops", "mfma_f16_random_tflops", "exp_tops", "fma_tops") + tuple(
            f"mix{hu}_{what}_clk" for hu in (1, 2, 3) for what in ("both", "valu", "mfma"))
        buf = (_f64 * len(names))()
        self.check(load_library().knm_probe_rates(self._h, buf, len(names)))
        return {k: float(v) for k, v in zip(names, buf)}

    def range_exceeded(self, reset: bool = True) -> int:
        """Operand conversions the split-fp16 cross term had to clamp since the last reset (waits for the stream)."""
        c = _i64(0)
        self.check(load_library().knm_range_exceeded(self._h, ctypes.byref(c), 1 if reset else 0))
        return int(c.value)

    def workspace_held(self) -> int:
        """Device bytes of workspace this context holds now."""
        return int(load_library().knm_workspace_held(self._h))

    def set_sparse_head_limit(self, max_features: int):
        """Sparse inputs: how many of the most frequent features may be handled densely (0: none)."""
        self.check(load_library().knm_set_sparse_head_limit(self._h, int(max_features)))

    def set_pack_limit(self, nbytes: int):
        """Cap on the workspace of the split-fp16 engines' converted operands (0: defaults)."""
        self.check(load_library().knm_set_pack_limit(self._h, int(nbytes)))

    def get_fit_timing(self):
        sec = (_f64 * 4)()
        self.check(load_library().knm_get_fit_timing(self._h, sec))
        return {"precond_s": sec[0], "rhs_s": sec[1], "iterations_s": sec[2], "tail_s": sec[3]}

    # ---- timing -----------------------------------------------------------------------
    def set_timing(self, enabled: bool):
        self.check(load_library().knm_set_timing(self._h, int(enabled)))

    def get_timing(self):
        ms = (_f32 * 4)()
        self.check(load_library().knm_get_timing(self._h, ms))
        return {"row_sweep_ms": ms[0], "col_sweep_ms": ms[1], "merge_ms": ms[2], "total_ms": ms[3]}


_default_ctx = {}


def default_context() -> Context:
    dev = torch.cuda.current_device()
    key = (dev, torch.cuda.current_stream().cuda_stream)
    if key not in _default_ctx:
        _default_ctx[key] = Context(dev)
    return _default_ctx[key]


def _geom(X, C):
    X, n, d, ldx = _points(X, "X")
    C, M, d2, ldc = _points(C, "C")
    if d != d2:
        raise ValueError("X and C must have the same number of features")
    return X, n, d, ldx, C, M, ldc


def knm_v(X, C, sigma: float, V, ctx: Optional[Context] = None) -> torch.Tensor:
    """W = k(X, C) V."""
    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    V, t, sq = _cols(V, M, "V")
    W = torch.empty(n, t, device=X.device, dtype=torch.float32)
    ctx.check(load_library().knm_v(ctx._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc, float(sigma),
                                   V.data_ptr(), t, W.data_ptr()))
    return W[:, 0] if sq else W


def knm_prod(X, C, sigma: float, V, return_w: bool = False, out: Optional[torch.Tensor] = None,
             ctx: Optional[Context] = None):
    """U = K_nm^T (K_nm V); optionally also W = K_nm V."""
    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    V, t, sq = _cols(V, M, "V")
    U = out if out is not None else torch.empty(M, t, device=X.device, dtype=torch.float32)
    W = torch.empty(n, t, device=X.device, dtype=torch.float32) if return_w else None
    ctx.check(load_library().knm_prod(ctx._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc, float(sigma),
                                      V.data_ptr(), t, W.data_ptr() if return_w else None, U.data_ptr()))
    if sq:
        U = U.reshape(M)
        W = W[:, 0] if return_w else None
    return (U, W) if return_w else U


def knm_prod_static(X, C, sigma: float, V, W, U, ctx: Optional[Context] = None) -> None:
    """U = K_nm^T (K_nm V), W = K_nm V into the caller's tensors; the library allocates nothing (its
    workspace is the static scratch array of knm_static_scratch_bytes() bytes)."""
    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    V, t, _ = _cols(V, M, "V")
    for name, T, rows in (("W", W, n), ("U", U, M)):
        if T.dtype != torch.float32 or not T.is_contiguous() or T.numel() != rows * t or T.device != X.device:
            raise ValueError(f"{name} must be a contiguous float32 tensor of {rows} x {t} on the inputs' device")
    ctx.check(load_library().knm_prod_static(ctx._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc, float(sigma),
                                             V.data_ptr(), t, W.data_ptr(), U.data_ptr()))


def knm_static_scratch_bytes() -> int:
    return int(load_library().knm_static_scratch_bytes())


def knm_prod_weighted(X, C, sigma: float, dw, V, ctx: Optional[Context] = None) -> torch.Tensor:
    """U = K_nm^T diag(dw) K_nm V."""
    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    V, t, sq = _cols(V, M, "V")
    dw = _dev_f32(dw, "dw").reshape(n).contiguous()
    U = torch.empty(M, t, device=X.device, dtype=torch.float32)
    ctx.check(load_library().knm_prod_weighted(ctx._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc,
                                               float(sigma), dw.data_ptr(), V.data_ptr(), t, U.data_ptr()))
    return U[:, 0] if sq else U


def knm_t_y(X, C, sigma: float, Y, ctx: Optional[Context] = None) -> torch.Tensor:
    """R = K_nm^T Y."""
    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    Y, t, sq = _cols(Y, n, "Y")
    R = torch.empty(M, t, device=X.device, dtype=torch.float32)
    ctx.check(load_library().knm_t_y(ctx._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc, float(sigma),
                                     Y.data_ptr(), t, R.data_ptr()))
    return R[:, 0] if sq else R


def _csr_parts(A, name: str):
    if not (isinstance(A, torch.Tensor) and A.layout == torch.sparse_csr and A.is_cuda and A.dim() == 2):
        raise TypeError(f"{name} must be a 2-D sparse CSR tensor on the GPU")
    crow, col, val = A.crow_indices(), A.col_indices(), A.values()
    if crow.dtype != torch.int64 or col.dtype != torch.int64 or val.dtype != torch.float32:
        raise TypeError(f"{name} must have int64 indices and float32 values")
    return crow.contiguous(), col.contiguous(), val.contiguous()


def knm_prod_csr(X, C, sigma: float, V, return_w: bool = False, ctx: Optional[Context] = None):
    """U = K^T (K V) for sparse CSR X (n x d) and C (M x d) (float32 values, int64 indices)."""
    ctx = ctx or default_context()
    xr, xc, xv = _csr_parts(X, "X")
    cr, cc, cv = _csr_parts(C, "C")
    n, d = X.shape
    M = C.shape[0]
    if C.shape[1] != d:
        raise ValueError("X and C must have the same number of features")
    V, t, sq = _cols(V, M, "V")
    U = torch.empty(M, t, device=V.device, dtype=torch.float32)
    W = torch.empty(n, t, device=V.device, dtype=torch.float32) if return_w else None
    ctx.check(load_library().knm_prod_csr(ctx._h, xr.data_ptr(), xc.data_ptr(), xv.data_ptr(), n, cr.data_ptr(),
                                          cc.data_ptr(), cv.data_ptr(), M, d, float(sigma), V.data_ptr(), t,
                                          W.data_ptr() if return_w else None, U.data_ptr()))
    if sq:
        U = U[:, 0]
        W = W[:, 0] if return_w else None
    return (U, W) if return_w else U


def knm_v_csr(X, C, sigma: float, V, ctx: Optional[Context] = None) -> torch.Tensor:
    """W = K V for sparse CSR X and C (also the predictor: V = alpha)."""
    ctx = ctx or default_context()
    xr, xc, xv = _csr_parts(X, "X")
    cr, cc, cv = _csr_parts(C, "C")
    n, d = X.shape
    M = C.shape[0]
    if C.shape[1] != d:
        raise ValueError("X and C must have the same number of features")
    V, t, sq = _cols(V, M, "V")
    W = torch.empty(n, t, device=V.device, dtype=torch.float32)
    ctx.check(load_library().knm_v_csr(ctx._h, xr.data_ptr(), xc.data_ptr(), xv.data_ptr(), n, cr.data_ptr(),
                                       cc.data_ptr(), cv.data_ptr(), M, d, float(sigma), V.data_ptr(), t, W.data_ptr()))
    return W[:, 0] if sq else W


def falkon_fit_csr(X, Y, C, sigma: float, lam: float, iters: int, jitter: float = 0.0, return_resid: bool = False,
                   ctx: Optional[Context] = None):
    """falkon_fit for sparse CSR X and C."""
    import numpy as np

    ctx = ctx or default_context()
    xr, xc, xv = _csr_parts(X, "X")
    cr, cc, cv = _csr_parts(C, "C")
    n, d = X.shape
    M = C.shape[0]
    if C.shape[1] != d:
        raise ValueError("X and C must have the same number of features")
    Y, t, sq = _cols(Y, n, "Y")
    alpha = torch.empty(M, t, device=Y.device, dtype=torch.float32)
    resid = np.zeros((iters + 1, t), dtype=np.float64)
    ctx.check(load_library().falkon_fit_csr(ctx._h, xr.data_ptr(), xc.data_ptr(), xv.data_ptr(), n, Y.data_ptr(), t,
                                            cr.data_ptr(), cc.data_ptr(), cv.data_ptr(), M, d, float(sigma), float(lam),
                                            float(jitter), int(iters), alpha.data_ptr(), resid.ctypes.data))
    out = alpha[:, 0] if sq else alpha
    return (out, resid) if return_resid else out


class Preconditioner:
    """Owns the fp64 factors T, A built by precond_build."""

    def __init__(self, C, sigma: float, lam: float, jitter: float = 0.0, ctx: Optional[Context] = None):
        self.ctx = ctx or default_context()
        C, M, d, ldc = _points(C, "C")
        h = _vp()
        bad = _i64(0)
        st = load_library().precond_build(self.ctx._h, C.data_ptr(), M, d, ldc, float(sigma), float(lam),
                                          float(jitter), ctypes.byref(h), ctypes.byref(bad))
        self.bad_pivot = bad.value
        if st != KNM_OK:
            raise KnmError(st, load_library().knm_last_error(self.ctx._h).decode() + f" (pivot {bad.value})")
        self._h = h
        self.M = M

    def factors(self):
        import numpy as np

        T = np.empty((self.M, self.M), dtype=np.float64)
        A = np.empty((self.M, self.M), dtype=np.float64)
        self.ctx.check(load_library().precond_get_factors(self.ctx._h, self._h, T.ctypes.data, A.ctypes.data))
        return T, A

    def block(self, second: bool, row0: int, col0: int, rows: int, cols: int):
        """rows x cols block of T (second=False) or A (second=True) as a numpy array."""
        import numpy as np

        out = np.empty((rows, cols), dtype=np.float64)
        self.ctx.check(load_library().precond_get_block(self.ctx._h, self._h, int(bool(second)), row0, col0, rows,
                                                        cols, out.ctypes.data))
        return out

    def reweight(self, lam: float, dw=None):
        """Rebuild A = chol(T diag(dw) T^T / M + lam I) in place (dw: float64 GPU tensor, M)."""
        ptr = None
        if dw is not None:
            if not (dw.is_cuda and dw.dtype == torch.float64 and dw.numel() == self.M):
                raise TypeError("dw must be a float64 GPU tensor with M entries")
            dw = dw.contiguous()
            ptr = dw.data_ptr()
        bad = _i64(0)
        st = load_library().precond_reweight(self.ctx._h, self._h, float(lam), ptr, ctypes.byref(bad))
        self.bad_pivot = bad.value
        if st != KNM_OK:
            raise KnmError(st, load_library().knm_last_error(self.ctx._h).decode() + f" (pivot {bad.value})")

    def solve(self, b, transpose: bool = False) -> torch.Tensor:
        """T^-1 A^-1 b, or A^-T T^-T b with transpose (b: float64 GPU tensor, M or M x t)."""
        if not (b.is_cuda and b.dtype == torch.float64 and b.shape[0] == self.M):
            raise TypeError("b must be a float64 GPU tensor with M rows")
        b2 = b.reshape(self.M, -1).contiguous()
        out = torch.empty_like(b2)
        self.ctx.check(load_library().precond_solve(self.ctx._h, self._h, int(bool(transpose)), b2.data_ptr(),
                                                    b2.shape[1], out.data_ptr()))
        return out.reshape(b.shape)

    def close(self):
        if getattr(self, "_h", None):
            load_library().precond_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rank_k_update(A, C, alpha: float = 1.0, beta: float = 0.0, form_nt: bool = False, w=None,
                  triangular: bool = False, shift: float = 0.0, ctx: Optional[Context] = None) -> None:
    """Upper triangle of C (n x n) <- alpha a diag(w) a^T + beta C + shift I, in place, fp64 on the matrix cores.

    A and C are float64 GPU tensors read as COLUMN-major storage: a torch tensor of shape (c, r)
    that is contiguous holds an r x c column-major matrix with leading dimension r.  With
    form_nt the operand is n x k (A.shape == (k, n)), otherwise k x n (A.shape == (n, k))."""
    ctx = ctx or default_context()
    for x in (A, C):
        if not (x.is_cuda and x.dtype == torch.float64 and x.dim() == 2 and x.is_contiguous()):
            raise TypeError("A and C must be contiguous 2-D float64 GPU tensors")
    n = C.shape[0]
    if C.shape[1] != n:
        raise ValueError("C must be square")
    if form_nt:
        k, lda = A.shape[0], A.shape[1]
        if A.shape[1] != n:
            raise ValueError("A must hold an n x k column-major matrix")
    else:
        k, lda = A.shape[1], A.shape[1]
        if A.shape[0] != n:
            raise ValueError("A must hold a k x n column-major matrix")
    wp = None
    if w is not None:
        if not (w.is_cuda and w.dtype == torch.float64 and w.numel() == k):
            raise TypeError("w must be a float64 GPU tensor with k entries")
        w = w.contiguous()
        wp = w.data_ptr()
    ctx.check(load_library().precond_rank_k_update(ctx._h, int(bool(form_nt)), n, k, float(alpha), A.data_ptr(),
                                                   max(lda, 1), wp, int(bool(triangular)), float(beta), float(shift),
                                                   C.data_ptr(), max(n, 1)))


def block_product(A, B, C, alpha: float = 1.0, beta: float = 0.0, a_nt: bool = False,
                  ctx: Optional[Context] = None) -> None:
    """C <- alpha op(A) B + beta C in place, fp64 on the matrix cores; op(A) = A^T, or A with a_nt.

    All three are contiguous float64 GPU tensors read as COLUMN-major storage (a torch tensor of
    shape (c, r) holds an r x c matrix): B is k x nj, C is ni x nj, A is k x ni (ni x k with a_nt)."""
    ctx = ctx or default_context()
    for x in (A, B, C):
        if not (x.is_cuda and x.dtype == torch.float64 and x.dim() == 2 and x.is_contiguous()):
            raise TypeError("A, B and C must be contiguous 2-D float64 GPU tensors")
    nj, ni = C.shape
    k = B.shape[1]
    if B.shape[0] != nj or tuple(A.shape) != ((k, ni) if a_nt else (ni, k)):
        raise ValueError("shapes do not match")
    ctx.check(load_library().precond_block_product(ctx._h, int(bool(a_nt)), ni, nj, k, float(alpha), A.data_ptr(),
                                                   max(A.shape[1], 1), B.data_ptr(), max(k, 1), float(beta),
                                                   C.data_ptr(), max(ni, 1)))


def precond_build(C, sigma: float, lam: float, jitter: float = 0.0, ctx: Optional[Context] = None) -> Preconditioner:
    return Preconditioner(C, sigma, lam, jitter, ctx)


def falkon_linop(precond: Preconditioner, X, C, sigma: float, lam: float, beta, dw=None) -> torch.Tensor:
    """Preconditioned operator of Eq. 9 applied to beta (float64, M x t); with dw (float32, n) the
    weighted operator of Alg. 2."""
    ctx = precond.ctx
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    if not (beta.is_cuda and beta.dtype == torch.float64):
        raise TypeError("beta must be a float64 tensor on the GPU")
    sq = beta.dim() == 1
    b2 = beta.reshape(M, -1).contiguous()
    t = b2.shape[1]
    out = torch.empty_like(b2)
    if dw is None:
        ctx.check(load_library().falkon_linop(ctx._h, precond._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc,
                                              float(sigma), float(lam), b2.data_ptr(), t, out.data_ptr()))
    else:
        dw, _, _ = _cols(dw, n, "dw")
        ctx.check(load_library().falkon_linop_weighted(ctx._h, precond._h, X.data_ptr(), n, d, ldx, C.data_ptr(), M,
                                                       ldc, float(sigma), float(lam), dw.data_ptr(), b2.data_ptr(),
                                                       t, out.data_ptr()))
    return out[:, 0] if sq else out


def falkon_fit(X, Y, C, sigma: float, lam: float, iters: int, jitter: float = 0.0, return_resid: bool = False,
               ctx: Optional[Context] = None):
    """alpha (M x t) after exactly `iters` preconditioned CG steps (Alg. 1)."""
    import numpy as np

    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    Y, t, sq = _cols(Y, n, "Y")
    alpha = torch.empty(M, t, device=X.device, dtype=torch.float32)
    resid = np.zeros((iters + 1, t), dtype=np.float64)
    ctx.check(load_library().falkon_fit(ctx._h, X.data_ptr(), n, d, ldx, Y.data_ptr(), t, C.data_ptr(), M, ldc,
                                        float(sigma), float(lam), float(jitter), int(iters), alpha.data_ptr(),
                                        resid.ctypes.data))
    if sq:
        alpha, resid = alpha[:, 0], resid[:, 0]
    return (alpha, resid) if return_resid else alpha


def logfalkon_fit(X, y, C, yC, sigma: float, lambdas, iters, jitter: float = 0.0, return_loss: bool = False,
                  ctx: Optional[Context] = None):
    """alpha (M) after the approximate Newton steps of Alg. 2 for the logistic loss; step k uses
    lambdas[k] and iters[k] CG iterations."""
    import numpy as np

    ctx = ctx or default_context()
    X, n, d, ldx, C, M, ldc = _geom(X, C)
    y, _, _ = _cols(y, n, "y")
    yC, _, _ = _cols(yC, M, "yC")
    lam = np.ascontiguousarray(lambdas, dtype=np.float64)
    its = np.ascontiguousarray(iters, dtype=np.int32)
    if lam.ndim != 1 or lam.shape != its.shape or lam.size == 0:
        raise ValueError("lambdas and iters must be equally long, non-empty sequences")
    alpha = torch.empty(M, device=X.device, dtype=torch.float32)
    loss = np.zeros(lam.size + 1, dtype=np.float64)
    ctx.check(load_library().logfalkon_fit(ctx._h, X.data_ptr(), n, d, ldx, y.data_ptr(), C.data_ptr(), M, ldc,
                                           yC.data_ptr(), float(sigma), lam.ctypes.data, its.ctypes.data,
                                           int(lam.size), float(jitter), alpha.data_ptr(), loss.ctypes.data))
    return (alpha, loss) if return_loss else alpha


def logfalkon_fit_csr(X, y, C, yC, sigma: float, lambdas, iters, jitter: float = 0.0, return_loss: bool = False,
                      ctx: Optional[Context] = None):
    """logfalkon_fit for sparse CSR X and C."""
    import numpy as np

    ctx = ctx or default_context()
    xr, xc, xv = _csr_parts(X, "X")
    cr, cc, cv = _csr_parts(C, "C")
    n, d = X.shape
    M = C.shape[0]
    if C.shape[1] != d:
        raise ValueError("X and C must have the same number of features")
    y, _, _ = _cols(y, n, "y")
    yC, _, _ = _cols(yC, M, "yC")
    lam = np.ascontiguousarray(lambdas, dtype=np.float64)
    its = np.ascontiguousarray(iters, dtype=np.int32)
    if lam.ndim != 1 or lam.shape != its.shape or lam.size == 0:
        raise ValueError("lambdas and iters must be equally long, non-empty sequences")
    alpha = torch.empty(M, device=xv.device, dtype=torch.float32)
    loss = np.zeros(lam.size + 1, dtype=np.float64)
    ctx.check(load_library().logfalkon_fit_csr(ctx._h, xr.data_ptr(), xc.data_ptr(), xv.data_ptr(), n, y.data_ptr(),
                                               cr.data_ptr(), cc.data_ptr(), cv.data_ptr(), M, d, yC.data_ptr(),
                                               float(sigma), lam.ctypes.data, its.ctypes.data, int(lam.size),
                                               float(jitter), alpha.data_ptr(), loss.ctypes.data))
    return (alpha, loss) if return_loss else alpha


def falkon_predict(Xtest, C, sigma: float, alpha, ctx: Optional[Context] = None) -> torch.Tensor:
    """out = k(Xtest, C) alpha (Eq. 4)."""
    ctx = ctx or default_context()
    Xt, n, d, ldx, C, M, ldc = _geom(Xtest, C)
    A, t, sq = _cols(alpha, M, "alpha")
    out = torch.empty(n, t, device=Xt.device, dtype=torch.float32)
    ctx.check(load_library().falkon_predict(ctx._h, Xt.data_ptr(), n, d, ldx, C.data_ptr(), M, ldc, float(sigma),
                                            A.data_ptr(), t, out.data_ptr()))
    return out[:, 0] if sq else out
