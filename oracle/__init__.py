"""fp64 CPU oracle for the Nystrom kernel ridge hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``knm_oracle.c`` (plain C, fp64, direct differences).  Only
tests, the smoke check and the CPU-baseline leg of the benchmark may import this
package; the GPU library never does, and nothing here imports the GPU package.

Arrays: data points ``X`` (n x d) and centres ``C`` (M x d) are float32 (the bits the
GPU sees); vectors are float64, shaped (rows, t) or (rows,) for t = 1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "knm_oracle.c")
_LIB = os.path.join(_HERE, "libknm_oracle.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64
_int = ctypes.c_int
_dbl = ctypes.c_double


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        pts = [_f32p, _i64, _int, _i64, _f32p, _i64, _i64, _dbl]  # X n d ldx C M ldc sigma
        lib.orc_num_threads.restype = _int
        lib.orc_gauss.restype = _dbl
        lib.orc_gauss.argtypes = [_f32p, _f32p, _int, _dbl]
        lib.orc_kernel_matrix.argtypes = pts + [_f64p]
        lib.orc_knm_v.argtypes = pts + [_f64p, _int, _f64p]
        lib.orc_knm_t_w.argtypes = pts + [_f64p, _int, _f64p]
        lib.orc_knm_prod.argtypes = pts + [_f64p, _int, _f64p, _f64p]
        lib.orc_knm_prod_weighted.argtypes = pts + [_f64p, _f64p, _int, _f64p, _f64p]
        lib.orc_chol_upper.restype = _i64
        lib.orc_chol_upper.argtypes = [_f64p, _i64]
        lib.orc_solve_upper.argtypes = [_f64p, _i64, _int, _f64p, _int]
        lib.orc_precond.restype = _i64
        lib.orc_precond.argtypes = [_f32p, _i64, _int, _i64, _dbl, _dbl, _dbl, _f64p, _f64p]
        lib.orc_linop.argtypes = pts + [_dbl, _f64p, _f64p, _f64p, _int, _f64p, _f64p, _f64p]
        lib.orc_falkon_fit.restype = _i64
        lib.orc_falkon_fit.argtypes = [_f32p, _i64, _int, _i64, _f64p, _int, _f32p, _i64, _i64,
                                       _dbl, _dbl, _dbl, _int, _f64p, _f64p]
        lib.orc_falkon_predict.argtypes = pts + [_f64p, _int, _f64p]
        _lib = lib
    return _lib


def _pts(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim != 2:
        raise ValueError("point sets must be 2-D (rows x d)")
    return a


def _vec(a, rows: int):
    a = np.asarray(a, dtype=np.float64)
    squeeze = a.ndim == 1
    a = np.ascontiguousarray(a.reshape(rows, -1))
    return a, squeeze


def _p32(a):
    return a.ctypes.data_as(_f32p)


def _p64(a):
    return a.ctypes.data_as(_f64p)


def _geom(X, C):
    X, C = _pts(X), _pts(C)
    if X.shape[1] != C.shape[1]:
        raise ValueError("X and C must have the same number of features")
    return X, C, (_p32(X), X.shape[0], X.shape[1], X.shape[1], _p32(C), C.shape[0], C.shape[1])


def num_threads() -> int:
    return int(_load().orc_num_threads())


def gauss(x, c, sigma: float) -> float:
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    c = np.ascontiguousarray(c, dtype=np.float32).ravel()
    return float(_load().orc_gauss(_p32(x), _p32(c), x.size, float(sigma)))


def kernel_matrix(X, C, sigma: float) -> np.ndarray:
    X, C, g = _geom(X, C)
    K = np.empty((X.shape[0], C.shape[0]), dtype=np.float64)
    _load().orc_kernel_matrix(*g, float(sigma), _p64(K))
    return K


def knm_v(X, C, sigma: float, V) -> np.ndarray:
    X, C, g = _geom(X, C)
    V, sq = _vec(V, C.shape[0])
    W = np.empty((X.shape[0], V.shape[1]), dtype=np.float64)
    _load().orc_knm_v(*g, float(sigma), _p64(V), V.shape[1], _p64(W))
    return W[:, 0] if sq else W


def knm_t_w(X, C, sigma: float, Wv) -> np.ndarray:
    X, C, g = _geom(X, C)
    Wv, sq = _vec(Wv, X.shape[0])
    U = np.empty((C.shape[0], Wv.shape[1]), dtype=np.float64)
    _load().orc_knm_t_w(*g, float(sigma), _p64(Wv), Wv.shape[1], _p64(U))
    return U[:, 0] if sq else U


knm_t_y = knm_t_w


def knm_prod(X, C, sigma: float, V, return_w: bool = False):
    X, C, g = _geom(X, C)
    V, sq = _vec(V, C.shape[0])
    t = V.shape[1]
    W = np.empty((X.shape[0], t), dtype=np.float64)
    U = np.empty((C.shape[0], t), dtype=np.float64)
    _load().orc_knm_prod(*g, float(sigma), _p64(V), t, _p64(W), _p64(U))
    if sq:
        U, W = U[:, 0], W[:, 0]
    return (U, W) if return_w else U


def knm_prod_weighted(X, C, sigma: float, dw, V) -> np.ndarray:
    X, C, g = _geom(X, C)
    V, sq = _vec(V, C.shape[0])
    t = V.shape[1]
    dw = np.ascontiguousarray(dw, dtype=np.float64).ravel()
    if dw.size != X.shape[0]:
        raise ValueError("dw must have one weight per data point")
    W = np.empty((X.shape[0], t), dtype=np.float64)
    U = np.empty((C.shape[0], t), dtype=np.float64)
    _load().orc_knm_prod_weighted(*g, float(sigma), _p64(dw), _p64(V), t, _p64(W), _p64(U))
    return U[:, 0] if sq else U


def chol_upper(G) -> np.ndarray:
    R = np.array(G, dtype=np.float64, order="C", copy=True)
    info = _load().orc_chol_upper(_p64(R), R.shape[0])
    if info:
        raise np.linalg.LinAlgError(f"pivot {info} not positive")
    return R


def solve_upper(R, B, trans: bool = False) -> np.ndarray:
    R = np.ascontiguousarray(R, dtype=np.float64)
    Z, sq = _vec(np.array(B, dtype=np.float64, copy=True), R.shape[0])
    _load().orc_solve_upper(_p64(R), R.shape[0], int(trans), _p64(Z), Z.shape[1])
    return Z[:, 0] if sq else Z


def precond(C, sigma: float, lam: float, jitter: float = 0.0):
    C = _pts(C)
    M = C.shape[0]
    T = np.empty((M, M), dtype=np.float64)
    A = np.empty((M, M), dtype=np.float64)
    info = _load().orc_precond(_p32(C), M, C.shape[1], C.shape[1], float(sigma), float(lam),
                               float(jitter), _p64(T), _p64(A))
    if info:
        raise np.linalg.LinAlgError(f"preconditioner Cholesky failed, info={info}")
    return T, A


def linop(X, C, sigma: float, lam: float, T, A, beta) -> np.ndarray:
    X, C, g = _geom(X, C)
    M = C.shape[0]
    beta, sq = _vec(beta, M)
    t = beta.shape[1]
    T = np.ascontiguousarray(T, dtype=np.float64)
    A = np.ascontiguousarray(A, dtype=np.float64)
    ww = np.empty((X.shape[0], t), dtype=np.float64)
    wm = np.empty((2 * M, t), dtype=np.float64)
    out = np.empty((M, t), dtype=np.float64)
    _load().orc_linop(*g, float(sigma), float(lam), _p64(T), _p64(A), _p64(beta), t,
                      _p64(ww), _p64(wm), _p64(out))
    return out[:, 0] if sq else out


def falkon_fit(X, Y, C, sigma: float, lam: float, iters: int, jitter: float = 0.0,
               return_resid: bool = False):
    X, C, _ = _geom(X, C)
    Y, sq = _vec(Y, X.shape[0])
    t = Y.shape[1]
    alpha = np.zeros((C.shape[0], t), dtype=np.float64)
    resid = np.zeros((iters + 1, t), dtype=np.float64)
    info = _load().orc_falkon_fit(_p32(X), X.shape[0], X.shape[1], X.shape[1], _p64(Y), t,
                                  _p32(C), C.shape[0], C.shape[1], float(sigma), float(lam),
                                  float(jitter), int(iters), _p64(alpha), _p64(resid))
    if info:
        raise np.linalg.LinAlgError(f"preconditioner Cholesky failed, info={info}")
    if sq:
        alpha, resid = alpha[:, 0], resid[:, 0]
    return (alpha, resid) if return_resid else alpha


def falkon_predict(Xtest, C, sigma: float, alpha) -> np.ndarray:
    return knm_v(Xtest, C, sigma, alpha)
