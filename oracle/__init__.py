"""fp64 CPU oracle for the Nystrom kernel ridge hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``knm_oracle.c`` (plain C, fp64, direct differences).  Only
tests, the smoke check and the CPU-baseline leg of the benchmark may import this
package; the GPU library never does, and nothing here imports the GPU package.

Arrays: data points ``X`` (n x d) and centres ``C`` (M x d) are float32 (the bits the
GPU sees); vectors are float64, shaped (rows, t) or (rows,) for t = 1.
"""
from __future__ import annotations

import contextlib
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
        lib.orc_set_kernel.argtypes = [_int]
        lib.orc_set_kernel.restype = _int
        lib.orc_get_kernel.restype = _int
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


KERNELS = {"gaussian": 0, "laplacian": 1, "matern32": 2, "matern52": 3}


@contextlib.contextmanager
def kernel(name: str):
    """Evaluate everything inside the block with the named kernel: "gaussian" (the paper's,
    Section 2: exp(-|x - c|^2 / (2 sigma^2))), or one of the kernels of r = |x - c| in textbook form
    (the paper's method takes any positive-definite kernel but writes out only the Gaussian one):
    "laplacian" exp(-r / sigma); "matern32" (1 + u) exp(-u), u = sqrt(3) r / sigma; "matern52"
    (1 + u + u^2 / 3) exp(-u), u = sqrt(5) r / sigma."""
    lib = _load()
    before = lib.orc_get_kernel()
    if lib.orc_set_kernel(KERNELS[name]) != 0:
        raise ValueError(name)
    try:
        yield
    finally:
        lib.orc_set_kernel(before)


def gauss(x, c, sigma: float) -> float:
    """k(x, c) of the kernel in force (Gaussian unless inside `kernel("laplacian")`)."""
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


def rank_k_upper(a, C0=None, alpha: float = 1.0, beta: float = 0.0, w=None, shift: float = 0.0,
                 triangular: bool = False) -> np.ndarray:
    """Upper triangle of alpha a diag(w) a^T + beta C0 + shift I for a (n x k): the trailing
    update of the block Cholesky column step (Sec. 4, block Cholesky paragraph) when
    a = (block row of the factor)^T, alpha = -1, beta = 1, and the product T diag(w) T^T of
    the (weighted) preconditioner when a = T (Alg. 1; Alg. 2, WeightedPreconditioner).
    With `triangular` the entries a[i, q], q < i, count as zero.  The strict lower triangle
    of the result is C0's (zero without C0): the operation leaves it alone."""
    a = np.array(a, dtype=np.float64, copy=True)
    n, k = a.shape
    if triangular:
        a = np.triu(a)
    ww = np.ones(k) if w is None else np.asarray(w, dtype=np.float64)
    full = alpha * (a * ww[None, :]) @ a.T + shift * np.eye(n)
    out = np.zeros((n, n)) if C0 is None else np.array(C0, dtype=np.float64, copy=True)
    iu = np.triu_indices(n)
    out[iu] = full[iu] + (beta * out[iu] if beta != 0.0 else 0.0)
    return out


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


# ---- logistic loss (Appendix "Logistic Falkon Algorithm", Alg. 2) -------------------------
#
# Reading of Alg. 2 used here (the listing's right-hand side and the text's equation both
# leave terms out; the Newton schedule mu_0, q is not in the paper, so the caller gives the
# sequence of regularisers and iteration counts):
#   objective   J(alpha) = 1/n sum_i l(z_i, y_i) + mu/2 alpha^T (K_MM + eps I) alpha,  z = K_nm alpha,
#               l(z, y) = log(1 + exp(-y z)),  y in {-1, +1};
#   one call of WeightedFalkon(mu, t, alpha_0) = one approximate Newton step: with
#   g_i = l'(z_i, y_i), D = diag l''(z_i, y_i) at alpha_0, t conjugate-gradient iterations from
#   zero on the preconditioned Newton system
#       P^T (K_nm^T D K_nm + mu n (K_MM + eps I)) P beta = -P^T (K_nm^T g + mu n (K_MM + eps I) alpha_0),
#   P = T^-1 A^-1, then alpha_1 = alpha_0 + P beta  (the operator is LinOp of Alg. 2 as printed);
#   WeightedPreconditioner: T^T T = K_MM + eps I, A^T A = T Dm T^T / M + mu I with
#   Dm = diag l''((K_MM alpha_0)_j, (y_m)_j) at the centres, as printed.

def logistic_terms(z, y):
    """Loss, first and second derivative in z of log(1 + exp(-y z)), elementwise, fp64."""
    z = np.asarray(z, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    m = y * z
    loss = np.logaddexp(0.0, -m)
    s = 0.5 * (1.0 - np.tanh(0.5 * m))  # sigma(-m), stable for either sign
    return loss, -y * s, s * (1.0 - s)


def precond_weighted(C, sigma: float, lam: float, jitter: float, dm):
    """T^T T = K_MM + jitter I;  A^T A = T diag(dm) T^T / M + lam I  (WeightedPreconditioner)."""
    C = _pts(C)
    M = C.shape[0]
    dm = np.asarray(dm, dtype=np.float64).reshape(M)
    T = chol_upper(kernel_matrix(C, C, sigma) + jitter * np.eye(M))
    G = np.zeros((M, M))
    for i in range(M):          # G = T diag(dm) T^T / M, entry by entry of the definition
        G[i, :] = (T[i, :] * dm) @ T.T / M
    A = chol_upper(G + lam * np.eye(M))
    return T, A


def linop_weighted(X, C, sigma: float, lam: float, T, A, dw, beta) -> np.ndarray:
    """A^-T ( T^-T K^T D K T^-1 A^-1 beta + lam n A^-1 beta )  (LinOp of Alg. 2), t = 1."""
    X, C, _ = _geom(X, C)
    v = solve_upper(A, np.asarray(beta, dtype=np.float64).reshape(-1))
    u = solve_upper(T, v)
    c = knm_prod_weighted(X, C, sigma, dw, u)
    w = solve_upper(T, np.asarray(c).reshape(-1), trans=True)
    return solve_upper(A, w + lam * X.shape[0] * v, trans=True)


def logfalkon_fit(X, y, C, yC, sigma: float, lambdas, iters, jitter: float = 0.0,
                  return_loss: bool = False):
    """Approximate Newton method of Alg. 2 with the reading above.  lambdas[k], iters[k]:
    regulariser and conjugate-gradient iterations of Newton step k.  Returns alpha (M,), and
    with return_loss the mean logistic loss before each step and after the last."""
    X, C, _ = _geom(X, C)
    n, M = X.shape[0], C.shape[0]
    y = np.asarray(y, dtype=np.float64).reshape(n)
    yC = np.asarray(yC, dtype=np.float64).reshape(M)
    alpha = np.zeros(M)
    losses = []
    Kmm = kernel_matrix(C, C, sigma)
    for mu, t in zip(lambdas, iters):
        z = knm_v(X, C, sigma, alpha)
        zc = Kmm @ alpha
        loss, g, dw = logistic_terms(z, y)
        losses.append(float(loss.mean()))
        _, _, dm = logistic_terms(zc, yC)
        T, A = precond_weighted(C, sigma, mu, jitter, dm)
        rhs = -(knm_t_w(X, C, sigma, g) + mu * n * (zc + jitter * alpha))
        r = solve_upper(A, solve_upper(T, rhs, trans=True), trans=True)
        beta = np.zeros(M)
        p = r.copy()
        rho = float(r @ r)
        for _ in range(int(t)):                      # Hestenes-Stiefel, from zero, t steps
            q = linop_weighted(X, C, sigma, mu, T, A, dw, p)
            pq = float(p @ q)
            a = rho / pq if pq != 0.0 else 0.0
            beta += a * p
            r -= a * q
            rho_new = float(r @ r)
            p = r + (rho_new / rho if rho != 0.0 else 0.0) * p
            rho = rho_new
        alpha = alpha + solve_upper(T, solve_upper(A, beta))
    loss, _, _ = logistic_terms(knm_v(X, C, sigma, alpha), y)
    losses.append(float(loss.mean()))
    return (alpha, np.array(losses)) if return_loss else alpha
