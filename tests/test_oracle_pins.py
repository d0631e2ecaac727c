"""Pins for the fp64 CPU oracle: each check ties an oracle function to something other
than itself -- hand values, closed forms, algebraic identities, or an independent
library routine (scikit-learn's RBF kernel, numpy/scipy factorisations and solves).

The paper prints no worked numerical example for this path, so the pins are the
definitions (Section 2, Eq. 4-9, Alg. 1) evaluated where they have a known answer.
"""
import math
import os

import numpy as np
import pytest
import scipy.linalg as sla
from sklearn.metrics.pairwise import rbf_kernel

import oracle

RNG = np.random.default_rng(20200610)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _pts(n, d, scale=1.0, rng=RNG):
    return (scale * rng.standard_normal((n, d))).astype(np.float32)


def _lib_K(X, C, sigma):
    """Independent library evaluation of the Gaussian kernel matrix in fp64."""
    return rbf_kernel(X.astype(np.float64), C.astype(np.float64), gamma=1.0 / (2.0 * sigma * sigma))


# ---------------------------------------------------------------- kernel (Section 2)

def test_gauss_hand_values():
    assert oracle.gauss([0.0], [0.0], 1.0) == 1.0
    # |x - c| = sigma  ->  e^{-1/2}
    assert oracle.gauss([1.5], [4.5], 3.0) == pytest.approx(math.exp(-0.5), rel=1e-15)
    # 3-4-5 triangle, sigma = 5: exp(-25/50)
    assert oracle.gauss([1.0, -2.0], [4.0, 2.0], 5.0) == pytest.approx(math.exp(-0.5), rel=1e-15)
    # the factor is 1/(2 sigma^2), not 1/sigma^2 and not 1/(2 sigma)
    assert oracle.gauss([0.0], [2.0], 2.0) == pytest.approx(math.exp(-0.5), rel=1e-15)
    assert oracle.gauss([0.0, 0.0, 0.0], [1.0, 1.0, 1.0], 0.5) == pytest.approx(math.exp(-6.0), rel=1e-15)


def test_gauss_range_and_underflow():
    X = _pts(40, 5, 3.0)
    K = oracle.kernel_matrix(X, X, 0.7)
    assert np.all(K >= 0.0) and np.all(K <= 1.0)
    assert np.array_equal(np.diag(K), np.ones(40))
    assert np.array_equal(K, K.T)
    far = oracle.gauss([0.0], [1.0e4], 1.0)
    assert far == 0.0 and not math.isnan(far)


def test_two_by_two_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "two_by_two.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = np.array([float(x) for x in v])
    X = np.array([[0.0], [2.0]], dtype=np.float32)
    C = np.array([[1.0], [2.0]], dtype=np.float32)
    v = np.array([1.0, 2.0])
    np.testing.assert_allclose(oracle.kernel_matrix(X, C, 1.0).ravel(), vals["K"], rtol=1e-15)
    np.testing.assert_allclose(oracle.knm_v(X, C, 1.0, v), vals["w"], rtol=1e-15)
    u, w = oracle.knm_prod(X, C, 1.0, v, return_w=True)
    np.testing.assert_allclose(w, vals["w"], rtol=1e-15)
    np.testing.assert_allclose(u, vals["u"], rtol=1e-15)
    # K^T y on a non-symmetric K: a transposed operand would give K y instead
    np.testing.assert_allclose(oracle.knm_t_y(X, C, 1.0, np.array([1.0, 0.0])), vals["K"][:2], rtol=1e-15)


def test_kernel_matrix_matches_library():
    X, C = _pts(57, 7), _pts(23, 7)
    for sigma in (0.5, 2.0, 11.0):
        np.testing.assert_allclose(oracle.kernel_matrix(X, C, sigma), _lib_K(X, C, sigma), rtol=1e-12, atol=1e-300)


# ------------------------------------------------------- products (Section 3.1, Eq. 4)

@pytest.mark.parametrize("n,M,d,t", [(200, 50, 3, 1), (131, 67, 9, 4), (64, 64, 28, 10)])
def test_products_match_explicit_library_matrix(n, M, d, t):
    X, C = _pts(n, d), _pts(M, d)
    sigma = 1.5 * math.sqrt(d)
    K = _lib_K(X, C, sigma)
    V = RNG.standard_normal((M, t))
    Y = RNG.standard_normal((n, t))
    np.testing.assert_allclose(oracle.knm_v(X, C, sigma, V), K @ V, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.knm_t_w(X, C, sigma, Y), K.T @ Y, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.knm_prod(X, C, sigma, V), K.T @ (K @ V), rtol=1e-11, atol=1e-11)
    dw = RNG.uniform(0.1, 2.0, n)
    np.testing.assert_allclose(oracle.knm_prod_weighted(X, C, sigma, dw, V), K.T @ (dw[:, None] * (K @ V)),
                               rtol=1e-11, atol=1e-11)


def test_prod_sigma_to_infinity_closed_form():
    # sigma -> inf: every kernel entry is 1, so u = n (sum_j v_j) 1
    n, M = 300, 41
    X, C = _pts(n, 4), _pts(M, 4)
    v = RNG.standard_normal(M)
    u = oracle.knm_prod(X, C, 1.0e9, v)
    np.testing.assert_allclose(u, np.full(M, n * v.sum()), rtol=1e-12)


def test_prod_unit_vector_returns_gram_column():
    X, C = _pts(90, 3), _pts(17, 3)
    K = _lib_K(X, C, 1.3)
    G = K.T @ K
    for j in (0, 5, 16):
        e = np.zeros(17)
        e[j] = 1.0
        np.testing.assert_allclose(oracle.knm_prod(X, C, 1.3, e), G[:, j], rtol=1e-11)


def test_prod_operator_symmetric_psd_linear():
    X, C = _pts(150, 6), _pts(30, 6)
    s = 2.0
    v1, v2 = RNG.standard_normal(30), RNG.standard_normal(30)
    p1, w1 = oracle.knm_prod(X, C, s, v1, return_w=True)
    p2 = oracle.knm_prod(X, C, s, v2)
    assert v2 @ p1 == pytest.approx(v1 @ p2, rel=1e-12)
    assert v1 @ p1 == pytest.approx(w1 @ w1, rel=1e-12)
    np.testing.assert_allclose(oracle.knm_prod(X, C, s, 2.0 * v1 - 3.0 * v2), 2.0 * p1 - 3.0 * p2, rtol=1e-10, atol=1e-10)


def test_prod_row_permutation_and_blocking_invariance():
    X, C = _pts(120, 5), _pts(25, 5)
    v = RNG.standard_normal(25)
    y = RNG.standard_normal(120)
    perm = RNG.permutation(120)
    np.testing.assert_allclose(oracle.knm_prod(X[perm], C, 1.7, v), oracle.knm_prod(X, C, 1.7, v), rtol=1e-12)
    np.testing.assert_allclose(oracle.knm_t_y(X[perm], C, 1.7, y[perm]), oracle.knm_t_y(X, C, 1.7, y), rtol=1e-12)
    # sum over row batches equals the unbatched product (the blockwise formula)
    parts = sum(oracle.knm_prod(X[a:b], C, 1.7, v) for a, b in ((0, 37), (37, 38), (38, 120)))
    np.testing.assert_allclose(parts, oracle.knm_prod(X, C, 1.7, v), rtol=1e-12)


def test_kronecker_structure_on_grids():
    # On product grids the Gaussian kernel factorises: K = K1 (x) K2, so
    # K vec(V) = vec(K1 V K2^T) with 1-D kernels K1, K2 built from hand formulas.
    a = np.array([0.0, 0.5, 2.0, 3.5], dtype=np.float32)
    b = np.array([-1.0, 0.25, 1.0], dtype=np.float32)
    ca = np.array([0.25, 3.0], dtype=np.float32)
    cb = np.array([0.0, 0.5, 0.75, 2.0], dtype=np.float32)
    sigma = 1.25
    X = np.array([[p, q] for p in a for q in b], dtype=np.float32)
    C = np.array([[p, q] for p in ca for q in cb], dtype=np.float32)
    K1 = np.exp(-(a[:, None].astype(float) - ca[None, :]) ** 2 / (2 * sigma ** 2))
    K2 = np.exp(-(b[:, None].astype(float) - cb[None, :]) ** 2 / (2 * sigma ** 2))
    V = RNG.standard_normal((len(ca), len(cb)))
    W = K1 @ V @ K2.T
    np.testing.assert_allclose(oracle.knm_v(X, C, sigma, V.ravel()), W.ravel(), rtol=1e-12)
    U = K1.T @ W @ K2
    np.testing.assert_allclose(oracle.knm_prod(X, C, sigma, V.ravel()), U.ravel(), rtol=1e-12)


# ------------------------------------------------ factorisations and solves (Eq. 6, 7)

def test_chol_and_solves_match_library():
    M = 60
    B = RNG.standard_normal((M, M))
    G = B @ B.T + M * np.eye(M)
    R = oracle.chol_upper(G)
    assert np.array_equal(np.tril(R, -1), np.zeros((M, M)))
    np.testing.assert_allclose(R, np.linalg.cholesky(G).T, rtol=1e-11, atol=1e-12)
    rhs = RNG.standard_normal((M, 3))
    np.testing.assert_allclose(oracle.solve_upper(R, rhs), sla.solve_triangular(R, rhs, lower=False), rtol=1e-10)
    np.testing.assert_allclose(oracle.solve_upper(R, rhs, trans=True),
                               sla.solve_triangular(R, rhs, lower=False, trans="T"), rtol=1e-10)
    with pytest.raises(np.linalg.LinAlgError):
        oracle.chol_upper(np.array([[1.0, 2.0], [2.0, 1.0]]))


def test_rank_k_upper_against_element_sums_and_a_cholesky_step():
    # element by element on a tiny case, every option at once
    n, k = 5, 4
    a = RNG.standard_normal((n, k))
    w = RNG.random(k) + 0.5
    C0 = RNG.standard_normal((n, n))
    got = oracle.rank_k_upper(a, C0, alpha=-0.7, beta=1.0, w=w, shift=0.25)
    for i in range(n):
        for j in range(n):
            if i <= j:
                want = -0.7 * sum(w[q] * a[i, q] * a[j, q] for q in range(k)) + C0[i, j] + (0.25 if i == j else 0.0)
            else:
                want = C0[i, j]  # the strict lower triangle is left alone
            assert got[i, j] == pytest.approx(want, rel=1e-13, abs=1e-13)
    # beta = 0 ignores C0's upper triangle; a triangular operand drops a[i, q], q < i
    sq = RNG.standard_normal((n, n))
    got = oracle.rank_k_upper(sq, None, triangular=True)
    np.testing.assert_allclose(got, np.triu(np.triu(sq) @ np.triu(sq).T), rtol=1e-13, atol=1e-14)
    # one block step of the factorisation: with R = chol(G), R11 and R12 its first block row,
    # G22 - R12^T R12 is the matrix whose factor is R22 (Sec. 4, block Cholesky paragraph)
    M, b = 40, 12
    B = RNG.standard_normal((M, M))
    G = B @ B.T + M * np.eye(M)
    R = np.linalg.cholesky(G).T
    S = oracle.rank_k_upper(R[:b, b:].T, G[b:, b:], alpha=-1.0, beta=1.0)
    S = np.triu(S) + np.triu(S, 1).T
    np.testing.assert_allclose(np.linalg.cholesky(S).T, R[b:, b:], rtol=1e-10, atol=1e-12)


def test_preconditioner_identities():
    M, d, sigma, lam, n = 80, 3, 0.6, 1e-3, 1000
    C = _pts(M, d)
    T, A = oracle.precond(C, sigma, lam)
    K = _lib_K(C, C, sigma)
    assert np.array_equal(np.tril(T, -1), np.zeros((M, M))) and np.array_equal(np.tril(A, -1), np.zeros((M, M)))
    np.testing.assert_allclose(T.T @ T, K, rtol=0, atol=1e-12)
    np.testing.assert_allclose(A.T @ A, T @ T.T / M + lam * np.eye(M), rtol=0, atol=1e-12)
    np.testing.assert_allclose(T, np.linalg.cholesky(K).T, rtol=1e-7, atol=1e-10)
    # Eq. 6-7: P P^T = (n/M K^2 + lambda n K)^-1 with P = T^-1 A^-1 / sqrt(n)
    P = np.linalg.inv(T) @ np.linalg.inv(A) / math.sqrt(n)
    H = n / M * K @ K + lam * n * K
    np.testing.assert_allclose(P @ P.T @ H, np.eye(M), rtol=0, atol=1e-5)
    # jitter is added to the diagonal of K_MM before the first factorisation
    Tj, _ = oracle.precond(C, sigma, lam, jitter=0.5)
    np.testing.assert_allclose(Tj.T @ Tj, K + 0.5 * np.eye(M), rtol=0, atol=1e-12)


# ------------------------------------------------------------ LinOp and the fit (Alg. 1)

def test_linop_matches_eq8_and_eq9_dense():
    n, M, d, sigma, lam = 140, 24, 2, 0.8, 1e-2
    X, C = _pts(n, d), _pts(M, d)
    T, A = oracle.precond(C, sigma, lam)
    Knm, Kmm = _lib_K(X, C, sigma), _lib_K(C, C, sigma)
    Ti, Ai = np.linalg.inv(T), np.linalg.inv(A)
    beta = RNG.standard_normal((M, 2))
    H = Knm.T @ Knm + lam * n * Kmm
    eq8 = Ai.T @ Ti.T @ H @ Ti @ Ai @ beta
    eq9 = Ai.T @ (Ti.T @ Knm.T @ Knm @ Ti + lam * n * np.eye(M)) @ Ai @ beta
    got = oracle.linop(X, C, sigma, lam, T, A, beta)
    np.testing.assert_allclose(got, eq9, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(got, eq8, rtol=1e-7, atol=1e-7)
    # the operator is symmetric (needed for CG)
    b2 = RNG.standard_normal((M, 2))
    g2 = oracle.linop(X, C, sigma, lam, T, A, b2)
    assert np.sum(b2[:, 0] * got[:, 0]) == pytest.approx(np.sum(beta[:, 0] * g2[:, 0]), rel=1e-9)


def test_linop_is_n_times_identity_when_centres_are_the_data():
    n, d, sigma, lam = 50, 2, 0.5, 1e-2
    X = _pts(n, d, 2.0)
    T, A = oracle.precond(X, sigma, lam)
    beta = RNG.standard_normal(n)
    np.testing.assert_allclose(oracle.linop(X, X, sigma, lam, T, A, beta), n * beta, rtol=1e-8, atol=1e-8)


def test_fit_with_all_points_as_centres_is_exact_krr_after_one_step():
    n, d, sigma, lam = 60, 2, 0.5, 1e-3
    X = _pts(n, d, 2.0)
    y = np.sin(X.astype(np.float64).sum(1)) + 0.1 * RNG.standard_normal(n)
    alpha = oracle.falkon_fit(X, y, X, sigma, lam, iters=1)
    K = _lib_K(X, X, sigma)
    exact = np.linalg.solve(K + n * lam * np.eye(n), y)
    np.testing.assert_allclose(K @ alpha, K @ exact, rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(alpha, exact, rtol=1e-5, atol=1e-6)
    # interpolation limit: tiny lambda, distinct points -> predictions reproduce y
    a0 = oracle.falkon_fit(X, y, X, sigma, 1e-13, iters=2)
    np.testing.assert_allclose(oracle.falkon_predict(X, X, sigma, a0), y, rtol=0, atol=1e-5)


@pytest.mark.parametrize("t", [1, 3])
def test_fit_converges_to_dense_nystrom_solution(t):
    n, M, d, sigma, lam = 400, 30, 2, 0.7, 1e-3
    X = _pts(n, d)
    C = X[RNG.choice(n, M, replace=False)]
    Y = RNG.standard_normal((n, t))
    Knm, Kmm = _lib_K(X, C, sigma), _lib_K(C, C, sigma)
    # Eq. 5 is the normal equation of min |Knm a - Y|^2 + lam n a^T Kmm a; solve that
    # least-squares problem in stacked form (better conditioned than Eq. 5 itself).
    Rm = np.linalg.cholesky(Kmm + 1e-14 * np.eye(M)).T
    stacked = np.vstack([Knm, math.sqrt(lam * n) * Rm])
    dense = np.linalg.lstsq(stacked, np.vstack([Y, np.zeros((M, t))]), rcond=None)[0]
    iters = 2 * M  # rounding delays CG's finite termination a little past M steps
    alpha, resid = oracle.falkon_fit(X, Y, C, sigma, lam, iters=iters, return_resid=True)
    np.testing.assert_allclose(Knm @ alpha, Knm @ dense, rtol=1e-7, atol=1e-9)
    Xt = _pts(37, d)
    np.testing.assert_allclose(oracle.falkon_predict(Xt, C, sigma, alpha), _lib_K(Xt, C, sigma) @ alpha, rtol=1e-9, atol=1e-12)
    assert resid.shape == (iters + 1, t)
    assert np.all(resid[-1] < 1e-8 * resid[0])
    # residual 0 is the norm of the preconditioned right-hand side A^-T T^-T K^T Y
    T, A = oracle.precond(C, sigma, lam)
    rhs = sla.solve_triangular(A, sla.solve_triangular(T, Knm.T @ Y, trans="T"), trans="T")
    np.testing.assert_allclose(resid[0], np.linalg.norm(rhs, axis=0), rtol=1e-9)


def test_fit_few_iterations_match_library_cg_iterates():
    # k steps of the oracle's CG equal k steps of textbook CG written with dense
    # library matrices on the same preconditioned system (start 0, no early exit).
    n, M, d, sigma, lam, k = 300, 40, 3, 1.0, 1e-4, 4
    X = _pts(n, d)
    C = X[:M]
    y = RNG.standard_normal(n)
    T, A = oracle.precond(C, sigma, lam)
    Knm = _lib_K(X, C, sigma)
    Ti, Ai = np.linalg.inv(T), np.linalg.inv(A)
    Bm = Ti @ Ai
    Hop = Bm.T @ (Knm.T @ Knm) @ Bm + lam * n * Ai.T @ Ai
    b = Bm.T @ Knm.T @ y
    x = np.zeros(M)
    r = b.copy()
    p = r.copy()
    for _ in range(k):
        q = Hop @ p
        a = (r @ r) / (p @ q)
        x += a * p
        rn = r - a * q
        p = rn + (rn @ rn) / (r @ r) * p
        r = rn
    alpha = oracle.falkon_fit(X, y, C, sigma, lam, iters=k)
    np.testing.assert_allclose(Knm @ alpha, Knm @ (Bm @ x), rtol=1e-6, atol=1e-8)


# ---------------------------------------------------------------- second kernel family (Laplacian)

def test_laplacian_hand_values_and_library():
    from scipy.spatial.distance import cdist

    with oracle.kernel("laplacian"):
        assert oracle.gauss([0.0], [0.0], 1.0) == 1.0
        # 3-4-5 triangle, sigma = 2.5: exp(-5 / 2.5); the Gaussian value would be exp(-2) too only for
        # sigma^2 = 6.25, so a second point with another distance separates the two forms
        assert oracle.gauss([1.0, -2.0], [4.0, 2.0], 2.5) == pytest.approx(math.exp(-2.0), rel=1e-15)
        assert oracle.gauss([0.0], [3.0], 2.0) == pytest.approx(math.exp(-1.5), rel=1e-15)
        X, C = _pts(57, 9), _pts(23, 9)
        D = cdist(X.astype(np.float64), C.astype(np.float64), metric="euclidean")
        assert np.allclose(oracle.kernel_matrix(X, C, 1.7), np.exp(-D / 1.7), rtol=1e-13, atol=0)
    # the setting ends with the block
    assert oracle.gauss([0.0], [3.0], 2.0) == pytest.approx(math.exp(-9.0 / 8.0), rel=1e-15)


def test_laplacian_setting_reaches_every_product_and_the_fit():
    from scipy.spatial.distance import cdist

    n, M, d, t, sigma, lam = 300, 40, 5, 2, 2.0, 1e-3
    X = _pts(n, d)
    C = X[RNG.choice(n, M, replace=False)].copy()
    V = RNG.standard_normal((M, t))
    Y = RNG.standard_normal((n, t))
    K = np.exp(-cdist(X.astype(np.float64), C.astype(np.float64)) / sigma)
    Kmm = np.exp(-cdist(C.astype(np.float64), C.astype(np.float64)) / sigma)
    with oracle.kernel("laplacian"):
        assert np.allclose(oracle.knm_v(X, C, sigma, V), K @ V, rtol=1e-12, atol=1e-12)
        assert np.allclose(oracle.knm_t_w(X, C, sigma, Y), K.T @ Y, rtol=1e-12, atol=1e-12)
        assert np.allclose(oracle.knm_prod(X, C, sigma, V), K.T @ (K @ V), rtol=1e-12, atol=1e-10)
        T, A = oracle.precond(C, sigma, lam)
        assert np.allclose(T.T @ T, Kmm, rtol=1e-10, atol=1e-12)
        # converged fit = dense Nystrom solution of Eq. 5-6 with the same kernel
        alpha = oracle.falkon_fit(X, Y, C, sigma, lam, 40)
        H = K.T @ K + lam * n * Kmm
        ref = sla.solve(H, K.T @ Y, assume_a="sym")
        assert np.linalg.norm(K @ alpha - K @ ref) <= 1e-6 * np.linalg.norm(K @ ref)


@pytest.mark.parametrize("name,nu", [("matern32", 1.5), ("matern52", 2.5)])
def test_matern_hand_values_and_library(name, nu):
    from sklearn.gaussian_process.kernels import Matern

    with oracle.kernel(name):
        assert oracle.gauss([0.0], [0.0], 1.0) == 1.0
        # r = sigma: u = sqrt(2 nu)
        u = math.sqrt(2.0 * nu)
        want = (1.0 + u) * math.exp(-u) if nu == 1.5 else (1.0 + u + u * u / 3.0) * math.exp(-u)
        assert oracle.gauss([1.0, -2.0], [4.0, 2.0], 5.0) == pytest.approx(want, rel=1e-15)
        X, C = _pts(41, 6), _pts(17, 6)
        lib = Matern(length_scale=1.3, nu=nu)(X.astype(np.float64), C.astype(np.float64))
        assert np.allclose(oracle.kernel_matrix(X, C, 1.3), lib, rtol=1e-12, atol=0)
        # the setting reaches the products
        V = RNG.standard_normal((17, 2))
        assert np.allclose(oracle.knm_prod(X, C, 1.3, V), lib.T @ (lib @ V), rtol=1e-12, atol=1e-12)
    assert oracle.gauss([0.0], [3.0], 2.0) == pytest.approx(math.exp(-9.0 / 8.0), rel=1e-15)
