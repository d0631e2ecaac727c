"""Pins of the oracle's logistic-loss functions (Appendix "Logistic Falkon Algorithm", Alg. 2)
to things other than itself: closed forms and finite differences of the loss, dense library
linear algebra for the weighted preconditioner and operator, a dense Newton step, and a
general-purpose optimiser for the minimiser the Newton iteration must reach.  CPU only.
"""
import numpy as np
import scipy.linalg as sla
from scipy.optimize import minimize
from sklearn.metrics.pairwise import rbf_kernel

import oracle


def _problem(n=260, M=36, d=3, seed=0):
    g = np.random.default_rng(seed)
    X = g.standard_normal((n, d)).astype(np.float32)
    idx = g.choice(n, M, replace=False)
    w = g.standard_normal(d)
    y = np.sign(X @ w + 0.4 * g.standard_normal(n))
    y[y == 0] = 1.0
    return X, y, X[idx].copy(), y[idx].copy()


def _dense(X, C, sigma):
    gam = 1.0 / (2.0 * sigma * sigma)
    return rbf_kernel(X.astype(np.float64), C.astype(np.float64), gamma=gam)


def test_logistic_terms_closed_forms_and_finite_differences():
    loss, g, dw = oracle.logistic_terms(np.zeros(2), np.array([1.0, -1.0]))
    assert np.allclose(loss, np.log(2.0)) and np.allclose(g, [-0.5, 0.5]) and np.allclose(dw, 0.25)
    z = np.linspace(-30.0, 30.0, 121)
    for yv in (1.0, -1.0):
        y = np.full_like(z, yv)
        loss, g, dw = oracle.logistic_terms(z, y)
        assert np.allclose(loss, np.log1p(np.exp(-np.clip(y * z, -700, 700))), rtol=1e-12, atol=1e-300)
        h = 1e-5
        lp, gp, _ = oracle.logistic_terms(z + h, y)
        lm, gm, _ = oracle.logistic_terms(z - h, y)
        assert np.allclose((lp - lm) / (2 * h), g, atol=1e-9)
        assert np.allclose((gp - gm) / (2 * h), dw, atol=1e-9)
        assert np.all(dw >= 0) and np.all(dw <= 0.25 + 1e-15)
    # far tails: no overflow, loss -> -m for very negative margins
    loss, g, dw = oracle.logistic_terms(np.array([-800.0, 800.0]), np.array([1.0, 1.0]))
    assert np.isfinite(loss).all() and loss[0] == 800.0 and loss[1] == 0.0 and dw[0] == 0.0 and g[1] == 0.0


def test_weighted_preconditioner_identities():
    X, y, C, yC = _problem()
    M = C.shape[0]
    sigma, lam, eps = 1.25, 1e-3, 1e-9
    dm = np.random.default_rng(1).uniform(0.01, 0.25, M)
    T, A = oracle.precond_weighted(C, sigma, lam, eps, dm)
    K = _dense(C, C, sigma) + eps * np.eye(M)
    assert np.allclose(np.triu(T), T) and np.allclose(np.triu(A), A)
    assert np.abs(T.T @ T - K).max() < 1e-12
    assert np.abs(A.T @ A - (T @ np.diag(dm) @ T.T / M + lam * np.eye(M))).max() < 1e-12
    # unit weights reduce to the unweighted preconditioner of Alg. 1
    T1, A1 = oracle.precond_weighted(C, sigma, lam, eps, np.ones(M))
    T0, A0 = oracle.precond(C, sigma, lam, eps)
    assert np.allclose(T1, T0, atol=1e-12) and np.allclose(A1, A0, atol=1e-12)
    # the approximate Hessian of the appendix: (P P^T)^-1 = T^T (T Dm T^T / M + lam I) T ... in alpha
    # coordinates P P^T = (1/M K Dm K + lam K)^-1 up to the jitter
    P = sla.solve_triangular(T, sla.solve_triangular(A, np.eye(M)))
    H = K @ np.diag(dm) @ K / M + lam * K
    assert np.abs(P @ P.T @ H - np.eye(M)).max() < 1e-5


def test_weighted_linop_matches_dense_matrices():
    X, y, C, yC = _problem()
    n, M = X.shape[0], C.shape[0]
    sigma, lam, eps = 1.25, 1e-3, 1e-9
    g = np.random.default_rng(2)
    dw = g.uniform(0.0, 0.25, n)
    dm = g.uniform(0.01, 0.25, M)
    T, A = oracle.precond_weighted(C, sigma, lam, eps, dm)
    Knm = _dense(X, C, sigma)
    Kmm = _dense(C, C, sigma) + eps * np.eye(M)
    P = sla.solve_triangular(T, sla.solve_triangular(A, np.eye(M)))
    dense = P.T @ (Knm.T @ (dw[:, None] * Knm) + lam * n * Kmm) @ P
    beta = g.standard_normal(M)
    got = oracle.linop_weighted(X, C, sigma, lam, T, A, dw, beta)
    assert np.allclose(got, dense @ beta, rtol=1e-8, atol=1e-8 * np.abs(dense @ beta).max())


def _objective(X, y, C, sigma, lam, eps):
    n, M = X.shape[0], C.shape[0]
    Knm = _dense(X, C, sigma)
    Kmm = _dense(C, C, sigma) + eps * np.eye(M)

    def J(a):
        return np.logaddexp(0.0, -y * (Knm @ a)).mean() + 0.5 * lam * a @ Kmm @ a

    def dJ(a):
        m = y * (Knm @ a)
        s = 0.5 * (1.0 - np.tanh(0.5 * m))
        return Knm.T @ (-y * s) / n + lam * Kmm @ a

    def HJ(a):
        m = y * (Knm @ a)
        s = 0.5 * (1.0 - np.tanh(0.5 * m))
        return Knm.T @ ((s * (1 - s))[:, None] * Knm) / n + lam * Kmm

    return Knm, J, dJ, HJ


def test_one_step_with_converged_cg_is_the_exact_newton_step():
    X, y, C, yC = _problem()
    sigma, lam, eps = 1.25, 1e-2, 1e-8
    Knm, J, dJ, HJ = _objective(X, y, C, sigma, lam, eps)
    M = C.shape[0]
    # two steps, so the second starts from a non-trivial alpha (weights differ from 1/4)
    a1 = oracle.logfalkon_fit(X, y, C, yC, sigma, [lam], [3 * M], eps)
    ref1 = -np.linalg.solve(HJ(np.zeros(M)), dJ(np.zeros(M)))
    assert np.linalg.norm(Knm @ a1 - Knm @ ref1) <= 1e-7 * np.linalg.norm(Knm @ ref1)
    a2 = oracle.logfalkon_fit(X, y, C, yC, sigma, [lam, lam], [3 * M, 3 * M], eps)
    ref2 = ref1 - np.linalg.solve(HJ(ref1), dJ(ref1))
    assert np.linalg.norm(Knm @ a2 - Knm @ ref2) <= 1e-6 * np.linalg.norm(Knm @ ref2)


def test_newton_iteration_reaches_the_minimiser_a_general_optimiser_finds():
    X, y, C, yC = _problem(seed=3)
    sigma, lam, eps = 1.5, 1e-3, 1e-8
    Knm, J, dJ, _ = _objective(X, y, C, sigma, lam, eps)
    M = C.shape[0]
    lambdas = [1e-1, 1e-2] + [lam] * 6
    alpha, loss = oracle.logfalkon_fit(X, y, C, yC, sigma, lambdas, [40] * len(lambdas), eps, return_loss=True)
    res = minimize(J, np.zeros(M), jac=dJ, method="L-BFGS-B", options=dict(maxiter=50000, ftol=1e-15, gtol=1e-12))
    assert J(alpha) <= res.fun + 1e-9
    assert np.linalg.norm(dJ(alpha)) < 1e-8
    assert np.linalg.norm(Knm @ alpha - Knm @ res.x) <= 1e-4 * np.linalg.norm(Knm @ res.x)
    # the reported losses: log 2 at alpha = 0, then decreasing along the decreasing schedule
    assert loss[0] == np.log(2.0) or abs(loss[0] - np.log(2.0)) < 1e-15
    assert np.all(np.diff(loss) < 1e-12)
    assert abs(loss[-1] - np.logaddexp(0.0, -y * (Knm @ alpha)).mean()) < 1e-12


def test_few_cg_iterations_still_decrease_the_objective():
    X, y, C, yC = _problem(seed=4)
    sigma, lam, eps = 1.5, 1e-3, 1e-8
    _, J, _, _ = _objective(X, y, C, sigma, lam, eps)
    prev = J(np.zeros(C.shape[0]))
    for steps in (1, 2, 4):
        a = oracle.logfalkon_fit(X, y, C, yC, sigma, [lam] * steps, [3] * steps, eps)
        assert J(a) < prev
        prev = J(a)
