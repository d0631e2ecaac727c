"""GPU parity for the kernels of the distance r = |x - c| -- Laplacian exp(-r / sigma) and the
Matern kernels with nu = 3/2 and 5/2: products, preconditioner and small fits against the fp64 CPU
oracle run with the same kernel, through the C ABI.

Bar: relative L2 error <= 1e-4 per product, <= 1e-3 for end-to-end predictions.  The centres are
rows of the data (Nystrom centres, Section 2), so every case holds exactly coincident pairs, whose
distance the engines get from a cancellation.
"""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

TOL = 1e-4
TIGHT = 2e-5  # measured: 2e-7 .. 4e-6


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def _rand(n, d, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (scale * torch.randn(n, d, generator=g)).to(torch.float32)


def _centres(X, M, seed):
    idx = torch.randperm(X.shape[0], generator=torch.Generator().manual_seed(seed))[:M]
    return X[idx].clone()


@pytest.fixture(params=[("laplacian", "f32"), ("laplacian", "f16x3"), ("matern32", "f16x3"), ("matern52", "f32"),
                        ("matern52", "f16x3")], ids=lambda p: f"{p[0]}-{p[1]}")
def lap(request, knm):
    """One of the kernels of r on the default context and in the oracle, with one of the two
    cross-term arithmetics."""
    kind, cross = request.param
    ctx = knm.default_context()
    ctx.set_cross_term(cross)
    ctx.set_kernel(kind)
    with oracle.kernel(kind):
        yield f"{kind}/{cross}"
    ctx.set_kernel("gaussian")
    ctx.set_cross_term("f16x3")


SHAPES = [
    # n, M, d, t, sigma -- small d (below the register-resident engines' limits too), large and
    # unaligned d, several columns, the matrix-core reduction (8-32 columns), two column groups
    (1000, 300, 8, 1, 2.0),
    (2049, 515, 28, 1, 6.0),
    (1500, 260, 1, 1, 0.7),
    (777, 129, 9, 3, 3.0),
    (515, 260, 130, 1, 16.0),
    (600, 300, 784, 10, 40.0),
    (400, 385, 99, 3, 12.0),
    (1100, 700, 20, 32, 5.0),
    (900, 300, 6, 40, 2.5),
    (2300, 700, 28, 9, 6.0),
    (700, 520, 28, 70, 6.0),
    (400, 320, 300, 70, 40.0),
    (300, 260, 290, 40, 40.0),
    (300, 260, 24, 150, 6.0),
]


@pytest.mark.parametrize("n,M,d,t,sigma", SHAPES)
def test_radial_products_match_oracle(knm, lap, n, M, d, t, sigma):
    print(f"case n={n} M={M} d={d} t={t} cross={lap}", flush=True)
    X = _rand(n, d, 1)
    C = _centres(X, M, 2)
    V, Y = _rand(M, t, 3), _rand(n, t, 4)
    Xd, Cd = X.cuda(), C.cuda()
    Xn, Cn = X.numpy(), C.numpy()

    W = knm.knm_v(Xd, Cd, sigma, V.cuda()).cpu().numpy()
    e_w = rel_l2(W, oracle.knm_v(Xn, Cn, sigma, V.numpy()))
    R = knm.knm_t_y(Xd, Cd, sigma, Y.cuda()).cpu().numpy()
    e_r = rel_l2(R, oracle.knm_t_y(Xn, Cn, sigma, Y.numpy()))
    U = knm.knm_prod(Xd, Cd, sigma, V.cuda()).cpu().numpy()
    Uo = oracle.knm_prod(Xn, Cn, sigma, V.numpy())
    e_u = rel_l2(U, Uo)
    print(f"errors: K v {e_w:.2e}  K^T y {e_r:.2e}  K^T K v {e_u:.2e}", flush=True)
    assert e_w < TIGHT and e_r < TIGHT and e_u < TIGHT
    for c in range(t):
        assert rel_l2(U.reshape(M, t)[:, c], np.asarray(Uo).reshape(M, t)[:, c]) < TOL


def test_radial_weighted_product(knm, lap):
    n, M, d, t, sigma = 2500, 300, 9, 2, 3.0
    X = _rand(n, d, 7)
    C, V = _centres(X, M, 8), _rand(M, t, 9)
    dw = torch.rand(n, generator=torch.Generator().manual_seed(10)) + 0.05
    U = knm.knm_prod_weighted(X.cuda(), C.cuda(), sigma, dw.cuda(), V.cuda()).cpu().numpy()
    assert rel_l2(U, oracle.knm_prod_weighted(X.numpy(), C.numpy(), sigma, dw.numpy(), V.numpy())) < TOL


def test_radial_large_norms_and_near_duplicates(knm, lap):
    """Points far from the origin (the norm expansion cancels seven digits), centres that are data
    rows, and centres that are data rows moved by 1e-3: the pairs below the refinement threshold
    are taken from differences, the others keep the accuracy of the expansion (the bar of the
    Gaussian kernel on the same data)."""
    n, M, d, sigma = 2000, 256, 8, 1.0
    X = 11.0 + 0.5 * _rand(n, d, 18)
    C = _centres(X, M, 19)
    C[::2] += 1e-3 * _rand(M // 2, d, 20)
    V = torch.ones(M, 1)
    W = knm.knm_v(X.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
    Wo = oracle.knm_v(X.numpy(), C.numpy(), sigma, V.numpy())
    err = rel_l2(W, Wo)
    print(f"large norms: {err:.2e}", flush=True)
    assert err < 1e-3
    # the rows that are centres (or next to one) carry a kernel value near 1: each within 1e-3 of it
    idx = torch.randperm(n, generator=torch.Generator().manual_seed(19))[:M].numpy()
    assert np.abs(W.ravel()[idx] - np.asarray(Wo).ravel()[idx]).max() < 1e-3


def test_radial_preconditioner_factors(knm, lap):
    M, d, sigma, lam, jitter = 700, 5, 1.5, 1e-4, 1e-9
    C = _rand(M, d, 31)
    pre = knm.precond_build(C.cuda(), sigma, lam, jitter)
    T, A = pre.factors()
    To, Ao = oracle.precond(C.numpy(), sigma, lam, jitter)
    assert rel_l2(T, To) < 1e-8
    assert rel_l2(A, Ao) < 1e-8
    K = oracle.kernel_matrix(C.numpy(), C.numpy(), sigma) + jitter * np.eye(M)
    assert np.abs(T.T @ T - K).max() < 1e-12
    pre.close()


def test_radial_fit_and_predict(knm, lap):
    n, M, d, t, sigma, lam, iters, jitter = 6000, 400, 6, 2, 3.0, 1e-5, 10, 1e-9
    X = _rand(n, d, 37)
    C = _centres(X, M, 38)
    Y = torch.stack([torch.sin(X.sum(1)), torch.cos(X[:, 0]) * X[:, 1]], dim=1).contiguous()
    alpha, resid = knm.falkon_fit(X.cuda(), Y.cuda(), C.cuda(), sigma, lam, iters, jitter, return_resid=True)
    ao, ro = oracle.falkon_fit(X.numpy(), Y.numpy(), C.numpy(), sigma, lam, iters, jitter, return_resid=True)
    Xt = _rand(1500, d, 39)
    pred = knm.falkon_predict(Xt.cuda(), C.cuda(), sigma, alpha).cpu().numpy()
    po = oracle.falkon_predict(Xt.numpy(), C.numpy(), sigma, ao)
    err = rel_l2(pred, po)
    print(f"prediction error {err:.3e}; residuals gpu {resid[:3].ravel()} oracle {np.asarray(ro)[:3].ravel()}")
    assert err < 1e-3
    for c in range(t):
        assert rel_l2(pred[:, c], po[:, c]) < 1e-3
    np.testing.assert_allclose(resid[:4].ravel(), np.asarray(ro)[:4].ravel(), rtol=1e-2)
    # the fit is useful: far better than predicting zero
    clean = np.sin(Xt.numpy().astype(np.float64).sum(1))
    assert np.mean((pred[:, 0] - clean) ** 2) < 0.5 * np.var(clean)


def test_radial_logistic_fit(knm, lap):
    """The Newton iteration for the logistic loss (Alg. 2) is kernel-agnostic: losses after every step
    and predictions against the oracle's iteration with the same kernel."""
    n, M, d, sigma, jitter = 5000, 250, 6, 3.0, 1e-7
    g = torch.Generator().manual_seed(9)
    X = torch.randn(n, d, generator=g)
    y = torch.sign(X @ torch.randn(d, generator=g) + 0.4 * torch.randn(n, generator=g))
    y[y == 0] = 1.0
    idx = torch.randperm(n, generator=g)[:M]
    C, yC = X[idx].contiguous(), y[idx].contiguous()
    lambdas, iters = [1e-2, 1e-3, 1e-4], [4, 4, 6]
    alpha, loss = knm.logfalkon_fit(X.cuda(), y.cuda(), C.cuda(), yC.cuda(), sigma, lambdas, iters, jitter,
                                    return_loss=True)
    ao, lo = oracle.logfalkon_fit(X.numpy(), y.numpy(), C.numpy(), yC.numpy(), sigma, lambdas, iters, jitter,
                                  return_loss=True)
    assert np.allclose(loss, lo, rtol=1e-4, atol=1e-6)
    assert np.all(np.diff(loss) < 0)
    Xt = _rand(1000, d, 10)
    pred = knm.falkon_predict(Xt.cuda(), C.cuda(), sigma, alpha).cpu().numpy()
    assert rel_l2(pred, oracle.falkon_predict(Xt.numpy(), C.numpy(), sigma, ao)) < 1e-3


def test_kernel_setting_is_per_context_and_validated(knm):
    n, M, d, sigma = 600, 200, 7, 2.0
    X = _rand(n, d, 50)
    C, v = _centres(X, M, 51), _rand(M, 1, 52)
    other = knm.Context()
    other.set_kernel("laplacian")
    U_l = knm.knm_prod(X.cuda(), C.cuda(), sigma, v.cuda(), ctx=other).cpu().numpy()
    U_g = knm.knm_prod(X.cuda(), C.cuda(), sigma, v.cuda()).cpu().numpy()  # default context: Gaussian
    assert rel_l2(U_g, oracle.knm_prod(X.numpy(), C.numpy(), sigma, v.numpy())) < TOL
    with oracle.kernel("laplacian"):
        assert rel_l2(U_l, oracle.knm_prod(X.numpy(), C.numpy(), sigma, v.numpy())) < TOL
    with pytest.raises(knm.KnmError):
        other.set_kernel(7)
    other.close()


def test_sparse_inputs_refuse_the_laplacian_kernel(knm):
    import synth

    n, M, d = 300, 40, 500
    s = synth.sparse_inputs(n, M, d, nnz_per_row=8.0, seed=3)
    mk = lambda p, r: torch.sparse_csr_tensor(s[p + "_indptr"].cuda(), s[p + "_indices"].cuda(), s[p + "_values"].cuda(),
                                              size=(r, d), check_invariants=False)
    ctx = knm.Context()
    ctx.set_kernel("laplacian")
    v = _rand(M, 1, 4).cuda()
    with pytest.raises(knm.KnmError) as e:
        knm.knm_prod_csr(mk("x", n), mk("c", M), 2.0, v, ctx=ctx)
    assert e.value.status == knm.KNM_UNSUPPORTED
    ctx.close()
