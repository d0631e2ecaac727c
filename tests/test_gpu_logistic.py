"""GPU parity for the weighted solver of the logistic loss (Appendix "Logistic Falkon
Algorithm", Alg. 2): weighted preconditioner, weighted operator and the approximate Newton
iteration, against the fp64 CPU oracle, through the C ABI.  End-to-end bar: relative L2 error
of predictions <= 1e-3.
"""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def _problem(n, M, d, seed, noise=0.4):
    g = torch.Generator().manual_seed(seed)
    X = torch.randn(n, d, generator=g)
    w = torch.randn(d, generator=g)
    y = torch.sign(X @ w + noise * torch.randn(n, generator=g))
    y[y == 0] = 1.0
    idx = torch.randperm(n, generator=g)[:M]
    return X, y, X[idx].contiguous(), y[idx].contiguous()


@pytest.mark.parametrize("M", [300, 1100])  # 2 and 5 block columns of the blocked T D T^T
def test_reweighted_factor_matches_oracle(knm, M):
    d, sigma, lam, jitter = 5, 0.75, 1e-4, 1e-9
    C = torch.randn(M, d, generator=torch.Generator().manual_seed(5))
    dm = torch.rand(M, generator=torch.Generator().manual_seed(6), dtype=torch.float64) * 0.25 + 1e-3
    pre = knm.precond_build(C.cuda(), sigma, 1.0, jitter)  # some other lambda first
    pre.reweight(lam, dm.cuda())
    T, A = pre.factors()
    To, Ao = oracle.precond_weighted(C.numpy(), sigma, lam, jitter, dm.numpy())
    assert rel_l2(T, To) < 1e-6 and rel_l2(A, Ao) < 1e-6
    assert np.array_equal(np.tril(A, -1), np.zeros_like(A))
    assert np.abs(A.T @ A - (T @ np.diag(dm.numpy()) @ T.T / M + lam * np.eye(M))).max() < 1e-12
    # back to unit weights: the unweighted second factor for the new lambda
    pre.reweight(2 * lam, None)
    _, A1 = pre.factors()
    _, A1o = oracle.precond(C.numpy(), sigma, 2 * lam, jitter)
    assert rel_l2(A1, A1o) < 1e-6
    with pytest.raises(knm.KnmError) as e:
        pre.reweight(-1.0, None)
    assert e.value.status == -1
    pre.close()


def test_weighted_linop_matches_oracle(knm):
    n, M, d, sigma, lam, jitter = 3000, 200, 6, 1.5, 1e-3, 1e-8
    X, y, C, yC = _problem(n, M, d, 7)
    g = torch.Generator().manual_seed(8)
    dw = torch.rand(n, generator=g) * 0.25
    dm = torch.rand(M, generator=g, dtype=torch.float64) * 0.25 + 1e-3
    beta = torch.randn(M, generator=g, dtype=torch.float64)
    pre = knm.precond_build(C.cuda(), sigma, lam, jitter)
    pre.reweight(lam, dm.cuda())
    out = knm.falkon_linop(pre, X.cuda(), C.cuda(), sigma, lam, beta.cuda(), dw=dw.cuda()).cpu().numpy()
    T, A = oracle.precond_weighted(C.numpy(), sigma, lam, jitter, dm.numpy())
    ref = oracle.linop_weighted(X.numpy(), C.numpy(), sigma, lam, T, A, dw.numpy().astype(np.float64), beta.numpy())
    assert rel_l2(out, ref) < 1e-4
    pre.close()


@pytest.mark.parametrize("d,sigma", [(6, 1.5), (28, 4.0)])
def test_logistic_fit_matches_oracle(knm, d, sigma):
    n, M, jitter = 6000, 250, 1e-7
    X, y, C, yC = _problem(n, M, d, 9)
    lambdas = [1e-2, 1e-3, 1e-4, 1e-4]
    iters = [4, 4, 6, 6]
    alpha, loss = knm.logfalkon_fit(X.cuda(), y.cuda(), C.cuda(), yC.cuda(), sigma, lambdas, iters, jitter,
                                    return_loss=True)
    ao, lo = oracle.logfalkon_fit(X.numpy(), y.numpy(), C.numpy(), yC.numpy(), sigma, lambdas, iters, jitter,
                                  return_loss=True)
    Xt, yt, _, _ = _problem(2000, 10, d, 10)
    pred = knm.falkon_predict(Xt.cuda(), C.cuda(), sigma, alpha).cpu().numpy()
    pred_o = oracle.falkon_predict(Xt.numpy(), C.numpy(), sigma, ao)
    print(f"\n  logistic fit d={d}: prediction error {rel_l2(pred, pred_o):.2e}, losses gpu {loss} oracle {lo}", flush=True)
    assert rel_l2(pred, pred_o) < 1e-3
    assert np.allclose(loss, lo, rtol=1e-4, atol=1e-6)
    assert loss[0] == pytest.approx(np.log(2.0), rel=1e-6) and np.all(np.diff(loss) < 0)
    # the fitted model separates the training labels better than chance
    acc = float((np.sign(knm.falkon_predict(X.cuda(), C.cuda(), sigma, alpha).cpu().numpy()) == y.numpy()).mean())
    assert acc > 0.8


def test_logistic_fit_rejects_bad_arguments(knm):
    X, y, C, yC = _problem(100, 10, 3, 11)
    with pytest.raises(knm.KnmError) as e:
        knm.logfalkon_fit(X.cuda(), y.cuda(), C.cuda(), yC.cuda(), 1.0, [1e-3, -1.0], [2, 2])
    assert e.value.status == -1
    with pytest.raises(knm.KnmError) as e:
        knm.logfalkon_fit(X.cuda(), y.cuda(), C.cuda(), yC.cuda(), 1.0, [1e-3], [0])
    assert e.value.status == -1
    with pytest.raises(ValueError):
        knm.logfalkon_fit(X.cuda(), y.cuda(), C.cuda(), yC.cuda(), 1.0, [1e-3, 1e-4], [2])
