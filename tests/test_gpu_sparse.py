"""Sparse-input product (CSR X and C) against the oracle's dense definition on the densified inputs."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def _dense(indptr, indices, values, rows, d):
    out = np.zeros((rows, d), dtype=np.float32)
    r = np.repeat(np.arange(rows), np.diff(indptr))
    out[r, indices] = values
    return out


def _csr(indptr, indices, values, rows, d):
    return torch.sparse_csr_tensor(indptr.cuda(), indices.cuda(), values.cuda(), size=(rows, d), check_invariants=False)


def _case(n, M, d, nnz, seed):
    s = synth.sparse_inputs(n, M, d, nnz_per_row=nnz, seed=seed)
    Xd = _dense(s["x_indptr"].numpy(), s["x_indices"].numpy(), s["x_values"].numpy(), n, d)
    Cd = _dense(s["c_indptr"].numpy(), s["c_indices"].numpy(), s["c_values"].numpy(), M, d)
    X = _csr(s["x_indptr"], s["x_indices"], s["x_values"], n, d)
    C = _csr(s["c_indptr"], s["c_indices"], s["c_values"], M, d)
    return s, X, C, Xd, Cd


# sigma = 8: typical |x|^2 / 2 sigma^2 around 1 (the rank-one part matters); sigma = 1: a_i b_j underflows
# and only the pairs that share features survive (a centre against its own row gives exactly 1)
@pytest.fixture(params=[128, 0, 3])
def head_limit(request, knm):
    """Runs a test with the dense treatment of the most frequent features at its default, switched
    off, and restricted to three features (so that frequent features remain in the sparse walk)."""
    ctx = knm.default_context()
    ctx.set_sparse_head_limit(request.param)
    yield request.param
    ctx.set_sparse_head_limit(128)


@pytest.mark.parametrize("n,M,d,nnz,sigma", [(3000, 400, 5000, 30.0, 8.0), (1500, 300, 800, 12.0, 3.0),
                                             (2000, 256, 3000, 40.0, 1.0), (130, 7, 64, 5.0, 4.0)])
def test_sparse_product_matches_dense_oracle(knm, head_limit, n, M, d, nnz, sigma):
    s, X, C, Xd, Cd = _case(n, M, d, nnz, seed=n + M)
    v = synth.probe_vector(M, 1, "normal", device="cuda")
    U, W = knm.knm_prod_csr(X, C, sigma, v, return_w=True)
    Uo, Wo = oracle.knm_prod(Xd, Cd, sigma, v.cpu().numpy(), return_w=True)
    print(f"head limit {head_limit}: errors W {rel_l2(W.cpu().numpy(), Wo):.2e} U {rel_l2(U.cpu().numpy(), Uo):.2e}", flush=True)
    assert rel_l2(W.cpu().numpy(), Wo) < 1e-5
    assert rel_l2(U.cpu().numpy(), Uo) < 1e-5


def test_frequent_features_are_found_and_change_nothing(knm):
    """A problem in which a few features occur in most points (their centre lists pass the
    threshold by a wide margin): with and without their dense treatment the product is the
    oracle's, also with weights and several columns, and for rows made of frequent features only."""
    n, M, d, sigma = 2500, 320, 600, 6.0
    s, X, C, Xd, Cd = _case(n, M, d, 20.0, seed=77)
    lens = np.bincount(s["c_indices"].numpy(), minlength=d)
    assert np.sort(lens)[-3] >= 64  # at least three long lists: the head set is not empty
    V = synth.probe_vector(M, 2, "normal", device="cuda")
    Uo = oracle.knm_prod(Xd, Cd, sigma, V.cpu().numpy())
    ctx = knm.default_context()
    got = {}
    for limit in (0, 128):
        ctx.set_sparse_head_limit(limit)
        got[limit] = knm.knm_prod_csr(X, C, sigma, V).cpu().numpy()
        assert rel_l2(got[limit], Uo) < 1e-5, limit
    ctx.set_sparse_head_limit(128)
    assert rel_l2(got[128], got[0]) < 1e-5


def test_sparse_product_several_columns_and_no_w(knm):
    n, M, d, sigma = 1200, 200, 2000, 6.0
    s, X, C, Xd, Cd = _case(n, M, d, 25.0, seed=5)
    V = synth.probe_vector(M, 3, "normal", device="cuda")
    U = knm.knm_prod_csr(X, C, sigma, V)
    Uo = oracle.knm_prod(Xd, Cd, sigma, V.cpu().numpy())
    assert U.shape == (M, 3)
    assert rel_l2(U.cpu().numpy(), Uo) < 1e-5


def test_feature_ids_spread_over_fifty_million_columns(knm):
    """The same problem with its features renamed injectively into [0, 5e7): the kernel only sees
    which features two points share, so the product must not change (the dense oracle cannot
    hold 5e7 columns; it evaluates the compact problem)."""
    n, M, d, sigma = 2000, 300, 4000, 7.0
    s, X, C, Xd, Cd = _case(n, M, d, 30.0, seed=9)
    big = 50_000_000
    rename = torch.from_numpy(np.sort(np.random.default_rng(3).choice(big, size=d, replace=False))).to(torch.int64)
    Xb = _csr(s["x_indptr"], rename[s["x_indices"]], s["x_values"], n, big)
    Cb = _csr(s["c_indptr"], rename[s["c_indices"]], s["c_values"], M, big)
    v = synth.probe_vector(M, 1, "normal", device="cuda")
    U, W = knm.knm_prod_csr(Xb, Cb, sigma, v, return_w=True)
    Uo, Wo = oracle.knm_prod(Xd, Cd, sigma, v.cpu().numpy(), return_w=True)
    assert rel_l2(W.cpu().numpy(), Wo) < 1e-5
    assert rel_l2(U.cpu().numpy(), Uo) < 1e-5


def test_all_rows_empty_is_the_rank_one_matrix(knm):
    """No stored entry anywhere: every point is the origin, K is all ones."""
    n, M, d = 70, 9, 1000
    X = _csr(torch.zeros(n + 1, dtype=torch.int64), torch.zeros(0, dtype=torch.int64), torch.zeros(0), n, d)
    C = _csr(torch.zeros(M + 1, dtype=torch.int64), torch.zeros(0, dtype=torch.int64), torch.zeros(0), M, d)
    v = synth.probe_vector(M, 1, "normal", device="cuda")
    U, W = knm.knm_prod_csr(X, C, 2.0, v, return_w=True)
    sv = float(v.sum())
    assert np.allclose(W.cpu().numpy(), sv, rtol=1e-6, atol=1e-6)
    assert np.allclose(U.cpu().numpy(), n * sv, rtol=1e-6, atol=1e-5)


def test_sparse_product_rejects_bad_structure(knm):
    n, M, d = 50, 8, 100
    s = synth.sparse_inputs(n, M, d, nnz_per_row=6.0, seed=2)
    C = _csr(s["c_indptr"], s["c_indices"], s["c_values"], M, d)
    v = synth.probe_vector(M, 1, "normal", device="cuda")
    bad_col = s["x_indices"].clone()
    bad_col[3] = d  # one past the last feature
    with pytest.raises(knm.KnmError):
        knm.knm_prod_csr(_csr(s["x_indptr"], bad_col, s["x_values"], n, d), C, 2.0, v)
    twice = s["x_indices"].clone()
    first = int(s["x_indptr"][1])  # row 1 has entries (row 0 is empty by construction)
    twice[first + 1] = twice[first]  # the same feature twice in a row
    with pytest.raises(knm.KnmError):
        knm.knm_prod_csr(_csr(s["x_indptr"], twice, s["x_values"], n, d), C, 2.0, v)
    bad_ptr = s["x_indptr"].clone()
    bad_ptr[5] = bad_ptr[6] + 1  # decreasing
    with pytest.raises(knm.KnmError):
        knm.knm_prod_csr(_csr(bad_ptr, s["x_indices"], s["x_values"], n, d), C, 2.0, v)
    with pytest.raises(TypeError):
        knm.knm_prod_csr(torch.zeros(n, d, device="cuda"), C, 2.0, v)


def test_sparse_fit_and_predict_match_the_dense_oracle(knm):
    """Alg. 1 on CSR inputs against the oracle's fit on the densified inputs: same centres, same
    iteration count; predictions on the training rows and on held-out sparse rows at the end-to-end
    bar (the coefficients themselves are ill-determined at this lambda, as in the dense fits)."""
    # lambda = 1e-3: with 1e-5 this problem amplifies the fp32 noise of the products tenfold per
    # iteration (the dense GPU fit leaves the fp64 oracle's trajectory at the same point), and the
    # sparse sweeps' atomics make that noise differ from run to run
    n, M, d, sigma, lam, jitter, iters = 2500, 200, 1500, 5.0, 1e-3, 1e-6, 6
    s, X, C, Xd, Cd = _case(n, M, d, 15.0, seed=21)
    g = torch.Generator().manual_seed(4)
    wtrue = torch.randn(d, generator=g)
    Y = torch.tanh(0.05 * torch.from_numpy(Xd) @ wtrue) + 0.05 * torch.randn(n, generator=g)
    alpha, resid = knm.falkon_fit_csr(X, Y.cuda(), C, sigma, lam, iters, jitter, return_resid=True)
    ao, ro = oracle.falkon_fit(Xd, Y.numpy(), Cd, sigma, lam, iters, jitter, return_resid=True)
    assert np.allclose(np.ravel(resid), np.ravel(ro), rtol=1e-3)
    fit = knm.knm_v_csr(X, C, sigma, alpha)
    assert rel_l2(fit.cpu().numpy(), oracle.falkon_predict(Xd, Cd, sigma, ao)) < 1e-3
    st, Xt, _, Xtd, _ = _case(400, 8, d, 15.0, seed=22)
    pred = knm.knm_v_csr(Xt, C, sigma, alpha)
    po = oracle.falkon_predict(Xtd, Cd, sigma, ao)
    assert rel_l2(pred.cpu().numpy(), po) < 1e-3


def test_sparse_logistic_fit_matches_the_dense_oracle(knm):
    """Alg. 2 on CSR inputs against the oracle's Newton iteration on the densified inputs: the loss
    after every step and the predictions on training and held-out rows."""
    n, M, d, sigma, jitter = 3000, 200, 1200, 5.0, 1e-6
    s, X, C, Xd, Cd = _case(n, M, d, 15.0, seed=41)
    g = torch.Generator().manual_seed(5)
    wtrue = torch.randn(d, generator=g)
    score = 0.08 * torch.from_numpy(Xd) @ wtrue + 0.3 * torch.randn(n, generator=g)
    y = torch.where(score >= score.median(), 1.0, -1.0).to(torch.float32)
    yC = y[s["centre_rows"]].clone()
    lambdas, iters = [1e-2, 1e-3, 1e-3], [4, 5, 5]
    alpha, loss = knm.logfalkon_fit_csr(X, y.cuda(), C, yC.cuda(), sigma, lambdas, iters, jitter, return_loss=True)
    ao, lo = oracle.logfalkon_fit(Xd, y.numpy(), Cd, yC.numpy(), sigma, lambdas, iters, jitter, return_loss=True)
    print(f"losses gpu {loss} oracle {lo}", flush=True)
    assert np.allclose(loss, lo, rtol=1e-4, atol=1e-6)
    assert loss[0] == pytest.approx(np.log(2.0), rel=1e-6) and np.all(np.diff(loss) < 0)
    fit = knm.knm_v_csr(X, C, sigma, alpha).cpu().numpy()
    assert rel_l2(fit, oracle.falkon_predict(Xd, Cd, sigma, ao)) < 1e-3
    st, Xt, _, Xtd, _ = _case(400, 8, d, 15.0, seed=42)
    pred = knm.knm_v_csr(Xt, C, sigma, alpha).cpu().numpy()
    assert rel_l2(pred, oracle.falkon_predict(Xtd, Cd, sigma, ao)) < 1e-3
    assert float((np.sign(fit) == y.numpy()).mean()) > 0.7
    with pytest.raises(knm.KnmError):
        knm.logfalkon_fit_csr(X, y.cuda(), C, yC.cuda(), sigma, [1e-2, -1.0], [3, 3], jitter)


def test_sparse_preconditioner_factors_match_oracle(knm):
    M, d, sigma, lam, jitter = 300, 900, 4.0, 1e-4, 1e-8
    s, X, C, Xd, Cd = _case(600, M, d, 12.0, seed=31)
    lib = knm.load_library()
    import ctypes

    ctx = knm.default_context()
    cr, cc, cv = C.crow_indices().contiguous(), C.col_indices().contiguous(), C.values().contiguous()
    h = ctypes.c_void_p()
    bad = ctypes.c_int64(0)
    ctx.check(lib.precond_build_csr(ctx._h, cr.data_ptr(), cc.data_ptr(), cv.data_ptr(), M, d, sigma, lam, jitter,
                                    ctypes.byref(h), ctypes.byref(bad)))
    T = np.empty((M, M))
    A = np.empty((M, M))
    ctx.check(lib.precond_get_factors(ctx._h, h, T.ctypes.data, A.ctypes.data))
    lib.precond_free(h)
    To, Ao = oracle.precond(Cd, sigma, lam, jitter)
    assert np.abs(T - To).max() < 1e-9 * max(1.0, np.abs(To).max())
    assert np.abs(A - Ao).max() < 1e-9 * max(1.0, np.abs(Ao).max())


def _check_product(knm, n, M, d, nnz, skew, sigma, t, seed, tol=1e-5):
    s = synth.sparse_inputs(n, M, d, nnz_per_row=nnz, skew=skew, seed=seed)
    Xd = _dense(s["x_indptr"].numpy(), s["x_indices"].numpy(), s["x_values"].numpy(), n, d)
    Cd = _dense(s["c_indptr"].numpy(), s["c_indices"].numpy(), s["c_values"].numpy(), M, d)
    X = _csr(s["x_indptr"], s["x_indices"], s["x_values"], n, d)
    C = _csr(s["c_indptr"], s["c_indices"], s["c_values"], M, d)
    V = torch.randn(M, t, generator=torch.Generator().manual_seed(seed))
    if seed % 3 == 0:
        V = V.abs()
    U, W = knm.knm_prod_csr(X, C, sigma, V.cuda(), return_w=True)
    Uo, Wo = oracle.knm_prod(Xd, Cd, sigma, V.numpy(), return_w=True)
    errs = (rel_l2(U.cpu().numpy(), Uo), rel_l2(W.cpu().numpy(), Wo))
    assert max(errs) < tol, (n, M, d, nnz, skew, sigma, t, seed, errs)


def test_rows_with_more_frequent_features_than_lanes(knm):
    """Dense-ish rows over few features: nearly every feature is frequent, the head set is full
    (128 features) and single rows hold more than 64 of them."""
    n = M = 100
    s = synth.sparse_inputs(n, M, 300, nnz_per_row=80.0, skew=1.0, seed=150)
    lens = np.bincount(s["c_indices"].numpy(), minlength=300)
    assert (lens >= 16).sum() >= 128
    _check_product(knm, n, M, 300, 80.0, 1.0, 20.0, 1, seed=150)


def test_small_length_scale_sends_the_frequent_features_back_to_the_sparse_walk(knm):
    """sigma far below the norms of the frequent features' parts: a dense product over them would
    form its exponent from a cancellation of terms in the thousands; the library must notice and
    keep the exact sparse walk (also: no overflow where the shared part of two rows is large)."""
    _check_product(knm, 1500, 64, 1000, 80.0, 8.0, 0.7, 2, seed=141)
    _check_product(knm, 64, 64, 1000, 10.0, 5.0, 0.7, 1, seed=139)


@pytest.mark.parametrize("block", range(4))
def test_random_sparse_draws_match_dense_oracle(knm, block):
    ctx = knm.default_context()
    try:
        for case in range(10):
            seed = 700 + 10 * block + case
            rng = np.random.default_rng(seed)
            M = int(rng.choice([1, 3, 17, 64, 100, 257, 400, 900]))
            n = int(max(M, rng.choice([1, 5, 63, 130, 500, 1500, 4000])))
            d = int(rng.choice([8, 64, 300, 1000, 5000]))
            nnz = min(float(rng.choice([1.0, 3.0, 10.0, 30.0, 80.0])), d / 2)
            skew = float(rng.choice([1.0, 2.5, 5.0, 8.0]))
            sigma = float(rng.choice([0.7, 2.0, 6.0, 20.0]))
            t = int(rng.choice([1, 1, 2, 3]))
            limit = int(rng.choice([128, 128, 0, 2, 7]))
            print(f"seed {seed}: n={n} M={M} d={d} nnz={nnz} skew={skew} sigma={sigma} t={t} head limit {limit}", flush=True)
            ctx.set_sparse_head_limit(limit)
            _check_product(knm, n, M, d, nnz, skew, sigma, t, seed)
    finally:
        ctx.set_sparse_head_limit(128)
