"""fp64 rank-k update on the matrix cores against its definition (oracle.rank_k_upper)."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def knm():
    import paper_2006_10350_amd as k

    k.load_library()
    return k


def _colmajor(a):
    """GPU tensor whose storage is the column-major image of the numpy matrix a."""
    return torch.from_numpy(np.ascontiguousarray(a.T)).cuda()


def _run(knm, a, C0, form_nt, alpha=1.0, beta=0.0, w=None, triangular=False, shift=0.0):
    n = a.shape[0]
    A = _colmajor(a) if form_nt else _colmajor(a.T)  # n x k, or k x n, column-major
    C = _colmajor(C0)
    wt = None if w is None else torch.from_numpy(w).cuda()
    knm.rank_k_update(A, C, alpha=alpha, beta=beta, form_nt=form_nt, w=wt, triangular=triangular, shift=shift)
    torch.cuda.synchronize()
    got = C.cpu().numpy().T
    assert got.shape == (n, n)
    return got


# several tiles and ragged edges in every direction: tile 256 x 128, stage depth 16, patch 1024
SHAPES = [(1, 1), (5, 3), (64, 16), (130, 40), (257, 129), (700, 333), (1100, 48), (2100, 272)]


@pytest.mark.parametrize("n,k", SHAPES)
@pytest.mark.parametrize("form_nt", [False, True])
def test_rank_k_update_matches_definition(knm, n, k, form_nt):
    rng = np.random.default_rng(1000 * n + k)
    a = rng.standard_normal((n, k))
    C0 = rng.standard_normal((n, n))
    w = rng.random(k) + 0.5
    got = _run(knm, a, C0, form_nt, alpha=-0.75, beta=1.0, w=w, shift=0.5)
    ref = oracle.rank_k_upper(a, C0, alpha=-0.75, beta=1.0, w=w, shift=0.5)
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= 1e-13 * scale * max(k, 8)
    # the strict lower triangle is bit-for-bit what it was
    il = np.tril_indices(n, -1)
    assert np.array_equal(got[il], C0[il])


@pytest.mark.parametrize("n", [3, 200, 1500])
def test_triangular_operand_and_overwrite(knm, n):
    """T diag(w) T^T from an upper-triangular T (zeros stored below its diagonal); beta = 0 must
    not read C (it holds NaN)."""
    rng = np.random.default_rng(n)
    T = np.triu(rng.standard_normal((n, n)))
    w = rng.random(n) + 0.1
    C0 = np.full((n, n), np.nan)
    got = _run(knm, T, C0, True, alpha=1.0 / n, beta=0.0, w=w, triangular=True, shift=1e-3)
    ref = oracle.rank_k_upper(T, None, alpha=1.0 / n, w=w, triangular=True, shift=1e-3)
    iu = np.triu_indices(n)
    assert np.isfinite(got[iu]).all()
    assert np.abs(got[iu] - ref[iu]).max() <= 1e-13 * np.abs(ref).max() * n
    il = np.tril_indices(n, -1)
    assert np.isnan(got[il]).all()


@pytest.mark.parametrize("k0", [100, 101])  # operand 16-byte aligned or not: wide and narrow loads
def test_leading_dimensions_larger_than_the_matrix(knm, k0):
    """Operand and result as sub-blocks of larger allocations (how the factorisation calls it)."""
    rng = np.random.default_rng(7)
    big = rng.standard_normal((900, 900))        # column-major image below
    w_, r0 = 64, 165                             # block row [k0, k0 + w_), trailing block from r0
    n = 900 - r0
    G = _colmajor(big)                           # G[j, i] = big[i, j]
    lib = knm.load_library()
    ctx = knm.default_context()
    base = G.data_ptr()
    A_ptr = base + 8 * (k0 + r0 * 900)           # big[k0:, r0:], k x n with lda = 900
    C_ptr = base + 8 * (r0 + r0 * 900)
    ctx.check(lib.precond_rank_k_update(ctx._h, 0, n, w_, -1.0, A_ptr, 900, None, 0, 1.0, 0.0, C_ptr, 900))
    torch.cuda.synchronize()
    got = G.cpu().numpy().T
    ref = big.copy()
    ref[r0:, r0:] = oracle.rank_k_upper(big[k0:k0 + w_, r0:].T, big[r0:, r0:], alpha=-1.0, beta=1.0)
    assert np.abs(got - ref).max() <= 1e-12 * np.abs(ref).max()


def test_rank_k_update_rejects_bad_arguments(knm):
    A = torch.zeros(8, 4, dtype=torch.float64, device="cuda")
    C = torch.zeros(8, 8, dtype=torch.float64, device="cuda")
    lib = knm.load_library()
    ctx = knm.default_context()
    assert lib.precond_rank_k_update(ctx._h, 0, 8, 4, 1.0, A.data_ptr(), 3, None, 0, 0.0, 0.0, C.data_ptr(), 8) != 0
    assert lib.precond_rank_k_update(ctx._h, 0, 8, 4, 1.0, A.data_ptr(), 4, None, 0, 0.0, 0.0, C.data_ptr(), 7) != 0
    assert lib.precond_rank_k_update(ctx._h, 0, 8, 4, 1.0, A.data_ptr(), 4, None, 1, 0.0, 0.0, C.data_ptr(), 8) != 0
    assert lib.precond_rank_k_update(ctx._h, 0, 8, 4, 1.0, None, 4, None, 0, 0.0, 0.0, C.data_ptr(), 8) != 0
    # nothing to do is not an error
    assert lib.precond_rank_k_update(ctx._h, 0, 0, 4, 1.0, A.data_ptr(), 4, None, 0, 0.0, 0.0, C.data_ptr(), 1) == 0
