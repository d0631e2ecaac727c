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
    # what is stored below the operand's diagonal is ignored (in the preconditioner's shared array
    # it belongs to the other factor): NaN there must not reach the result
    Tn = T.copy()
    Tn[il] = np.nan
    got2 = _run(knm, Tn, C0, True, alpha=1.0 / n, beta=0.0, w=w, triangular=True, shift=1e-3)
    assert np.array_equal(got2[iu], got[iu])


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


# general block product: ragged shapes around the 128 x 128 tile, the 16-deep stage and the patch shapes
GEMM_SHAPES = [(1, 1, 1), (5, 7, 3), (128, 128, 128), (128, 1000, 48), (130, 257, 33), (300, 90, 129),
               (1100, 700, 64), (64, 2100, 272), (2100, 64, 17)]


@pytest.mark.parametrize("ni,nj,k", GEMM_SHAPES)
@pytest.mark.parametrize("a_nt", [False, True])
def test_block_product_matches_definition(knm, ni, nj, k, a_nt):
    rng = np.random.default_rng(7 * ni + 3 * nj + k)
    a = rng.standard_normal((ni, k))      # a(i, q)
    b = rng.standard_normal((nj, k))      # b(j, q)
    C0 = rng.standard_normal((ni, nj))
    A = _colmajor(a) if a_nt else _colmajor(a.T)   # ni x k, or k x ni, column-major
    B = _colmajor(b.T)                             # k x nj
    C = _colmajor(C0)
    knm.block_product(A, B, C, alpha=-0.5, beta=1.0, a_nt=a_nt)
    torch.cuda.synchronize()
    ref = -0.5 * a @ b.T + C0
    assert np.abs(C.cpu().numpy().T - ref).max() <= 1e-13 * np.abs(ref).max() * max(k, 8)
    # beta = 0 overwrites without reading
    Cn = _colmajor(np.full((ni, nj), np.nan))
    knm.block_product(A, B, Cn, alpha=2.0, beta=0.0, a_nt=a_nt)
    torch.cuda.synchronize()
    ref = 2.0 * a @ b.T
    assert np.abs(Cn.cpu().numpy().T - ref).max() <= 1e-13 * np.abs(ref).max() * max(k, 8)
