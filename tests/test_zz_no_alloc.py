"""The allocation-free product entry point (static scratch array) against the ordinary one, through
the C ABI: two calls in a row, the second on a smaller input, so that stale contents of the shared
scratch would show."""
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


# both register-resident layouts and the K-loop engine; with 20, 40 and 70 columns its reduction on the matrix
# cores, where the allocating call hands the vectors over as a packed image and takes more columns per launch
@pytest.mark.parametrize("d,t", [(8, 1), (28, 1), (50, 3), (50, 20), (28, 40), (300, 70)])
def test_static_scratch_product_matches_the_allocating_one(knm, d, t):
    ctx = knm.default_context()
    assert knm.knm_static_scratch_bytes() == 64 << 20
    for n, M in ((30000, 1300), (4111, 257)):  # several chunks and a ragged tail, then a smaller input
        g = torch.Generator().manual_seed(100 * d + t + n)
        X = torch.randn(n, d, generator=g).cuda()
        C = X[torch.randperm(n, generator=g)[:M].cuda()].contiguous()
        V = torch.randn(M, t, generator=g).cuda()
        W = torch.full((n, t), float("nan"), device="cuda")
        U = torch.full((M, t), float("nan"), device="cuda")
        held = ctx.workspace_held()
        knm.knm_prod_static(X, C, 2.0, V, W, U, ctx=ctx)
        torch.cuda.synchronize()
        assert ctx.workspace_held() == held  # the context's own workspace did not grow
        U_ref, W_ref = knm.knm_prod(X, C, 2.0, V, return_w=True, ctx=ctx)
        # same chunks, same kernels, same order of the merge: the same bits
        assert torch.equal(W, W_ref.reshape(n, t)) and torch.equal(U, U_ref.reshape(M, t))
        Uo = oracle.knm_prod(X.cpu().numpy(), C.cpu().numpy(), 2.0, V.cpu().numpy())
        assert rel_l2(U.cpu().numpy(), Uo) < 1e-4


def test_static_scratch_product_in_slabs(knm):
    """A stream image larger than the scratch (600000 points x 128 bytes) is built slab by slab."""
    n, M, d = 600000, 500, 28
    g = torch.Generator().manual_seed(77)
    X = torch.randn(n, d, generator=g).cuda()
    C = X[:M].contiguous()
    V = torch.randn(M, 1, generator=g).cuda()
    W = torch.empty(n, 1, device="cuda")
    U = torch.empty(M, 1, device="cuda")
    assert n * 128 > knm.knm_static_scratch_bytes()
    knm.knm_prod_static(X, C, 4.0, V, W, U)
    U_ref, W_ref = knm.knm_prod(X, C, 4.0, V, return_w=True)
    assert torch.equal(W, W_ref) and torch.equal(U, U_ref)
    rows = torch.arange(0, n, 997)
    Wo = oracle.knm_v(X[rows.cuda()].cpu().numpy(), C.cpu().numpy(), 4.0, V.cpu().numpy())
    assert rel_l2(W[rows.cuda()].cpu().numpy(), Wo) < 1e-4


def test_static_scratch_rejects_what_does_not_fit(knm):
    # 64 MiB hold the partials of chunks x M x t floats only up to a point
    n, M, d, t = 300000, 60000, 8, 16
    X = torch.zeros(n, d, device="cuda")
    C = torch.zeros(M, d, device="cuda")
    V = torch.zeros(M, t, device="cuda")
    W = torch.empty(n, t, device="cuda")
    U = torch.empty(M, t, device="cuda")
    with pytest.raises(knm.KnmError) as e:
        knm.knm_prod_static(X, C, 1.0, V, W, U)
    assert e.value.status == -2 and "static scratch" in str(e.value)
    with pytest.raises(knm.KnmError) as e:
        knm.load_library()  # keep the library handle alive for the raw call below
        ctx = knm.default_context()
        ctx.check(knm.load_library().knm_prod_static(ctx._h, X.data_ptr(), n, d, d, C.data_ptr(), M, d, 1.0,
                                                     V.data_ptr(), t, None, U.data_ptr()))
    assert e.value.status == -1
