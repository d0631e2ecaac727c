"""GPU parity on seeded random draws of everything a product call can vary: sizes around the tile
boundaries, feature counts around the engines' limits, column counts around the launch groups,
leading dimensions, pointer alignment, the kernel function, the cross-term arithmetic, centres that
are data rows or not.  Every draw is checked against the fp64 CPU oracle through the C ABI.

Bar: relative L2 error <= 1e-4 per product; the assertion uses 2e-5 (measured: below 4e-6 over
1200 draws).
"""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

SIZES_N = [1, 2, 31, 33, 64, 127, 129, 255, 257, 300, 511, 513, 1000, 1025, 2047, 3000]
SIZES_M = [1, 2, 31, 32, 33, 63, 65, 127, 129, 255, 256, 257, 400, 513, 1030]
SIZES_D = [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 28, 31, 32, 33, 43, 44, 45, 47, 48, 49, 63, 64, 65, 70, 100, 130, 257]
SIZES_T = [1, 1, 1, 2, 3, 4, 5, 7, 8, 9, 12, 15, 16, 17, 31, 32, 33]
KINDS = ["gaussian", "gaussian", "laplacian", "matern32", "matern52"]


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


@pytest.mark.parametrize("block", range(8))
def test_random_draws_match_oracle(knm, block):
    ctx = knm.default_context()
    try:
        for case in range(12):
            seed = 9000 + 12 * block + case
            rng = np.random.default_rng(seed)
            n, M = int(rng.choice(SIZES_N)), int(rng.choice(SIZES_M))
            d, t = int(rng.choice(SIZES_D)), int(rng.choice(SIZES_T))
            kind, cross = str(rng.choice(KINDS)), str(rng.choice(["f16x3", "f32"]))
            # length-scales from small (the norm terms are large in the engines' units) to large
            # (they are far below one)
            sigma = float(rng.choice([0.5, 1.0, 2.0, 8.0]) * np.sqrt(d))
            padx, padc = int(rng.integers(0, 4)), int(rng.integers(0, 4))
            offx, offc = int(rng.integers(0, 2)), int(rng.integers(0, 2))
            g = torch.Generator().manual_seed(seed)
            Xw = torch.randn(n * (d + padx) + offx, generator=g)
            Cw = torch.randn(M * (d + padc) + offc, generator=g)
            if rng.random() < 0.5 and n >= M:  # Nystrom centres: rows of the data
                rows = torch.randperm(n, generator=g)[:M]
                Cw[offc:].reshape(M, d + padc)[:, :d] = Xw[offx:].reshape(n, d + padx)[rows, :d]
            V, Y = torch.randn(M, t, generator=g), torch.randn(n, t, generator=g)
            dw = torch.rand(n, generator=g) + 0.1
            print(f"seed {seed}: n={n} M={M} d={d} t={t} sigma={sigma:.3g} {kind} {cross} ld=({d + padx},{d + padc}) "
                  f"offset=({offx},{offc})", flush=True)
            Xd = Xw.cuda()[offx:].reshape(n, d + padx)[:, :d]
            Cd = Cw.cuda()[offc:].reshape(M, d + padc)[:, :d]
            Xn = Xw[offx:].reshape(n, d + padx)[:, :d].contiguous().numpy()
            Cn = Cw[offc:].reshape(M, d + padc)[:, :d].contiguous().numpy()
            ctx.set_cross_term(cross)
            ctx.set_kernel(kind)
            with oracle.kernel(kind):
                U, W = knm.knm_prod(Xd, Cd, sigma, V.cuda(), return_w=True)
                Uo, Wo = oracle.knm_prod(Xn, Cn, sigma, V.numpy(), return_w=True)
                R = knm.knm_t_y(Xd, Cd, sigma, Y.cuda())
                Ro = oracle.knm_t_y(Xn, Cn, sigma, Y.numpy())
                Uw = knm.knm_prod_weighted(Xd, Cd, sigma, dw.cuda(), V.cuda())
                Uwo = oracle.knm_prod_weighted(Xn, Cn, sigma, dw.numpy(), V.numpy())
            errs = [rel_l2(U.cpu().numpy(), Uo), rel_l2(W.cpu().numpy(), Wo), rel_l2(R.cpu().numpy(), Ro),
                    rel_l2(Uw.cpu().numpy(), Uwo)]
            assert max(errs) < 2e-5, (seed, errs)
    finally:
        ctx.set_kernel("gaussian")
        ctx.set_cross_term("f16x3")


@pytest.mark.parametrize("cross", ["f16x3", "f32"])
def test_distance_kernels_with_norms_far_below_one(knm, cross):
    """A length-scale so large that the norm terms the engines carry are far below one: coincident
    pairs (centres are data rows) must still be recognised as close and evaluated from differences."""
    n, M, d = 511, 31, 15
    g = torch.Generator().manual_seed(77)
    X = torch.randn(n, d, generator=g)
    C = X[torch.randperm(n, generator=g)[:M]].clone()
    Y = torch.randn(n, 1, generator=g)
    ctx = knm.default_context()
    ctx.set_cross_term(cross)
    try:
        for kind in ("laplacian", "matern32"):
            ctx.set_kernel(kind)
            for sigma in (8.0, 30.0, 300.0):
                with oracle.kernel(kind):
                    R = knm.knm_t_y(X.cuda(), C.cuda(), sigma, Y.cuda()).cpu().numpy()
                    Ro = oracle.knm_t_y(X.numpy(), C.numpy(), sigma, Y.numpy())
                    W = knm.knm_v(X.cuda(), C.cuda(), sigma, torch.ones(M, 1).cuda()).cpu().numpy()
                    Wo = oracle.knm_v(X.numpy(), C.numpy(), sigma, np.ones((M, 1)))
                print(f"{kind} sigma={sigma}: {rel_l2(R, Ro):.2e} {rel_l2(W, Wo):.2e}", flush=True)
                assert rel_l2(R, Ro) < 2e-5 and rel_l2(W, Wo) < 2e-5
    finally:
        ctx.set_kernel("gaussian")
        ctx.set_cross_term("f16x3")
