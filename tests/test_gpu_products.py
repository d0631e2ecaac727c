"""GPU parity: the HIP kernel-matrix-vector products against the fp64 CPU oracle,
element by element on the same seeded inputs, through the C ABI (ctypes binding).

Bar: relative L2 error <= 1e-4 per product (the stated target); measured errors are
~1e-6, so the assertions use 2e-5 to catch regressions early.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4
TIGHT = 2e-5


@pytest.fixture(params=["f32", "f16x3"])
def cross(request, knm):
    """Runs a test once per cross-term arithmetic (fp32 MFMA / split-fp16 MFMA)."""
    ctx = knm.default_context()
    ctx.set_cross_term(request.param)
    yield request.param
    ctx.set_cross_term("f16x3")


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def _rand(n, d, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (scale * torch.randn(n, d, generator=g)).to(torch.float32)


SHAPES = [
    # n, M, d, t, sigma  -- several tiles plus ragged tails in every dimension
    (1000, 300, 8, 1, 2.0),
    (2049, 515, 28, 1, 4.0),
    (777, 129, 9, 1, 1.5),
    (4100, 1030, 5, 3, 1.0),
    (515, 2049, 28, 2, 4.0),
    (1500, 260, 1, 1, 0.7),
    (1300, 400, 33, 1, 5.0),
    (900, 300, 64, 1, 8.0),
    (640, 256, 12, 10, 2.5),
    # K-loop engine: d above the register-resident limit, several columns, unaligned d
    (515, 260, 130, 1, 8.0),
    (300, 129, 70, 5, 6.0),
    (600, 300, 784, 10, 24.0),
    (257, 385, 99, 3, 7.0),
    (1000, 2100, 16, 17, 3.0),
    # 8 columns and more: reduction against the vectors on the matrix cores, in 1, 2 or 4 groups of 32
    # columns per launch (5 groups, 160 columns, for the Gaussian kernel)
    (700, 390, 20, 32, 3.0),
    (500, 300, 6, 40, 1.5),
    (2300, 700, 28, 9, 4.0),
    (900, 520, 28, 64, 4.0),
    (520, 900, 50, 65, 5.0),
    (1100, 300, 440, 128, 20.0),
    (640, 385, 33, 144, 5.0),
    (300, 260, 300, 50, 18.0),
    (257, 300, 280, 70, 17.0),
    # five groups in one launch (160 columns), and one column left over
    (520, 385, 40, 161, 6.0),
]


@pytest.mark.parametrize("n,M,d,t,sigma", SHAPES)
def test_products_match_oracle(knm, cross, n, M, d, t, sigma):
    print(f"case n={n} M={M} d={d} t={t}", flush=True)
    X, C = _rand(n, d, 1), _rand(M, d, 2)
    V = _rand(M, t, 3)
    Y = _rand(n, t, 4)
    Xd, Cd, Vd, Yd = X.cuda(), C.cuda(), V.cuda(), Y.cuda()
    Xn, Cn = X.numpy(), C.numpy()

    W = knm.knm_v(Xd, Cd, sigma, Vd).cpu().numpy()
    assert rel_l2(W, oracle.knm_v(Xn, Cn, sigma, V.numpy())) < TIGHT

    R = knm.knm_t_y(Xd, Cd, sigma, Yd).cpu().numpy()
    assert rel_l2(R, oracle.knm_t_y(Xn, Cn, sigma, Y.numpy())) < TIGHT

    U, W2 = knm.knm_prod(Xd, Cd, sigma, Vd, return_w=True)
    Uo, Wo = oracle.knm_prod(Xn, Cn, sigma, V.numpy(), return_w=True)
    assert rel_l2(U.cpu().numpy(), Uo) < TIGHT
    assert rel_l2(W2.cpu().numpy(), Wo) < TIGHT
    # element by element as well: no single output may hide behind the norm of the others
    for got, ref in ((W, oracle.knm_v(Xn, Cn, sigma, V.numpy())), (R, oracle.knm_t_y(Xn, Cn, sigma, Y.numpy())),
                     (U.cpu().numpy(), Uo)):
        ref = np.asarray(ref).reshape(got.shape)
        assert np.max(np.abs(got - ref)) < TOL * np.max(np.abs(ref))
    for c in range(t):  # per column as well as Frobenius
        assert rel_l2(U.cpu().numpy().reshape(M, t)[:, c], np.asarray(Uo).reshape(M, t)[:, c]) < TOL
    # without the W output the library uses its own workspace: same result bit for bit
    U2 = knm.knm_prod(Xd, Cd, sigma, Vd)
    assert torch.equal(U2, U)


@pytest.mark.parametrize("kind", ["ones", "unit"])
def test_special_vectors(knm, cross, kind):
    n, M, d, sigma = 3000, 700, 28, 4.0
    X, C = _rand(n, d, 5), _rand(M, d, 6)
    v = synth.probe_vector(M, 1, kind, j=123)
    U = knm.knm_prod(X.cuda(), C.cuda(), sigma, v.cuda()).cpu().numpy()
    assert rel_l2(U, oracle.knm_prod(X.numpy(), C.numpy(), sigma, v.numpy())) < TIGHT


def test_columns_of_very_different_scale(knm):
    """Matrix-core reduction: every vector column is scaled by its own power of two into the fp16
    range, so columns of magnitude 1e-6 and 1e5, an all-zero column and a column dominated by one
    entry must each keep the product accuracy."""
    n, M, d, t, sigma = 1500, 600, 12, 12, 2.0
    X, C, V = _rand(n, d, 90), _rand(M, d, 91), _rand(M, t, 92)
    V[:, 1] *= 1e-6
    V[:, 2] *= 1e5
    V[:, 3] = 0.0
    V[17, 4] = 3.0e4           # one entry 1e4 times the rest of its column
    V[:, 5] = 1.0
    V[:, 6] *= 1e-30           # near the bottom of the fp32 range
    knm.default_context().set_cross_term("f16x3")
    W = knm.knm_v(X.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
    Wo = oracle.knm_v(X.numpy(), C.numpy(), sigma, V.numpy())
    assert np.array_equal(W[:, 3], np.zeros(n, dtype=np.float32))
    for c in range(t):
        if c != 3:
            assert rel_l2(W[:, c], Wo[:, c]) < TOL, c
    # the small entries of the outlier column are resolved relative to its largest entry
    assert np.abs(W[:, 4] - Wo[:, 4]).max() < 1e-6 * 3.0e4
    U = knm.knm_prod(X.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
    Uo = oracle.knm_prod(X.numpy(), C.numpy(), sigma, V.numpy())
    for c in range(t):
        if c != 3:
            assert rel_l2(U[:, c], Uo[:, c]) < TOL, c


@pytest.mark.parametrize("t", [2, 9, 70])  # vector-ALU reduction, matrix-core reduction, and its wide launch
def test_weighted_product(knm, cross, t):
    n, M, d, sigma = 2500, 300, 9, 2.0
    X, C, V = _rand(n, d, 7), _rand(M, d, 8), _rand(M, t, 9)
    dw = torch.rand(n, generator=torch.Generator().manual_seed(10)) + 0.05
    U = knm.knm_prod_weighted(X.cuda(), C.cuda(), sigma, dw.cuda(), V.cuda()).cpu().numpy()
    ref = oracle.knm_prod_weighted(X.numpy(), C.numpy(), sigma, dw.numpy(), V.numpy())
    assert rel_l2(U, ref) < TIGHT


def test_strided_points_and_determinism(knm, cross):
    n, M, d, sigma = 1200, 333, 10, 2.0
    Xw = _rand(n, 16, 11).cuda()
    Cw = _rand(M, 13, 12).cuda()
    X, C = Xw[:, :d], Cw[:, :d]  # leading dimension larger than d, odd for C
    V = _rand(M, 1, 13).cuda()
    U1 = knm.knm_prod(X, C, sigma, V)
    U2 = knm.knm_prod(X, C, sigma, V)
    assert torch.equal(U1, U2)
    ref = oracle.knm_prod(X.cpu().numpy(), C.cpu().numpy(), sigma, V.cpu().numpy())
    assert rel_l2(U1.cpu().numpy(), ref) < TIGHT


@pytest.mark.parametrize("d,t", [(10, 3), (70, 1), (52, 1)])
def test_strided_unaligned_points_on_the_k_loop_engine(knm, cross, d, t):
    # leading dimensions larger than d and base pointers that are only 4-byte aligned: the
    # scalar-load paths of the packing and staging code
    n, M, sigma = 900, 333, 3.0
    Xw = _rand(n, d + 7, 41).cuda()
    Cw = _rand(M * (d + 3) + 1, 1, 42).cuda().reshape(-1)[1:].reshape(M, d + 3)
    X, C = Xw[:, 1:d + 1], Cw[:, :d]
    V = _rand(M, t, 43).cuda()
    U = knm.knm_prod(X, C, sigma, V)
    ref = oracle.knm_prod(X.cpu().numpy(), C.cpu().numpy(), sigma, V.cpu().numpy())
    assert rel_l2(U.cpu().numpy(), ref) < TIGHT


def test_degenerate_sizes(knm, cross):
    sigma = 1.0
    X, C = _rand(1, 3, 14), _rand(1, 3, 15)
    v = torch.tensor([[2.0]])
    U = knm.knm_prod(X.cuda(), C.cuda(), sigma, v.cuda()).cpu().numpy()
    k = oracle.gauss(X.numpy()[0], C.numpy()[0], sigma)
    assert U.ravel()[0] == pytest.approx(2.0 * k * k, rel=1e-5)
    # identical points: kernel exactly 1 on the diagonal, never above
    P = _rand(200, 28, 16, scale=3.0).cuda()
    W = knm.knm_v(P, P, 0.5, torch.ones(200, 1).cuda())  # small sigma: off-diagonal underflows to 0
    Wn = W.cpu().numpy()
    assert np.all(np.isfinite(Wn)) and Wn.max() <= 1.0 and Wn.min() >= 0.0
    assert np.allclose(Wn, 1.0, atol=2e-3)
    # far-apart points: exact zeros, no NaN / Inf
    far = torch.zeros(64, 4)
    far[:, 0] = 1.0e4
    W = knm.knm_v(far.cuda(), torch.zeros(64, 4).cuda(), 1.0, torch.ones(64, 1).cuda()).cpu().numpy()
    assert np.array_equal(W, np.zeros_like(W))


def test_large_norm_close_pairs(knm, cross):
    """Data far from the origin (|x|^2 ~ 1000 sigma^2) with small mutual distances: the norm expansion
    alone would keep only ~1e-4 of the exponent; the engines expand around the centres' mean, so the
    accuracy is that of centred data.  A second case moves single points far away from that mean."""
    n, M, d, sigma = 2000, 256, 8, 1.0
    X = 11.0 + 0.5 * _rand(n, d, 18)
    C = 11.0 + 0.5 * _rand(M, d, 19)
    V = torch.ones(M, 1)
    W = knm.knm_v(X.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
    err = rel_l2(W, oracle.knm_v(X.numpy(), C.numpy(), sigma, V.numpy()))
    print(f"offset data: {err:.2e}", flush=True)
    assert err < TIGHT
    U = knm.knm_t_y(X.cuda(), C.cuda(), sigma, torch.ones(n, 1).cuda()).cpu().numpy()
    assert rel_l2(U, oracle.knm_t_y(X.numpy(), C.numpy(), sigma, np.ones((n, 1)))) < TIGHT
    # outliers in the data (not among the centres): their rows are far from everything, the rest is unaffected
    X2 = X.clone()
    X2[::97] += 40.0
    W2 = knm.knm_v(X2.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
    assert rel_l2(W2, oracle.knm_v(X2.numpy(), C.numpy(), sigma, V.numpy())) < TIGHT


def test_split_half_range_limits(knm):
    """The split-fp16 cross term saturates instead of producing Inf/NaN, and huge norms
    (far outliers) still give exact zeros against ordinary points."""
    ctx = knm.default_context()
    ctx.set_cross_term("f16x3")
    try:
        n, M, d, sigma = 512, 256, 9, 1.0
        X, C = _rand(n, d, 50), _rand(M, d, 51)
        X[7, 3] = 3.0e2       # norm term ~ 6.5e4: needs the upper fixed-point digits
        X[11, 0] = 2.0e5      # beyond fp16: saturates
        C[5] = X[7]           # an outlier centre equal to an outlier row
        V = torch.ones(M, 1)
        W = knm.knm_v(X.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
        Wo = oracle.knm_v(X.numpy(), C.numpy(), sigma, V.numpy())
        assert np.all(np.isfinite(W))
        keep = np.ones(n, dtype=bool)
        keep[11] = False
        keep[7] = False       # its twin centre: |x|^2 ~ 1e5 cancels to 0; the split halves leave out 2.4e-7 of it,
                              # about 0.02 in the exponent (unless 300 minus the common shift happens to be a half)
        assert rel_l2(W[keep], Wo[keep]) < 1e-4
        assert W[7, 0] == pytest.approx(Wo[7, 0], rel=5e-2) and Wo[7, 0] >= 1.0  # sees its twin centre
        assert abs(W[11, 0]) < 1e-6
        # the clamped conversion of row 11 is reported, and only that one
        assert ctx.range_exceeded() >= 1
        assert ctx.range_exceeded() == 0  # the query resets the count
        X[11, 0] = 1.0
        knm.knm_v(X.cuda(), C.cuda(), sigma, V.cuda())
        assert ctx.range_exceeded() == 0
    finally:
        ctx.set_cross_term("f16x3")


@pytest.mark.parametrize("d,t", [(9, 1), (28, 1), (60, 1), (12, 3)])  # every packing kernel and the fixed-point prologue
def test_clamped_and_non_finite_operands_are_counted(knm, d, t):
    """Scaled features beyond +-65000, norm terms beyond 2^21 and NaNs are clamped by the split-fp16
    conversion: the device counter reports them, whichever operand role the point has, and the
    fp32-MFMA mode counts nothing."""
    ctx = knm.default_context()
    n, M, sigma = 700, 300, 2.0
    X, C, V = _rand(n, d, 52), _rand(M, d, 53), _rand(M, t, 54)
    ctx.range_exceeded()
    knm.knm_prod(X.cuda(), C.cuda(), sigma, V.cuda())
    assert ctx.range_exceeded() == 0
    for where, row, value in (("X", 650, 4.0e5), ("X", 3, float("nan")), ("C", 299, 7000.0), ("C", 0, float("inf"))):
        Xb, Cb = X.clone(), C.clone()
        (Xb if where == "X" else Cb)[row, d - 1] = value  # 7000 / sigma: norm term 9e6 > 2^21, feature in range
        knm.knm_prod(Xb.cuda(), Cb.cuda(), sigma, V.cuda())
        assert ctx.range_exceeded() >= 1, (where, row, value)
        ctx.set_cross_term("f32")
        try:
            knm.knm_prod(Xb.cuda(), Cb.cuda(), sigma, V.cuda())
            assert ctx.range_exceeded() == 0
        finally:
            ctx.set_cross_term("f16x3")


@pytest.mark.parametrize("d,t,limit", [(28, 1, 300 << 10), (9, 1, 200 << 10), (130, 1, 4 << 20), (16, 5, 1 << 20)])
def test_results_do_not_depend_on_the_pack_workspace_cap(knm, d, t, limit):
    """With a small cap the split-fp16 engines convert and sweep their operands slab by slab (the
    path the billion-row workload takes); the results must be the same bit for bit."""
    n, M, sigma = 20000, 3000, 3.0
    X, C, V = _rand(n, d, 60).cuda(), _rand(M, d, 61).cuda(), _rand(M, t, 62).cuda()
    ctx = knm.default_context()
    ctx.set_cross_term("f16x3")
    U0, W0 = knm.knm_prod(X, C, sigma, V, return_w=True)
    try:
        ctx.set_pack_limit(limit)
        U1, W1 = knm.knm_prod(X, C, sigma, V, return_w=True)
    finally:
        ctx.set_pack_limit(0)
    assert torch.equal(W0, W1) and torch.equal(U0, U1)
    ref = oracle.knm_prod(X[:3000].cpu().numpy(), C.cpu().numpy(), sigma, V.cpu().numpy())
    assert rel_l2(knm.knm_prod(X[:3000], C, sigma, V).cpu().numpy(), ref) < TIGHT


def test_invalid_arguments_are_rejected(knm):
    X, C, V = _rand(10, 4, 20).cuda(), _rand(5, 4, 21).cuda(), _rand(5, 1, 22).cuda()
    with pytest.raises(knm.KnmError) as e:
        knm.knm_prod(X, C, -1.0, V)
    assert e.value.status == -1
    big = _rand(4, knm.load_library().knm_max_d() + 1, 23).cuda()
    with pytest.raises(knm.KnmError) as e:
        knm.knm_v(big, big, 1.0, _rand(4, 1, 24).cuda())
    assert e.value.status == -2
    with pytest.raises(ValueError):
        knm.knm_v(X, _rand(5, 3, 25).cuda(), 1.0, V)


def test_tiny_workload_full_product(knm, cross):
    w = synth.workload("tiny")
    inp = synth.make_inputs(w, device="cpu")
    X, C = inp["X"], inp["C"]
    v = synth.probe_vector(w.M, w.t, "normal")
    U, W = knm.knm_prod(X.cuda(), C.cuda(), w.sigma, v.cuda(), return_w=True)
    Uo, Wo = oracle.knm_prod(X.numpy(), C.numpy(), w.sigma, v.numpy(), return_w=True)
    assert rel_l2(W.cpu().numpy(), Wo) < TIGHT
    assert rel_l2(U.cpu().numpy(), Uo) < TIGHT
    R = knm.knm_t_y(X.cuda(), C.cuda(), w.sigma, inp["Y"].cuda())
    assert rel_l2(R.cpu().numpy(), oracle.knm_t_y(X.numpy(), C.numpy(), w.sigma, inp["Y"].numpy())) < TIGHT


@pytest.mark.parametrize("name,n_sub,M_sub", [("mid", 1 << 15, 4096), ("lowdim", 1 << 15, 4096), ("billion", 1 << 15, 4096)])
def test_workload_shaped_sample(knm, cross, name, n_sub, M_sub):
    """Rows and centres drawn with a workload's distribution (heavy tails included)."""
    w = synth.workload(name, n=n_sub, M=M_sub)
    inp = synth.make_inputs(w, device="cpu", with_targets=False)
    X, C = inp["X"], inp["C"]
    v = synth.probe_vector(w.M, 1, "normal")
    U = knm.knm_prod(X.cuda(), C.cuda(), w.sigma, v.cuda()).cpu().numpy()
    assert rel_l2(U, oracle.knm_prod(X.numpy(), C.numpy(), w.sigma, v.numpy())) < TOL


@pytest.mark.parametrize("n,M,d,t,sigma", [(3000, 700, 28, 1, 4.0), (2100, 600, 100, 12, 7.0), (1500, 400, 9, 3, 2.0),
                                             (1800, 500, 40, 40, 5.0)])  # the last: packed vector image, wide launch
def test_product_replays_in_a_graph(knm, n, M, d, t, sigma):
    """Once the workspace exists (one eager call with the same shapes) a product only enqueues kernels
    on the context's stream, so it can be captured into a graph.  Every replay, with new inputs and
    eager work in between, must give the eager result bit for bit."""
    side = torch.cuda.Stream()
    X, C, V = _rand(n, d, 70).cuda(), _rand(M, d, 71).cuda(), _rand(M, t, 72).cuda()
    U = torch.empty(M, t, device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        ctx = knm.Context()  # bound to the side stream
        knm.knm_prod(X, C, sigma, V, out=U, ctx=ctx)  # allocates the workspace
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            knm.knm_prod(X, C, sigma, V, out=U, ctx=ctx)
    torch.cuda.synchronize()
    for rep in range(4):
        print(f"replay {rep}", flush=True)
        X.copy_(_rand(n, d, 80 + rep).cuda())
        V.copy_(_rand(M, t, 90 + rep).cuda())
        if rep == 2:
            V[:, 0] = 0.0
        U.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = U.clone()
        want = knm.knm_prod(X, C, sigma, V)  # eager, default context and stream
        torch.cuda.synchronize()
        assert torch.equal(got, want.reshape(M, t)), rep
        assert rel_l2(got.cpu().numpy(), oracle.knm_prod(X.cpu().numpy(), C.cpu().numpy(), sigma, V.cpu().numpy())) < TIGHT
    del graph
    ctx.close()


@pytest.mark.parametrize("n,M,d,t", [(30000, 2000, 8, 1), (9000, 1500, 100, 3), (5000, 700, 28, 12), (4000, 900, 60, 70)])
def test_workspace_held_stays_within_the_announced_bound(knm, n, M, d, t):
    """knm_workspace_bytes is an upper bound on what a context holds after the products of that
    shape, in every arithmetic mode and for both kernel functions."""
    X, C, V, Y = _rand(n, d, 60).cuda(), _rand(M, d, 61).cuda(), _rand(M, t, 62).cuda(), _rand(n, t, 63).cuda()
    bound = int(knm.load_library().knm_workspace_bytes(n, M, d, t))
    for mode in ("f16x3", "f32"):
        for kind in ("gaussian", "laplacian"):
            ctx = knm.Context()
            ctx.set_cross_term(mode)
            ctx.set_kernel(kind)
            assert ctx.workspace_held() == 0
            knm.knm_prod(X, C, 3.0, V, ctx=ctx)
            knm.knm_t_y(X, C, 3.0, Y, ctx=ctx)
            held = ctx.workspace_held()
            print(f"{mode} {kind}: held {held} of {bound}", flush=True)
            assert 0 < held <= bound
            ctx.close()


@pytest.mark.parametrize("t", [9, 20])
def test_matrix_core_reduction_keeps_small_kernel_values(knm, t):
    """Data and centres in two clusters far apart: the kernel values lie around and below fp16's
    normal range (6e-5), most of them by orders of magnitude.  With 8 or more columns the kernel values go through
    fp16 halves, which must still resolve them relative to themselves."""
    n, M, d = 600, 300, 28
    X, C, V = _rand(n, d, 101), _rand(M, d, 102) + 3.0, _rand(M, t, 103)
    knm.default_context().set_cross_term("f16x3")
    for sigma in (3.1, 2.7):  # kernel values up to 5e-4 and up to 5e-5 (median 1e-7 and 1e-9)
        assert oracle.kernel_matrix(X.numpy(), C.numpy(), sigma).max() < 1e-3
        Wo = oracle.knm_v(X.numpy(), C.numpy(), sigma, V.numpy())
        W = knm.knm_v(X.cuda(), C.cuda(), sigma, V.cuda()).cpu().numpy()
        print(f"sigma {sigma}: |W| {np.linalg.norm(Wo):.2e} error {rel_l2(W, Wo):.2e}", flush=True)
        assert rel_l2(W, Wo) < TOL
