"""Full-size parity in the launch configuration the benchmark times: the mid workload
(n = 11M, d = 28, M = 100k), the low-dimensional one (n = 5.9M, d = 8, M = 100k) and the
high-dimensional multi-output one (n = 2M, d = 784, M = 50k, t = 10; the K-loop engine).

The oracle cannot sweep 1e12 entries, so it checks sampled outputs one by one: rows of
W = K V (each needs all M centres) and entries of R = K^T Y (each needs all n rows), plus
identities that hold at any size.
"""
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


@pytest.fixture
def kernel_kind(request, knm):
    """Sets the kernel function on the default context and in the oracle for one test."""
    kind = getattr(request, "param", "gaussian")
    knm.default_context().set_kernel(kind)
    with oracle.kernel(kind):
        yield kind
    knm.default_context().set_kernel("gaussian")


@pytest.fixture
def cross_term(request, knm):
    """Sets the arithmetic of the cross term on the default context for one test."""
    mode = getattr(request, "param", "f16x3")
    knm.default_context().set_cross_term(mode)
    yield mode
    knm.default_context().set_cross_term("f16x3")


@pytest.mark.parametrize("name,n_rows,n_cols,kernel_kind,cross_term",
                         [("mid", 503, 6, "gaussian", "f16x3"), ("mid", 503, 6, "gaussian", "f32"),
                          ("lowdim", 503, 6, "gaussian", "f16x3"), ("highdim", 120, 2, "gaussian", "f16x3"),
                          ("mid", 503, 6, "laplacian", "f16x3")], indirect=["kernel_kind", "cross_term"])
def test_full_size_sampled_outputs(knm, name, n_rows, n_cols, kernel_kind, cross_term):
    w = synth.workload(name)
    print(f"workload {name}: n={w.n} d={w.d} M={w.M} kernel={kernel_kind} cross term={cross_term}", flush=True)
    inp = synth.make_inputs(w, device="cuda", with_targets=True)
    X, C, Y = inp["X"], inp["C"], inp["Y"]
    v = synth.probe_vector(w.M, w.t, "normal", device="cuda")
    U, W = knm.knm_prod(X, C, w.sigma, v, return_w=True)
    R = knm.knm_t_y(X, C, w.sigma, Y)
    torch.cuda.synchronize()
    print("gpu products done", flush=True)

    Cn = C.cpu().numpy()
    vn = v.cpu().numpy()
    g = np.random.default_rng(7)

    # rows of W = K V: first and last tiles plus random rows
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 255, 256, w.n - 257, w.n - 2, w.n - 1], g.integers(0, w.n, n_rows)]))
    Xs = X[torch.from_numpy(rows).cuda()].cpu().numpy()
    Wo = oracle.knm_v(Xs, Cn, w.sigma, vn)
    Wg = W[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert rel_l2(Wg, Wo) < 1e-4
    assert np.max(np.abs(Wg - Wo)) < 1e-4 * np.max(np.abs(Wo)) + 1e-6
    print("row samples ok", flush=True)

    # entries of R = K^T Y: every one is a sum over all n rows
    cols = np.unique(np.concatenate([[0, 31, 32, 255, 256, w.M - 1], g.integers(0, w.M, n_cols)]))
    Xn = X.cpu().numpy()
    Yn = Y.cpu().numpy()
    Ro = oracle.knm_t_y(Xn, Cn[cols], w.sigma, Yn)
    Rg = R[torch.from_numpy(cols).cuda()].cpu().numpy()
    assert rel_l2(Rg, Ro) < 1e-4
    print("column samples ok", flush=True)

    # the same column entries of U = K^T W, with the GPU's own W as the oracle's input
    Wn = W.cpu().numpy()
    Uo = oracle.knm_t_y(Xn, Cn[cols], w.sigma, Wn)
    Ug = U[torch.from_numpy(cols).cuda()].cpu().numpy()
    assert rel_l2(Ug, Uo) < 1e-4

    # identities at full size: v^T K^T K v = |K v|^2 and U = K^T W bit for bit
    uv = float((U.double() * v.double()).sum())
    ww = float((W.double() ** 2).sum())
    assert abs(uv - ww) <= 1e-4 * float(U.double().norm() * v.double().norm())
    U2 = knm.knm_t_y(X, C, w.sigma, W)
    assert torch.equal(U2, U)


def test_more_than_2_pow_31_elements(knm):
    """64-bit indexing end to end: n d = 2.34e9 > 2^31 elements of X (billion-shaped rows, n = 260M).
    Rows of W at both ends of the array against the oracle; K^T W of the last rows against the
    oracle; and the whole product as the sum of the products of two row ranges (linearity)."""
    w = synth.workload("billion", n=260_000_000)
    assert w.n * w.d > 2 ** 31
    print(f"workload billion-shaped: n={w.n} d={w.d} M={w.M}", flush=True)
    inp = synth.make_inputs(w, device="cuda", with_targets=False)
    X, C = inp["X"], inp["C"]
    v = synth.probe_vector(w.M, 1, "normal", device="cuda")
    U, W = knm.knm_prod(X, C, w.sigma, v, return_w=True)
    torch.cuda.synchronize()
    print("gpu product done", flush=True)
    Cn, vn = C.cpu().numpy(), v.cpu().numpy()
    g = np.random.default_rng(11)
    rows = np.unique(np.concatenate([[0, 1, 255, 256], w.n - 1 - np.arange(300), g.integers(0, w.n, 200)]))
    ridx = torch.from_numpy(rows).cuda()
    Wo = oracle.knm_v(X[ridx].cpu().numpy(), Cn, w.sigma, vn)
    assert rel_l2(W[ridx].cpu().numpy(), Wo) < 1e-4
    print("row samples ok", flush=True)

    tail = 1_000_000
    Xt, Wt = X[w.n - tail:], W[w.n - tail:]
    Ut = knm.knm_t_y(Xt, C, w.sigma, Wt)
    cols = np.array([0, 31, 32, 4097, w.M - 1])
    Uo = oracle.knm_t_y(Xt.cpu().numpy(), Cn[cols], w.sigma, Wt.cpu().numpy())
    assert rel_l2(Ut[torch.from_numpy(cols).cuda()].cpu().numpy(), Uo) < 1e-4
    Uh = knm.knm_t_y(X[: w.n - tail], C, w.sigma, W[: w.n - tail])
    assert rel_l2((Uh.double() + Ut.double()).cpu().numpy(), U.double().cpu().numpy()) < 1e-5
    uv = float((U.double() * v.double()).sum())
    ww = float((W.double() ** 2).sum())
    assert abs(uv - ww) <= 1e-4 * float(U.double().norm() * v.double().norm())


def test_billion_point_workload_sampled_outputs(knm):
    """The billion-point workload at its own size (n = 1e9, d = 9: 9e9 elements of X, past 2^32;
    36 GB resident), both sweeps launched over all n rows.  Rows of W = K V at both ends of the array
    and at random places against the oracle.  For the column sweep the oracle cannot sum 1e9 rows,
    so the sweep runs on a vector that is W on the last million rows and on scattered single rows
    (some past element 2^32, some before) and zero elsewhere: its result is a sum over those rows
    only, which the oracle computes from the gathered rows, while the kernel still indexes all of X."""
    w = synth.workload("billion")
    assert w.n * w.d > 2 ** 32
    inp = synth.make_inputs(w, device="cuda", with_targets=False)
    X, C = inp["X"], inp["C"]
    v = synth.probe_vector(w.M, 1, "normal", device="cuda")
    W = knm.knm_v(X, C, w.sigma, v)
    torch.cuda.synchronize()
    print("row sweep done", flush=True)
    Cn, vn = C.cpu().numpy(), v.cpu().numpy()
    g = np.random.default_rng(13)
    first_past = 2 ** 32 // w.d  # first row with an element past 2^32
    rows = np.unique(np.concatenate([[0, 1, 255, 256, first_past - 1, first_past, first_past + 1], w.n - 1 - np.arange(300),
                                     g.integers(0, w.n, 200)]))
    ridx = torch.from_numpy(rows).cuda()
    Wo = oracle.knm_v(X[ridx].cpu().numpy(), Cn, w.sigma, vn)
    Wg = W[ridx].cpu().numpy()
    assert rel_l2(Wg, Wo) < 1e-4
    assert np.max(np.abs(Wg - Wo)) < 1e-4 * np.max(np.abs(Wo)) + 1e-6
    print("row samples ok", flush=True)

    tail = 1_000_000
    single = np.unique(np.concatenate([[0, 1, 4095, first_past - 1, first_past, first_past + 4097],
                                       g.integers(0, w.n - tail, 2000)]))
    keep = torch.cat([torch.from_numpy(single).cuda(), torch.arange(w.n - tail, w.n, device="cuda")])
    Wm = torch.zeros_like(W)
    Wm[keep] = W[keep]
    Um = knm.knm_t_y(X, C, w.sigma, Wm)
    torch.cuda.synchronize()
    print("column sweep done", flush=True)
    cols = np.array([0, 31, 32, 4097, w.M - 1])
    Uo = oracle.knm_t_y(X[keep].cpu().numpy(), Cn[cols], w.sigma, W[keep].cpu().numpy())
    assert rel_l2(Um[torch.from_numpy(cols).cuda()].cpu().numpy(), Uo) < 1e-4
    # and the full product's identity v^T K^T K v = |K v|^2 over all 1e9 rows
    U = knm.knm_t_y(X, C, w.sigma, W)
    uv = float((U.double() * v.double()).sum())
    ww = float((W.double() ** 2).sum())
    assert abs(uv - ww) <= 1e-4 * float(U.double().norm() * v.double().norm())


@pytest.mark.parametrize("M", [100_000, 140_001])
def test_full_size_preconditioner_sampled_entries(knm, M):
    """Both factors at M = 100k (80 GB in one shared array) and at an odd M = 140001 (157 GB; two
    separate arrays of that order would not fit the GPU) against their defining identities on sampled index
    pairs: T^T T = K_MM + jitter I entry by entry against the oracle's kernel values, and
    A^T A = T T^T / M + lambda I with the right-hand side summed on the host from rows of T.
    The blocked solves are checked through the adjoint identity c^T (T^-1 A^-1 b) = (A^-T T^-T c)^T b."""
    w = synth.workload("mid", n=1_000_000, M=M)
    jitter = 1e-8
    inp = synth.make_inputs(w, device="cuda", with_targets=False)
    C = inp["C"]
    del inp
    print(f"building the preconditioner: M={M} d={w.d} lambda={w.lam}", flush=True)
    free0 = torch.cuda.mem_get_info()[0]
    pre = knm.precond_build(C, w.sigma, w.lam, jitter)
    held = free0 - torch.cuda.mem_get_info()[0]
    print(f"preconditioner built, holds {held / 1e9:.1f} GB", flush=True)
    assert held < 1.06 * 8.0 * M * M  # one shared array (+ the inverted diagonal blocks), not two
    Cn = C.cpu().numpy()
    g = np.random.default_rng(11)
    # (rows of a factor are strided in memory and slow to copy out: fewer samples at the larger size)
    idx = np.concatenate([[0, 1, 127, 128, 2047, 2048, 4095, 4096, M - 4097, M - 2, M - 1], g.integers(0, M, 8)])
    if M > 100_000:
        idx = np.concatenate([[0, 128, 4095, 4096, M - 4097, M - 1], g.integers(0, M, 2)])
    pairs = [(int(min(a, b)), int(max(a, b))) for a, b in zip(idx, g.permutation(idx))] + [(int(a), int(a)) for a in idx[:6]]
    worst_t = worst_a = 0.0
    for i, j in pairs:
        ti = pre.block(False, 0, i, i + 1, 1)[:, 0]          # column i of T down to its diagonal
        tj = pre.block(False, 0, j, i + 1, 1)[:, 0]          # column j of T, same rows
        want = oracle.gauss(Cn[i], Cn[j], w.sigma) + (jitter if i == j else 0.0)
        worst_t = max(worst_t, abs(float(ti @ tj) - want))
        ai = pre.block(True, 0, i, i + 1, 1)[:, 0]
        aj = pre.block(True, 0, j, i + 1, 1)[:, 0]
        ri = pre.block(False, i, j, 1, M - j)[0]              # row i of T from column j on
        rj = pre.block(False, j, j, 1, M - j)[0]              # row j of T from its diagonal on
        want = float(ri @ rj) / M + (w.lam if i == j else 0.0)
        worst_a = max(worst_a, abs(float(ai @ aj) - want))
    print(f"worst |T^T T - K| = {worst_t:.3e}, worst |A^T A - (T T^T / M + lambda I)| = {worst_a:.3e}", flush=True)
    assert worst_t < 1e-12  # entries of K are in [0, 1]; measured 2e-15
    assert worst_a < 1e-12  # entries of T T^T / M are below max K_ii = 1; measured 3e-16

    gt = torch.Generator().manual_seed(12)
    b = torch.randn(M, generator=gt, dtype=torch.float64)
    c = torch.randn(M, generator=gt, dtype=torch.float64)
    x = pre.solve(b.cuda()).cpu()
    y = pre.solve(c.cuda(), transpose=True).cpu()
    lhs, rhs = float(c @ x), float(y @ b)
    print(f"adjoint identity: {lhs:.12e} vs {rhs:.12e}", flush=True)
    assert abs(lhs - rhs) <= 1e-8 * float(torch.linalg.norm(c) * torch.linalg.norm(x))
    pre.close()


def test_full_size_sparse_sampled_outputs(knm):
    """The sparse product at the benchmark's size (n = 1.5M rows, d = 6.5e7 features, M = 50k
    centres), with and without the dense treatment of the most frequent features.  The dense
    oracle cannot hold 6.5e7 columns, so a sampled output is checked on the features of the one
    point it belongs to: with S the features of x_r, k(x_r, c_j) is the oracle's kernel of the
    parts in S times exp(-(|c_j|^2 - |c_j restricted to S|^2) / 2 sigma^2), a factor computed here in
    fp64 and folded into the vector; likewise for a column of U with S the features of c_j."""
    n, M, d, sigma = 1_500_000, 50_000, 65_000_000, 20.0
    s = synth.sparse_inputs(n, M, d, nnz_per_row=100.0, skew=2.5, seed=6, device="cuda")
    X = torch.sparse_csr_tensor(s["x_indptr"], s["x_indices"], s["x_values"], size=(n, d), check_invariants=False)
    C = torch.sparse_csr_tensor(s["c_indptr"], s["c_indices"], s["c_values"], size=(M, d), check_invariants=False)
    v = synth.probe_vector(M, 1, "normal", device="cuda")
    ctx = knm.default_context()

    def parts(prefix, rows):
        ip, ix, val = s[prefix + "_indptr"], s[prefix + "_indices"], s[prefix + "_values"]
        owner = torch.repeat_interleave(torch.arange(rows, device="cuda"), torch.diff(ip))
        norms = torch.zeros(rows, dtype=torch.float64, device="cuda").index_add_(0, owner, val.double() ** 2)
        return ip, ix, val, owner, norms

    def restricted(prefix, rows, S):
        """Dense (rows x |S|) image of the matrix's entries in the sorted feature set S, and the
        fp64 factor of every row's remaining squared norm."""
        ip, ix, val, owner, norms = parts(prefix, rows)
        keep = torch.isin(ix, S)
        dense = torch.zeros(rows, max(int(S.numel()), 1), dtype=torch.float32, device="cuda")
        dense[owner[keep], torch.searchsorted(S, ix[keep])] = val[keep]
        rest = (norms - (dense.double() ** 2).sum(1)).clamp_min(0.0)
        return dense.cpu().numpy(), torch.exp(-rest / (2.0 * sigma * sigma)).cpu().numpy()

    def check(v, label):
        results = {}
        for limit in (128, 0):
            ctx.set_sparse_head_limit(limit)
            U, W = knm.knm_prod_csr(X, C, sigma, v, return_w=True)
            torch.cuda.synchronize()
            results[limit] = (U, W)
            print(f"{label}, head limit {limit}: product done", flush=True)
        ctx.set_sparse_head_limit(128)
        vn = v.cpu().numpy().astype(np.float64).reshape(M)

        centre_rows = s["centre_rows"].cpu().numpy()
        sample_rows = [0, 1, 97, int(centre_rows[0]), int(centre_rows[-1]), n - 1, 123_457, 1_000_003]  # 0 and 97 are empty rows
        for r in sample_rows:
            p0, p1 = int(s["x_indptr"][r]), int(s["x_indptr"][r + 1])
            S = s["x_indices"][p0:p1]
            x_r = s["x_values"][p0:p1].reshape(1, -1).cpu().numpy() if p1 > p0 else np.zeros((1, 1), dtype=np.float32)
            Cs, factor = restricted("c", M, S)
            ref = float(oracle.knm_v(x_r, Cs, sigma, factor * vn).ravel()[0])
            for limit, (U, W) in results.items():
                got = float(W.reshape(n)[r])
                assert abs(got - ref) <= 1e-4 * abs(ref) + 1e-6, (r, limit, got, ref)
        print("row samples ok", flush=True)

        for j in (0, 17, M - 1):
            p0, p1 = int(s["c_indptr"][j]), int(s["c_indptr"][j + 1])
            S = s["c_indices"][p0:p1]
            c_j = s["c_values"][p0:p1].reshape(1, -1).cpu().numpy() if p1 > p0 else np.zeros((1, 1), dtype=np.float32)
            Xs, factor = restricted("x", n, S)
            for limit, (U, W) in results.items():
                Wn = W.reshape(n).cpu().numpy().astype(np.float64)  # the GPU's own W as the oracle's input
                ref = float(oracle.knm_t_y(Xs, c_j, sigma, factor * Wn).ravel()[0])
                got = float(U.reshape(M)[j])
                print(f"column {j}, head limit {limit}: relative error {abs(got - ref) / abs(ref):.2e}", flush=True)
                assert abs(got - ref) <= 1e-4 * abs(ref), (j, limit, got, ref)
        # the two formulations agree with each other over all outputs
        assert rel_l2(results[128][0].cpu().numpy(), results[0][0].cpu().numpy()) < 2e-5
        assert rel_l2(results[128][1].cpu().numpy(), results[0][1].cpu().numpy()) < 2e-5

    check(v, "mixed signs")
    # all terms of one sign: the all-pairs part of every output is orders of magnitude above a
    # single term of the sparse walk, the case in which accumulating the two together loses bits
    check(v.abs(), "positive vector")
