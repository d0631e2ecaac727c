"""Seeded synthetic inputs with the shapes and value distributions of the workloads.

This module only draws random numbers and labels; it holds none of the kernel method's
arithmetic.  Both the CPU oracle's tests and the GPU library's tests/benchmark take
their inputs from here, so both sides see identical fp32 bits.

Each workload stands in for a public dataset the paper measures on (HIGGS-, AIRLINE-,
image/multi-class-, TAXI- and TIMIT-shaped problems); nothing of those datasets is reproduced,
only (n, d, M, t), the value distributions and the hyper-parameters.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    d: int
    M: int
    t: int
    sigma: float
    lam: float
    iters: int
    seed: int
    stands_in_for: str


WORKLOADS = {
    "tiny": Workload("tiny", 20_000, 8, 1_000, 1, 2.0, 1e-6, 10, 1234, "small KRR sanity problem"),
    "mid": Workload("mid", 11_000_000, 28, 100_000, 1, 4.0, 1e-8, 20, 2, "HIGGS-shaped binary classification"),
    "lowdim": Workload("lowdim", 5_900_000, 8, 100_000, 1, 1.0, 1e-8, 20, 3, "AIRLINE-shaped regression"),
    "highdim": Workload("highdim", 2_000_000, 784, 50_000, 10, 24.0, 1e-9, 20, 4, "image-like multi-class"),
    "billion": Workload("billion", 1_000_000_000, 9, 100_000, 1, 1.0, 1e-10, 10, 5, "TAXI-shaped regression"),
    # not one of the five measured configurations: the paper's many-class shape and its settings (the
    # hyper-parameter table of the experimental appendix), for products and solves with many right-hand sides
    "manyclass": Workload("manyclass", 1_200_000, 440, 100_000, 144, 14.5, 5e-9, 5, 6, "TIMIT-shaped multi-class"),
}


def workload(name: str, n: Optional[int] = None, M: Optional[int] = None) -> Workload:
    """Look up a workload, optionally with fewer rows / centres (same distributions)."""
    w = WORKLOADS[name]
    if n is not None:
        w = replace(w, n=int(n))
    if M is not None:
        w = replace(w, M=int(M))
    return w


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


_CHUNK = 1 << 22  # rows generated at a time


def _rows(w: Workload, n: int, g: torch.Generator, device, out: torch.Tensor) -> None:
    """Fill out[n, d] (fp32) with the workload's feature distribution, chunk by chunk."""
    d = w.d
    step = max(1, min(_CHUNK, (1 << 27) // d))  # bound the temporaries of one chunk
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        m = hi - lo
        dst = out[lo:hi]
        if w.name in ("tiny", "mid", "manyclass"):
            dst.copy_(torch.randn(m, d, generator=g, device=device, dtype=torch.float32))
        elif w.name == "lowdim":
            # 4 columns uniform integers in [0, 24], 4 columns lognormal(3, 1); standardised
            # with the distributions' exact mean and standard deviation.
            ui = torch.randint(0, 25, (m, 4), generator=g, device=device).to(torch.float32)
            ln = torch.exp(3.0 + torch.randn(m, d - 4, generator=g, device=device, dtype=torch.float32))
            dst[:, :4] = (ui - 12.0) / math.sqrt((25.0 ** 2 - 1.0) / 12.0)
            mu = math.exp(3.5)
            sd = math.sqrt((math.e - 1.0) * math.exp(7.0))
            dst[:, 4:] = (ln - mu) / sd
        elif w.name == "billion":
            # 4 columns uniform(0, 1), 5 columns lognormal(2, 1); standardised as above.
            un = torch.rand(m, 4, generator=g, device=device, dtype=torch.float32)
            ln = torch.exp(2.0 + torch.randn(m, d - 4, generator=g, device=device, dtype=torch.float32))
            dst[:, :4] = (un - 0.5) / math.sqrt(1.0 / 12.0)
            mu = math.exp(2.5)
            sd = math.sqrt((math.e - 1.0) * math.exp(5.0))
            dst[:, 4:] = (ln - mu) / sd
        elif w.name == "highdim":
            mask = torch.rand(m, d, generator=g, device=device, dtype=torch.float32) < 0.2
            val = torch.rand(m, d, generator=g, device=device, dtype=torch.float32)
            dst.copy_(torch.where(mask, val, torch.zeros_like(val)))
        else:
            raise KeyError(w.name)


def _targets(w: Workload, X: torch.Tensor, g: torch.Generator, device) -> torch.Tensor:
    n, d = X.shape
    if w.name == "tiny":
        y = torch.sin(X.sum(dim=1)) + 0.1 * torch.randn(n, generator=g, device=device)
        return y.to(torch.float32).reshape(n, 1)
    if w.name == "mid":
        a = torch.randn(d, generator=g, device=device)
        Q = torch.randn(d, d, generator=g, device=device)
        Q = 0.5 * (Q + Q.T)
        y = torch.empty(n, device=device, dtype=torch.float32)
        flip = torch.empty(n, device=device, dtype=torch.bool)
        for lo in range(0, n, _CHUNK):
            hi = min(n, lo + _CHUNK)
            x = X[lo:hi]
            lin = (x @ a) / a.norm()
            quad = ((x @ Q) * x).sum(dim=1) - torch.trace(Q)
            quad = quad / (math.sqrt(2.0) * Q.norm())
            y[lo:hi] = torch.where(lin + quad >= 0, 1.0, -1.0)
            flip[lo:hi] = torch.rand(hi - lo, generator=g, device=device) < 0.1
        y = torch.where(flip, -y, y)
        return y.reshape(n, 1)
    if w.name in ("lowdim", "billion"):
        # log of a lognormal "duration": a smooth function of the features plus noise
        a = torch.randn(d, generator=g, device=device) / math.sqrt(d)
        y = torch.empty(n, device=device, dtype=torch.float32)
        for lo in range(0, n, _CHUNK):
            hi = min(n, lo + _CHUNK)
            x = X[lo:hi]
            y[lo:hi] = 0.5 * torch.tanh(x @ a) + 0.5 * torch.randn(hi - lo, generator=g, device=device)
        return y.reshape(n, 1)
    if w.name in ("highdim", "manyclass"):
        protos = torch.empty(w.t, d, device=device, dtype=torch.float32)
        _rows(w, w.t, g, device, protos)
        Y = torch.zeros(n, w.t, device=device, dtype=torch.float32)
        for lo in range(0, n, 1 << 18):
            hi = min(n, lo + (1 << 18))
            x = X[lo:hi]
            d2 = (x * x).sum(1, keepdim=True) - 2.0 * (x @ protos.T) + (protos * protos).sum(1)[None, :]
            Y[lo:hi].scatter_(1, d2.argmin(dim=1, keepdim=True), 1.0)
        return Y
    raise KeyError(w.name)


def make_inputs(w: Workload, device="cpu", with_targets: bool = True, n_test: int = 0) -> dict:
    """Generate X (n x d), Y (n x t), centres C (M x d: rows of X drawn uniformly without
    replacement) and, if asked, a fresh test set, all fp32 on `device`."""
    device = torch.device(device)
    g = _gen(device, w.seed)
    X = torch.empty(w.n, w.d, device=device, dtype=torch.float32)
    _rows(w, w.n, g, device, X)
    out = {"workload": w, "X": X}
    if w.M <= w.n:
        if w.n <= (1 << 24):
            idx = torch.randperm(w.n, generator=g, device=device)[: w.M]
        else:  # a full permutation of 1e9 rows is too large; draw, de-duplicate, trim
            idx = torch.unique(torch.randint(0, w.n, (int(w.M * 1.05) + 16,), generator=g, device=device))
            idx = idx[torch.randperm(idx.numel(), generator=g, device=device)][: w.M]
            assert idx.numel() == w.M
        out["centre_rows"] = idx
        out["C"] = X[idx].contiguous()
    else:
        raise ValueError("M must not exceed n")
    if with_targets:
        out["Y"] = _targets(w, X, g, device)
    if n_test:
        Xt = torch.empty(n_test, w.d, device=device, dtype=torch.float32)
        _rows(w, n_test, _gen(device, w.seed + 7919), device, Xt)
        out["Xtest"] = Xt
    return out


def probe_vector(M: int, t: int, kind: str = "normal", device="cpu", seed: int = 99, j: int = 0) -> torch.Tensor:
    """The vector v (M x t) a product is evaluated on: N(0,1), all ones, or e_j."""
    device = torch.device(device)
    if kind == "normal":
        return torch.randn(M, t, generator=_gen(device, seed), device=device, dtype=torch.float32)
    if kind == "ones":
        return torch.ones(M, t, device=device, dtype=torch.float32)
    if kind == "unit":
        v = torch.zeros(M, t, device=device, dtype=torch.float32)
        v[j % M, :] = 1.0
        return v
    raise KeyError(kind)


def sparse_inputs(n: int, M: int, d: int, nnz_per_row: float = 40.0, skew: float = 5.0, seed: int = 77,
                  device="cpu") -> dict:
    """Sparse rows shaped like n-gram count vectors (the paper's sparse text workload: about 1e6
    reviews over about 1e7 3-gram features): row lengths lognormal around `nnz_per_row`, feature
    ids with a heavy head (id = floor(d u^skew), u uniform: a few features occur in a large
    share of the rows, most in almost none), small integer counts as values, feature ids
    strictly increasing within a row.  The M centres are rows of X.
    Returns CSR pieces (int64 row pointers and feature ids, float32 values) for X and C."""
    device = torch.device(device)
    g = _gen(device, seed)
    lengths = torch.exp(math.log(nnz_per_row) + 0.5 * torch.randn(n, generator=g, device=device)).round().clamp(min=0)
    lengths = lengths.to(torch.int64)
    lengths[::97] = 0  # some empty rows
    draws = int(lengths.sum())
    u = torch.rand(draws, generator=g, device=device, dtype=torch.float64)
    col = (d * u.pow(skew)).to(torch.int64).clamp(max=d - 1)
    cnt = torch.randint(1, 4, (draws,), generator=g, device=device).to(torch.float32)
    row = torch.arange(n, device=device).repeat_interleave(lengths)
    # canonical CSR: a feature drawn several times in a row becomes one entry with the counts added
    key, inverse = torch.unique(row * d + col, sorted=True, return_inverse=True)
    val = torch.zeros(key.numel(), device=device, dtype=torch.float32).index_add_(0, inverse, cnt)
    row, col = key // d, key % d
    lengths = torch.bincount(row, minlength=n)
    crow = torch.zeros(n + 1, dtype=torch.int64, device=device)
    crow[1:] = torch.cumsum(lengths, 0)
    pick = torch.randperm(n, generator=g, device=device)[:M].sort().values
    len_c = lengths[pick]
    crow_c = torch.zeros(M + 1, dtype=torch.int64, device=device)
    crow_c[1:] = torch.cumsum(len_c, 0)
    nnz_c = int(crow_c[-1])
    src = crow[pick].repeat_interleave(len_c) + (torch.arange(nnz_c, device=device) - crow_c[:-1].repeat_interleave(len_c))
    return {"x_indptr": crow, "x_indices": col, "x_values": val, "c_indptr": crow_c, "c_indices": col[src],
            "c_values": val[src], "n": n, "M": M, "d": d, "centre_rows": pick}
