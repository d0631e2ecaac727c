#!/usr/bin/env python3
"""Benchmark of the hot path u = K_nm^T (K_nm v) on one MI355X.

A step is one full product (row sweep, column sweep, merge) on synthetic inputs that are
resident in HBM before the timed region.  Prints ONE JSON line with the whole-job
throughput in logical kernel entries per second (n * M per product, each entry counted
once although the two sweeps both evaluate it), the fp32-MFMA roofline fraction of the
tile kernel measured with HIP events on the library's stream, and the fp64 CPU oracle
timed on a bounded row sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix peak: 256 CU x 256 flop/clk x 2.4 GHz
PEAK_FP32_VALU_TFLOPS = 78.6   # fp32 vector peak without packed issue: 256 CU x 64 lanes x 2 flop x 2.4 GHz
PEAK_FP16_MFMA_TFLOPS = 2500.0  # MI355X dense fp16 matrix peak
PEAK_HBM_GBS = 8000.0  # MI355X HBM3E peak


def cpu_baseline(w, X_rows, C, v, budget_entries: float):
    """Time the oracle's knm_prod on `X_rows` (a strided row sample) x all centres."""
    import numpy as np

    import oracle

    Xn = X_rows.cpu().numpy()
    Cn = C.cpu().numpy()
    vn = v.cpu().numpy().astype(np.float64)
    t0 = time.perf_counter()
    oracle.knm_prod(Xn, Cn, w.sigma, vn)
    dt = time.perf_counter() - t0
    entries = Xn.shape[0] * Cn.shape[0]
    return {
        "value": entries / dt / 1e9,
        "unit": "G entries/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"{Xn.shape[0]} strided rows x all {Cn.shape[0]} centres, d={Xn.shape[1]}, t={vn.shape[1]}, "
                  f"fp64, {dt:.1f} s",
    }


def measured_traffic_bytes(workload: str):
    """HBM-side bytes per launch of the tile kernel, from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE, each scaled by its copy-probe factor); None if not profiled."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            t = json.load(f).get(workload)
        if not t:
            return None
        return 1024.0 * (t["fetch_kib_raw"] * t["fetch_scale"] + t["write_kib_raw"] * t["write_scale"])
    except (OSError, ValueError, KeyError):
        return None


def fit_benchmark(w, args) -> int:
    """falkon_fit end to end (preconditioner, right-hand side, CG iterations) with phase timings."""
    import torch

    import paper_2006_10350_amd as knm
    import synth

    inp = synth.make_inputs(w, device="cuda", with_targets=True)
    X, C, Y = inp["X"], inp["C"], inp["Y"]
    ctx = knm.default_context()
    ctx.set_cross_term(args.cross)
    iters = args.iters or w.iters
    if args.loss == "logistic":
        # Newton schedule: regularisers decreasing by 10x per step to the workload's lambda, then
        # repeated; `iters` CG iterations per step (the paper leaves the schedule to its reference)
        if w.t != 1:
            print("bench.py: the logistic loss needs a binary (t = 1) workload", file=sys.stderr)
            return 2
        y = torch.where(Y[:, 0] >= Y[:, 0].median(), 1.0, -1.0).contiguous()
        yC = y[inp["centre_rows"]].contiguous()
        steps = args.newton_steps
        lambdas = [max(w.lam, w.lam * 10.0 ** (steps - 2 - k)) for k in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        alpha, loss = knm.logfalkon_fit(X, y, C, yC, w.sigma, lambdas, [iters] * steps, args.jitter, return_loss=True,
                                        ctx=ctx)
        torch.cuda.synchronize()
        total = time.perf_counter() - t0
        print(json.dumps({
            "metric": "s per Newton step (logfalkon_fit)",
            "value": total / steps,
            "unit": "s",
            "higher_is_better": False,
            "n_gpus": 1,
            "config": {"workload": w.name, "n": w.n, "d": w.d, "M": w.M, "sigma": w.sigma, "lambdas": lambdas,
                       "cg_iters_per_step": iters, "newton_steps": steps, "jitter": args.jitter},
            "cross_term": args.cross,
            "fit_total_s": total,
            "mean_loss": [float(v) for v in loss],
            "alpha_finite": bool(torch.isfinite(alpha).all()),
        }))
        return 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    alpha, resid = knm.falkon_fit(X, Y, C, w.sigma, w.lam, iters, args.jitter, return_resid=True, ctx=ctx)
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    ft = ctx.get_fit_timing()
    print(json.dumps({
        "metric": "s per CG iteration (falkon_fit)",
        "value": ft["iterations_s"] / iters,
        "unit": "s",
        "higher_is_better": False,
        "n_gpus": 1,
        "config": {"workload": w.name, "n": w.n, "d": w.d, "M": w.M, "t": w.t, "sigma": w.sigma, "lambda": w.lam,
                   "iters": iters, "jitter": args.jitter},
        "cross_term": args.cross,
        "fit_total_s": total,
        "precond_s": ft["precond_s"],
        "rhs_s": ft["rhs_s"],
        "iterations_s": ft["iterations_s"],
        "residual_first_last": [float(resid.reshape(iters + 1, -1)[0].max()), float(resid.reshape(iters + 1, -1)[-1].max())],
        "alpha_finite": bool(torch.isfinite(alpha).all()),
    }))
    return 0


def sparse_benchmark(args) -> int:
    """K_nm^T (K_nm v) on sparse CSR inputs shaped like the paper's sparse text workload."""
    import torch

    import paper_2006_10350_amd as knm
    import synth

    n, M, d = args.n or 1_500_000, args.M or 50_000, 65_000_000
    sigma = 20.0
    s = synth.sparse_inputs(n, M, d, nnz_per_row=100.0, skew=args.sparse_skew, seed=6, device="cuda")
    X = torch.sparse_csr_tensor(s["x_indptr"], s["x_indices"], s["x_values"], size=(n, d), check_invariants=False)
    C = torch.sparse_csr_tensor(s["c_indptr"], s["c_indices"], s["c_values"], size=(M, d), check_invariants=False)
    if args.fit:
        # falkon_fit_csr end to end: labels from a sparse linear score, squashed
        iters = args.iters or 10
        g = torch.Generator(device="cuda").manual_seed(7)
        wtrue = torch.randn(d, device="cuda", generator=g)
        rows = torch.repeat_interleave(torch.arange(n, device="cuda"), torch.diff(s["x_indptr"]))
        score = torch.zeros(n, device="cuda").index_add_(0, rows, s["x_values"] * wtrue[s["x_indices"]])
        Y = torch.tanh(0.05 * score).reshape(n, 1).contiguous()
        del wtrue, rows, score
        ctx = knm.default_context()
        lam = 1e-6
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        alpha, resid = knm.falkon_fit_csr(X, Y, C, sigma, lam, iters, args.jitter, return_resid=True, ctx=ctx)
        torch.cuda.synchronize()
        total = time.perf_counter() - t0
        ft = ctx.get_fit_timing()
        print(json.dumps({
            "metric": "s per CG iteration (falkon_fit_csr)", "value": ft["iterations_s"] / iters, "unit": "s",
            "higher_is_better": False, "n_gpus": 1,
            "config": {"workload": "sparse-text-like", "n": n, "d": d, "M": M, "t": 1, "sigma": sigma, "lambda": lam,
                       "iters": iters, "jitter": args.jitter, "feature_skew": args.sparse_skew,
                       "nnz_x": int(s["x_indptr"][-1]), "nnz_c": int(s["c_indptr"][-1])},
            "fit_total_s": total, "precond_s": ft["precond_s"], "rhs_s": ft["rhs_s"], "iterations_s": ft["iterations_s"],
            "residual_first_last": [float(resid[0].max()), float(resid[-1].max())],
            "alpha_finite": bool(torch.isfinite(alpha).all()),
        }))
        return 0
    v = synth.probe_vector(M, 1, "normal", device="cuda")
    # work of one sweep: for every stored entry of X, the centres that have its feature
    counts = torch.bincount(s["c_indices"])
    lens = torch.zeros(d, dtype=torch.int64, device="cuda")
    lens[: counts.numel()] = counts
    pairs = int(lens[s["x_indices"]].sum())
    del lens
    for _ in range(args.warmup):
        knm.knm_prod_csr(X, C, sigma, v)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        U = knm.knm_prod_csr(X, C, sigma, v)
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t0) / args.steps
    nnz_x = int(s["x_indptr"][-1])
    # algorithmic bytes of the two sweeps: per visited (entry of X, centre) pair and pass one list entry
    # (8 B) and one accumulator update (4 B read + 4 B written); per entry of X and pass its id, value and
    # two list pointers (20 B)
    bytes_per_product = 2 * 2 * (16.0 * pairs + 20.0 * nnz_x)
    print(json.dumps({
        "metric": "G kernel-entries/s in K_nm^T(K_nm v), sparse CSR inputs",
        "value": n * M / elapsed / 1e9, "unit": "G entries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "sparse-text-like", "n": n, "d": d, "M": M, "t": 1, "sigma": sigma,
                   "nnz_x": nnz_x, "nnz_c": int(s["c_indptr"][-1]), "feature_skew": args.sparse_skew,
                   "stands_in_for": "YELP-shaped sparse n-gram counts"},
        "pair_updates_per_sweep": pairs, "pair_updates_per_s": 2 * 2 * pairs / elapsed,
        "roofline": {"bound": "hbm", "kernel": "sparse_sweep_kernel", "achieved": bytes_per_product / elapsed / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": bytes_per_product / elapsed / 1e9 / PEAK_HBM_GBS,
                     "traffic": None,
                     "note": "bytes of the all-sparse walk (every pair that shares a feature); the most frequent features' "
                             "pairs are in fact covered by one dense product, the rest by scattered 4-byte atomics bound by "
                             "L2 atomic latency, far from the HBM roofline"},
        "u_finite": bool(torch.isfinite(U).all()),
    }))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="mid", help="tiny | mid | lowdim | highdim | billion")
    ap.add_argument("--n", type=int, default=None, help="override the number of rows (same distribution)")
    ap.add_argument("--M", type=int, default=None, help="override the number of centres")
    ap.add_argument("--cpu-rows", type=int, default=None, help="rows of the oracle's timing sample")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cross", default="f16x3", choices=["f32", "f16x3"],
                    help="arithmetic of the cross term (d <= 44, t = 1): three split-fp16 MFMA products (library "
                         "default) or fp32 MFMA")
    ap.add_argument("--kernel", default="gaussian", choices=["gaussian", "laplacian", "matern32", "matern52"],
                    help="kernel function of the product (the headline metric is quoted on the Gaussian one)")
    ap.add_argument("--fit", action="store_true",
                    help="instead of the product benchmark, run falkon_fit end to end on the workload and "
                         "report seconds per conjugate-gradient iteration")
    ap.add_argument("--iters", type=int, default=None, help="CG iterations for --fit (default: the workload's)")
    ap.add_argument("--loss", default="squared", choices=["squared", "logistic"],
                    help="--fit: squared loss (falkon_fit) or logistic loss (logfalkon_fit, labels = sign of the "
                         "targets about their median)")
    ap.add_argument("--newton-steps", type=int, default=4, help="Newton steps for --fit --loss logistic")
    ap.add_argument("--jitter", type=float, default=1e-8, help="diagonal jitter on K_MM for --fit")
    ap.add_argument("--no-fp32-leg", action="store_true",
                    help="skip the extra (untimed-region) product in the fp32-MFMA cross-term mode")
    ap.add_argument("--sparse", action="store_true",
                    help="instead of a dense workload, time knm_prod_csr on synthetic sparse rows (n = 1.5M, "
                         "d = 6.5e7, M = 50k, about 100 stored features per row)")
    ap.add_argument("--sparse-skew", type=float, default=2.5,
                    help="--sparse: feature id = floor(d u^skew); 2.5 puts the commonest feature in about 10 %% of the rows")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a dispatch of known "
                         "traffic that calibrates the HBM byte counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (rows of X would be sharded across GPUs with one "
              "all-reduce of the M x t result per product; not built). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2006_10350_amd as knm
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.sparse:
        return sparse_benchmark(args)
    w = synth.workload(args.workload, n=args.n, M=args.M)
    if args.fit:
        return fit_benchmark(w, args)
    inp = synth.make_inputs(w, device="cuda", with_targets=False)
    X, C = inp["X"], inp["C"]
    v = synth.probe_vector(w.M, w.t, "normal", device="cuda")
    U = torch.empty(w.M, w.t, device="cuda", dtype=torch.float32)
    ctx = knm.default_context()
    ctx.set_cross_term(args.cross)
    ctx.set_kernel(args.kernel)
    torch.cuda.synchronize()
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib * (1 << 18), device="cuda", dtype=torch.float32)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
    torch.cuda.synchronize()

    ctx.set_timing(True)
    row_ms, col_ms, merge_ms = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
        tm = ctx.get_timing()  # HIP events on the library's stream; waits for this step
        row_ms.append(tm["row_sweep_ms"])
        col_ms.append(tm["col_sweep_ms"])
        merge_ms.append(tm["merge_ms"])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ctx.set_timing(False)

    ms_per_step = 1e3 * elapsed / args.steps
    entries = float(w.n) * float(w.M)
    value = entries / (elapsed / args.steps) / 1e9

    # Which tile engine ran (same rule as the library): the K-loop engine for t > 1 (up to 16 columns
    # per launch) or d beyond the register-resident engine's limit (44 features with the split-fp16
    # cross term, the default; 64 with fp32 MFMA); otherwise the register-resident engine.  Two sweeps
    # per step.
    # The kernels of the distance (Laplacian, Matern) always run on the K-loop engine.
    k_loop = args.kernel != "gaussian" or w.t > 1 or w.d > (44 if args.cross == "f16x3" else 64)
    f16 = (not k_loop) and args.cross == "f16x3" and w.d <= 44
    k_loop_f16 = k_loop and args.cross == "f16x3"
    kernel_name = (("gauss_gemm_f16_kernel" if k_loop_f16 else "gauss_gemm_kernel") if k_loop
                   else ("gauss_sweep_f16_kernel" if f16 else "gauss_sweep_kernel"))
    launches = 2 * ((w.t + 15) // 16) * args.steps
    avg_launch_ms = (sum(row_ms) + sum(col_ms)) / launches
    # algorithmic contraction work: one evaluation of every entry, 2 d flop each
    flop_per_launch = entries * 2.0 * w.d
    if f16:
        # Bound by the vector ALU, not the matrix cores: per entry one v_exp_f32 (half rate: two issue
        # slots) and one FMA (one slot) = 3 lane-slots = 6 flop-equivalents at 2 flop per slot, against
        # the un-packed fp32 vector peak 256 CU x 64 lanes x 2 flop x 2.4 GHz = 78.6 TFLOP/s.
        alu_per_launch = entries * 6.0
        achieved = alu_per_launch / (avg_launch_ms * 1e-3) / 1e12
        bound, peak, work = "alu", PEAK_FP32_VALU_TFLOPS, alu_per_launch
    elif k_loop_f16:
        # Dense contraction on the f16 matrix cores: the split-fp16 cross term is three f16 products per
        # feature pair (fh.xh + fh.xl + fl.xh), 6 d flop per entry, against the dense fp16 MFMA peak.
        f16_flop = 3.0 * flop_per_launch
        achieved = f16_flop / (avg_launch_ms * 1e-3) / 1e12
        bound, peak, work = "mfma", PEAK_FP16_MFMA_TFLOPS, f16_flop
    else:
        achieved = flop_per_launch / (avg_launch_ms * 1e-3) / 1e12
        bound, peak, work = "mfma", PEAK_FP32_MFMA_TFLOPS, flop_per_launch
    roofline = {
        "bound": bound,
        "kernel": kernel_name,
        "achieved": achieved,
        "peak": peak,
        "unit": "TFLOP/s",
        "frac": achieved / peak,
        "traffic": measured_traffic_bytes(w.name + ("" if f16 or k_loop_f16 else "_f32"))
        if (args.n is None and args.M is None and args.kernel == "gaussian") else None,
        "avg_launch_ms": avg_launch_ms,
        "row_sweep_ms": sum(row_ms) / len(row_ms),
        "col_sweep_ms": sum(col_ms) / len(col_ms),
        "merge_ms": sum(merge_ms) / len(merge_ms),
        "work_per_launch": work,
        "contraction_flop_per_launch": flop_per_launch,
        # the same launch priced as if its 2 d flop per entry had run on fp32 MFMA
        "fp32_mfma_equiv_frac": flop_per_launch / (avg_launch_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
    }

    fp32_mode = None
    if (f16 or k_loop_f16) and not args.no_fp32_leg:
        # the fp32-MFMA cross-term mode on the same inputs, outside the timed region
        ctx.set_cross_term("f32")
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
        ctx.set_timing(True)
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
        tm = ctx.get_timing()
        ctx.set_timing(False)
        ctx.set_cross_term(args.cross)
        l_ms = 0.5 * (tm["row_sweep_ms"] + tm["col_sweep_ms"])
        fp32_mode = {"kernel": "gauss_gemm_kernel" if k_loop else "gauss_sweep_kernel", "ms_per_product": tm["total_ms"], "avg_launch_ms": l_ms,
                     "frac_of_fp32_mfma_peak": flop_per_launch / (l_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}

    out = {
        "metric": "G kernel-entries/s in K_nm^T(K_nm v)",
        "value": value,
        "unit": "G entries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "d": w.d, "M": w.M, "t": w.t, "sigma": w.sigma,
                   "kernel": args.kernel, "stands_in_for": w.stands_in_for},
        "s_per_product": ms_per_step / 1e3,
        "mfma_frac_two_sweeps": 2.0 * entries * 2.0 * w.d / (elapsed / args.steps) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "cross_term": "f16x3" if (f16 or k_loop_f16) else "f32",
        "roofline": roofline,
    }
    if fp32_mode is not None:
        out["fp32_mfma_mode"] = fp32_mode

    if not args.no_cpu:
        # bounded sample: about 10-30 s of oracle work on the host cores
        rows = args.cpu_rows or max(64, int(3.2e11 / (w.M * (w.d + 30.0))))
        rows = min(rows, w.n)
        stride = max(1, w.n // rows)
        idx = torch.arange(0, rows, device="cuda") * stride
        import oracle

        with oracle.kernel(args.kernel):
            out["cpu_baseline"] = cpu_baseline(w, X[idx], C, v, 0.0)
    ctx.set_kernel("gaussian")
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
