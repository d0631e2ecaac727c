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
    print(json.dumps({
        "metric": "G kernel-entries/s in K_nm^T(K_nm v), sparse CSR inputs",
        "value": n * M / elapsed / 1e9, "unit": "G entries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "sparse-text-like", "n": n, "d": d, "M": M, "t": 1, "sigma": sigma,
                   "nnz_x": nnz_x, "nnz_c": int(s["c_indptr"][-1]), "feature_skew": args.sparse_skew,
                   "stands_in_for": "YELP-shaped sparse n-gram counts"},
        "pair_updates_per_sweep": pairs, "pair_updates_per_s": 2 * 2 * pairs / elapsed,
        # the walk is bound by scattered 4-byte L2 atomics on the per-wavefront accumulators; there is no
        # published peak for those, so the rate is stated without a fraction
        "roofline": {"bound": "l2-atomics", "kernel": "sparse_sweep_kernel", "achieved": 2 * 2 * pairs / elapsed / 1e9,
                     "peak": None, "unit": "G pair updates/s", "frac": None, "traffic": None},
        "u_finite": bool(torch.isfinite(U).all()),
    }))
    return 0


def counters(workload: str):
    """Per-launch counters of the tile kernel from the committed rocprofv3 --pmc summaries
    (profiles/hbm_traffic.json): HBM-side bytes (FETCH_SIZE and WRITE_SIZE, each scaled by its
    copy-probe factor) and issued matrix-core instructions; None where not profiled."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            t = json.load(f).get(workload)
    except (OSError, ValueError):
        t = None
    if not t:
        return None, None
    traffic = None
    if "fetch_kib_raw" in t:
        traffic = 1024.0 * (t["fetch_kib_raw"] * t["fetch_scale"] + t["write_kib_raw"] * t["write_scale"])
    return traffic, t.get("mfma_insts_per_launch")


def engine_of(w, cross: str, kernel: str):
    """Which tile engine the library runs for this shape (same rule as the library): the K-loop engine
    for t > 1 or for d beyond the register-resident engine's limit (44 features with the split-fp16
    cross term, the default, 28 for the kernels of the distance; 64 with fp32 MFMA, Gaussian only)."""
    k_loop = w.t > 1 or w.d > (44 if cross == "f16x3" else 64) or (kernel != "gaussian" and (cross != "f16x3" or w.d > 28))
    f16 = cross == "f16x3"
    name = (("gauss_gemm_f16_kernel" if f16 else "gauss_gemm_kernel") if k_loop
            else ("gauss_sweep_f16_kernel" if f16 else "gauss_sweep_kernel"))
    return name, k_loop, f16


def product_leg(knm, synth, torch, ctx, w, steps: int, warmup: int, cross: str, kernel: str, inputs=None, probe=None):
    """Times `steps` full products K_nm^T (K_nm v) on workload w; returns the metrics of the leg."""
    inp = inputs or synth.make_inputs(w, device="cuda", with_targets=False)
    X, C = inp["X"], inp["C"]
    v = synth.probe_vector(w.M, w.t, "normal", device="cuda")
    U = torch.empty(w.M, w.t, device="cuda", dtype=torch.float32)
    ctx.set_cross_term(cross)
    ctx.set_kernel(kernel)
    for _ in range(warmup):
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
    torch.cuda.synchronize()
    ctx.set_timing(True)
    row_ms, col_ms, merge_ms = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
        tm = ctx.get_timing()  # HIP events on the library's stream; waits for this step
        row_ms.append(tm["row_sweep_ms"])
        col_ms.append(tm["col_sweep_ms"])
        merge_ms.append(tm["merge_ms"])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ctx.set_timing(False)

    s_per_product = elapsed / steps
    entries = float(w.n) * float(w.M)
    kernel_name, k_loop, f16 = engine_of(w, cross, kernel)
    # columns per launch of the K-loop engines (split-fp16: with its packed vector image)
    group = (160 if kernel == "gaussian" else 128) if (k_loop and f16) else 16
    launches = 2 * ((w.t + group - 1) // group if k_loop else 1) * steps
    avg_launch_ms = (sum(row_ms) + sum(col_ms)) / launches
    # Algorithmic contraction work of one launch (one sweep): every kernel entry once, 2 d flop each.
    # Padded or augmented contraction slots, the 2 t reduction flop and the exp are not counted.
    flop_per_launch = entries * 2.0 * w.d
    tflops = flop_per_launch / (avg_launch_ms * 1e-3) / 1e12
    default = kernel == "gaussian"
    traffic, mfma_insts = counters(w.name + ("" if f16 else "_f32")) if default else (None, None)
    roofline = {
        "bound": "mfma",
        "kernel": kernel_name,
        # the contraction's own dtype: f16 matrix cores (three split products per feature pair,
        # fp32 accumulate) in the default mode, fp32 matrix cores otherwise
        "contraction_dtype": "f16" if f16 else "f32",
        "achieved": tflops,
        "peak": PEAK_FP16_MFMA_TFLOPS if f16 else PEAK_FP32_MFMA_TFLOPS,
        "unit": "TFLOP/s",
        "frac": tflops / (PEAK_FP16_MFMA_TFLOPS if f16 else PEAK_FP32_MFMA_TFLOPS),
        "traffic": traffic,
        "avg_launch_ms": avg_launch_ms,
        "row_sweep_ms": sum(row_ms) / len(row_ms),
        "col_sweep_ms": sum(col_ms) / len(col_ms),
        "merge_ms": sum(merge_ms) / len(merge_ms),
        "flop_per_launch": flop_per_launch,
        # the same launch priced against the fp32 matrix peak (what the 2 d flop per entry would cost there)
        "fp32_mfma_equiv_frac": tflops / PEAK_FP32_MFMA_TFLOPS,
    }
    if f16:
        # counting the three split products that fp32-class accuracy costs in that dtype
        roofline["frac_split_x3"] = 3.0 * roofline["frac"]
        if mfma_insts:
            # issued: matrix-core instructions per launch from the committed SQ_INSTS_MFMA count
            # (32 x 32 x 16 x 2 flop each; includes padding of d and the norm slots)
            roofline["frac_issued"] = mfma_insts * 32768.0 / (avg_launch_ms * 1e-3) / 1e12 / PEAK_FP16_MFMA_TFLOPS
        if not k_loop and probe:
            # The register-resident engine at small d is bound by the vector ALU's exp + FMA per entry
            # together with the matrix cores they share issue with, not by the matrix cores alone: the
            # engine's clocks per pair of 32 x 32 tiles against the same instruction mix run from
            # registers only (measured now, on this device: both pipes, and each pipe alone).
            hu = 1 if w.d <= 12 else (2 if w.d <= 28 else 3)
            per_pair = avg_launch_ms * 1e-3 * 2.4e9 / (entries / 2048.0 / (256 * 4))  # per SIMD
            roofline["alu"] = {
                "nominal_clk_per_tile_pair": per_pair,
                "probe_mix_clk_per_tile_pair": {k: probe[f"mix{hu}_{k}_clk"] for k in ("both", "valu", "mfma")},
                "frac_of_probe_mix": probe[f"mix{hu}_both_clk"] / per_pair,
            }
    return {
        "workload": w.name, "n": w.n, "d": w.d, "M": w.M, "t": w.t, "sigma": w.sigma, "kernel": kernel,
        "steps": steps, "warmup": warmup,
        "s_per_product": s_per_product,
        "g_entries_per_s": entries / s_per_product / 1e9,
        "g_entry_evaluations_per_s": 2.0 * entries / s_per_product / 1e9,
        "cross_term": "f16x3" if f16 else "f32",
        # fractions of the fp32 matrix peak: the method's two evaluations of every entry, and one
        "fp32_mfma_frac_two_sweeps": 2.0 * entries * 2.0 * w.d / s_per_product / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "fp32_mfma_frac_single_eval": entries * 2.0 * w.d / s_per_product / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "roofline": roofline,
        "_tensors": (X, C, v, U),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="mid", help="tiny | mid | lowdim | highdim | billion | manyclass")
    ap.add_argument("--n", type=int, default=None, help="override the number of rows (same distribution)")
    ap.add_argument("--M", type=int, default=None, help="override the number of centres")
    ap.add_argument("--cpu-rows", type=int, default=None, help="rows of the oracle's timing sample")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cross", default="f16x3", choices=["f32", "f16x3"],
                    help="arithmetic of the cross term: three split-fp16 MFMA products (library default) or fp32 MFMA")
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
    ap.add_argument("--jitter", type=float, default=1e-8, help="diagonal jitter on K_MM for the fits")
    ap.add_argument("--no-fp32-leg", action="store_true",
                    help="skip the extra (untimed-region) product in the fp32-MFMA cross-term mode")
    ap.add_argument("--no-cg-leg", action="store_true",
                    help="skip the short falkon_fit (preconditioner + 4 CG iterations) that measures s per CG iteration")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short product legs on the other workloads (lowdim, highdim, billion)")
    ap.add_argument("--no-probe", action="store_true", help="skip the instruction-rate probe")
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
    ctx = knm.default_context()
    full_size = args.n is None and args.M is None
    headline = full_size and args.workload == "mid" and args.kernel == "gaussian" and args.cross == "f16x3"
    probe = None if args.no_probe else ctx.probe_rates()
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib * (1 << 18), device="cuda", dtype=torch.float32)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    inp = synth.make_inputs(w, device="cuda", with_targets=headline and not args.no_cg_leg)
    leg = product_leg(knm, synth, torch, ctx, w, args.steps, args.warmup, args.cross, args.kernel, inputs=inp, probe=probe)
    X, C, v, U = leg.pop("_tensors")
    if not full_size:
        leg["roofline"]["traffic"] = None
    f16 = leg["cross_term"] == "f16x3"

    fp32_mode = None
    if f16 and not args.no_fp32_leg:
        # the fp32-MFMA cross-term mode on the same inputs, outside the timed region
        ctx.set_cross_term("f32")
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
        ctx.set_timing(True)
        knm.knm_prod(X, C, w.sigma, v, out=U, ctx=ctx)
        tm = ctx.get_timing()
        ctx.set_timing(False)
        ctx.set_cross_term(args.cross)
        launches = 2 * ((w.t + 15) // 16 if engine_of(w, "f32", args.kernel)[1] else 1)
        l_ms = (tm["row_sweep_ms"] + tm["col_sweep_ms"]) / launches
        fp32_mode = {"kernel": engine_of(w, "f32", args.kernel)[0], "ms_per_product": tm["total_ms"], "avg_launch_ms": l_ms,
                     "frac_of_fp32_mfma_peak": leg["roofline"]["flop_per_launch"] / (l_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}

    out = {
        "metric": "G kernel-entries/s in K_nm^T(K_nm v) + % fp32 MFMA peak; s per CG iteration",
        "value": leg["g_entries_per_s"],
        "unit": "G entries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * leg["s_per_product"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # fp32 inputs, outputs and accumulation throughout; the contraction over d runs as three
        # split-fp16 products on the f16 matrix cores (library default) or on the fp32 matrix cores
        "dtype": "f32 data, f16x3 cross term" if f16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "d": w.d, "M": w.M, "t": w.t, "sigma": w.sigma,
                   "kernel": args.kernel, "stands_in_for": w.stands_in_for},
        "s_per_product": leg["s_per_product"],
        "g_entry_evaluations_per_s": leg["g_entry_evaluations_per_s"],
        "fp32_mfma_frac_two_sweeps": leg["fp32_mfma_frac_two_sweeps"],
        "fp32_mfma_frac_single_eval": leg["fp32_mfma_frac_single_eval"],
        "cross_term": leg["cross_term"],
        "roofline": leg["roofline"],
    }
    if fp32_mode is not None:
        out["fp32_mfma_mode"] = fp32_mode
    if probe is not None:
        out["probe"] = probe

    if headline and not args.no_cg_leg:
        # The third part of the metric: the preconditioner is built (outside any timed product), then
        # a few iterations of preconditioned CG run inside falkon_fit; s per CG iteration = product +
        # 4 fp64 triangular solves + vector updates, host clock around iterations that each end with a
        # synchronising dot product.
        iters = 4
        torch.cuda.synchronize()
        alpha, resid = knm.falkon_fit(X, inp["Y"], C, w.sigma, w.lam, iters, args.jitter, return_resid=True, ctx=ctx)
        torch.cuda.synchronize()
        ft = ctx.get_fit_timing()
        out["s_per_cg_iter"] = ft["iterations_s"] / iters
        out["precond_s"] = ft["precond_s"]
        out["cg_leg"] = {"iters": iters, "rhs_s": ft["rhs_s"], "iterations_s": ft["iterations_s"], "lambda": w.lam,
                         "jitter": args.jitter, "alpha_finite": bool(torch.isfinite(alpha).all()),
                         "residual_first_last": [float(resid.reshape(iters + 1, -1)[0].max()),
                                                 float(resid.reshape(iters + 1, -1)[-1].max())]}
        del alpha

    if not args.no_cpu:
        # bounded sample: about 10-30 s of oracle work on the host cores
        rows = args.cpu_rows or max(64, int(3.2e11 / (w.M * (w.d + 30.0))))
        rows = min(rows, w.n)
        stride = max(1, w.n // rows)
        idx = torch.arange(0, rows, device="cuda") * stride
        import oracle

        with oracle.kernel(args.kernel):
            out["cpu_baseline"] = cpu_baseline(w, X[idx], C, v, 0.0)

    if headline and not args.no_others:
        # Short legs on the other workloads (not part of `value`): one line each with the same fields.
        del X, C, v, U, inp
        torch.cuda.empty_cache()
        others = {}
        for name, steps, warmup in (("lowdim", 5, 1), ("highdim", 3, 1), ("billion", 1, 0)):
            wo = synth.workload(name)
            # the many-output workload also gets a short fit: its CG iteration carries 10 right-hand sides
            # through the solves (the others' preconditioners and solves are those of the headline leg)
            fit_too = name == "highdim" and not args.no_cg_leg
            io = synth.make_inputs(wo, device="cuda", with_targets=True) if fit_too else None
            lo = product_leg(knm, synth, torch, ctx, wo, steps, warmup, args.cross, args.kernel, inputs=io, probe=probe)
            lo.pop("_tensors")
            if fit_too:
                iters = 2
                alpha = knm.falkon_fit(io["X"], io["Y"], io["C"], wo.sigma, wo.lam, iters, args.jitter, ctx=ctx)
                torch.cuda.synchronize()
                ft = ctx.get_fit_timing()
                lo["s_per_cg_iter"] = ft["iterations_s"] / iters
                lo["precond_s"] = ft["precond_s"]
                lo["cg_leg"] = {"iters": iters, "rhs_s": ft["rhs_s"], "lambda": wo.lam, "jitter": args.jitter,
                                "alpha_finite": bool(torch.isfinite(alpha).all())}
                del alpha
            del io
            others[name] = lo
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    ctx.set_kernel("gaussian")
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
