#!/usr/bin/env python3
"""Benchmark of the BBMM hot path on one MI355X.

One "step" is one full bbmm_solve_logdet_grad call (preconditioner, probes, mBCG, SLQ
log-det, derivative traces) on the n = 50,000, d = 16, t = 10 Matern-5/2 ARD workload
(rank-20 preconditioner, 50 mBCG iterations), inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--mode sym|mat|otf|sgpr] [--config 3|2|4] [--n N] [--no-cpu]

The default mode keeps the fp32 K_hat materialised as its upper triangle (half the HBM bytes per
product, every tile used for both of its contributions; the product is then bound by the fp64
matrix rate).  --mode mat keeps the whole matrix (HBM-bound product), --mode otf rebuilds the tiles
from X in every product.  --mode sgpr measures the widened path instead (config 5: subset-of-regressors covariance,
n = 500,000, m = 1024 inducing inputs, d = 8, t = 10, rank-10 preconditioner, 50 iterations);
the default line is the exact-GP workload above.  --config 2 runs the second roofline point instead
(RBF, n = 10,000, d = 8, rank-10 preconditioner, stop at a relative residual of 1e-2 or 50 iterations),
--config 4 the largest exact-GP workload (RBF on 20 Gaussian clusters, n = 200,000, d = 8, t = 16, rank-20
preconditioner, 100 iterations; on the fly unless --mode says otherwise).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix, published
MFMA_F64_PEAK_TFLOPS = 78.6    # MI355X dense fp64 matrix, published
FP64_VALU_PEAK_TFLOPS = 78.6   # MI355X fp64 vector, published
# HBM bytes per k_mm_mat launch at n = 50000 from rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by a
# 1 GiB copy (profiles/k_mm_mat_cfg3_n50000_hbm_counters.txt); only valid for that workload.
MEASURED_TRAFFIC_MAT_N50000 = 10.141e9
# HBM bytes per SGPR product (both k_mm_mat launches) at n = 500000, m = 1024, measured the same way
# (profiles/k_mm_mat_cfg5_n500000_sgpr_hbm_counters.txt); only valid for that workload.
MEASURED_TRAFFIC_SGPR_N500000_M1024 = 4.261e9
# HBM bytes per product from the upper triangle at n = 50000 (both launches), measured the same way
# (profiles/k_mm_sym_cfg3_n50000_counters.txt); only valid for that workload.
MEASURED_TRAFFIC_SYM_N50000 = 5.527e9


def _cores():
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    return min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))


def cpu_baseline_full_n(cfg: int, n: int, iters: int, rows_build: int = 2048, rows_mm: int = 8192):
    """The fp64 oracle timed ON the benchmark workload, piece by piece at full width n: every O(n^2)
    stage of oracle.bbmm_inference is linear in the number of matrix ROWS it handles, so each is timed
    on a block of rows of the full n-column problem and scaled by n / rows (no scaling in n itself):
      build      kernel_block(X[rows_build], X)                -> K_hat, once per call
      product    K_hat[rows_mm] @ D (n x c), fp64              -> one per mBCG iteration
      derivative kernel_derivative_blocks(X[rows_build], X) and its products with [W, u_0], once per call
    plus the O(n k^2 + n c) vector work of `iters` iterations measured directly on n x c blocks.
    Returns (milliseconds for one call of `iters` iterations, description, seconds of CPU time used)."""
    from oracle import bbmm_oracle as O
    from paper_1809_11165_amd import inputs
    w = inputs.make(cfg, n=n)
    X64 = w.X.astype(np.float64)
    c, t = w.t + 1, w.t
    rng = np.random.default_rng(0)
    t_all = time.perf_counter()
    rb = min(rows_build, n)
    t0 = time.perf_counter()
    Kb = O.kernel_block(w.kernel, X64[:rb], X64, w.lengthscale, w.outputscale)
    t_build = (time.perf_counter() - t0) * n / rb
    rm = min(rows_mm, n)
    slab = np.ascontiguousarray(np.tile(Kb, (-(-rm // rb), 1))[:rm])      # rows_mm x n fp64, values do not matter
    D = rng.standard_normal((n, c))
    slab @ D                                                                # warm the BLAS threads
    t0 = time.perf_counter()
    for _ in range(3):
        slab @ D
    t_mm = (time.perf_counter() - t0) / 3 * n / rm
    del slab
    U, W = rng.standard_normal((n, c)), rng.standard_normal((n, t))
    t0 = time.perf_counter()
    mats = O.kernel_derivative_blocks(w.kernel, X64[:rb], X64, w.lengthscale, w.outputscale)
    for M in mats:
        float(np.sum(U[:rb, 1:] * (M @ W)) / t)
        float(U[:rb, 0] @ (M @ U[:, 0]))
    t_dk = (time.perf_counter() - t0) * n / rb
    del mats, Kb
    # per-iteration vector work: the preconditioner solve and the updates of Alg. 2 on n x c blocks
    L = rng.standard_normal((n, w.k))
    P = O.make_preconditioner(L, w.noise)
    R = rng.standard_normal((n, c))
    t0 = time.perf_counter()
    for _ in range(3):
        Z = P.solve(R)
        np.sum(R * Z, axis=0)
        U2 = U + D * 0.5
        R2 = R - D * 0.5
        np.sum(D * R, axis=0)
        D2 = Z + D * 0.3
    t_vec = (time.perf_counter() - t0) / 3
    total = t_build + iters * (t_mm + t_vec) + t_dk
    used = time.perf_counter() - t_all
    desc = ("fp64 numpy oracle at full n=%d, timed by stage on blocks of rows of the full-width problem and scaled "
            "by n/rows only: K_hat build %.1f s (from %d rows), %d x (product %.3f s from %d rows + vector "
            "updates %.3f s), derivative pass %.1f s (from %d rows); %.0f s of CPU time used"
            % (n, t_build, rb, iters, t_mm, rm, t_vec, t_dk, rb, used))
    return total * 1e3, desc, {"build_s": t_build, "product_s_per_iteration": t_mm,
                               "vector_s_per_iteration": t_vec, "derivative_s": t_dk}


def cpu_baseline(cfg: int, n_sample: int, n_full: int, iters: int):
    """Times the fp64 oracle (as it stands) on an n_sample-point instance of the same recipe, for the
    number of iterations the GPU call ran, and scales by (n_full / n_sample)^2, the cost ratio of the
    O(n^2) products that dominate."""
    from oracle import bbmm_oracle as O
    from paper_1809_11165_amd import inputs
    w = inputs.make(cfg, n=n_sample)
    t0 = time.perf_counter()
    O.bbmm_inference(w.kernel, w.X, w.y, w.lengthscale, w.outputscale, w.noise, w.E1, w.E2,
                     w.k, iters)
    dt = time.perf_counter() - t0
    small = {"value": dt * 1e3 * (n_full / n_sample) ** 2, "unit": "ms", "cores": _cores(),
             "kind": "oracle",
             "sample": "fp64 numpy oracle, full call (k=%d, t=%d, %d iterations) on n=%d points of the same "
                       "recipe: %.1f s measured, scaled by (n/n_sample)^2 = %.0f"
                       % (w.k, w.t, iters, n_sample, dt, (n_full / n_sample) ** 2)}
    if n_sample >= n_full:
        return small
    # the headline figure: the oracle's stages timed at the benchmark's own n; the small-n
    # extrapolation is kept beside it for comparison
    ms, desc, parts = cpu_baseline_full_n(cfg, n_full, iters)
    return {"value": ms, "unit": "ms", "cores": _cores(), "kind": "oracle", "sample": desc, "stages": parts,
            "extrapolated_from_small_n": {"value": small["value"], "unit": "ms", "sample": small["sample"]}}


def cpu_baseline_sgpr(n_sample: int, n_full: int, m: int):
    """The SGPR oracle on n_sample points of config 5 (same m), scaled by n_full / n_sample: every
    O(n) term of the SoR path (products n m c, root n m^2, derivative pairs n m) is linear in n."""
    from oracle import sgpr_oracle as S
    from paper_1809_11165_amd import inputs
    w = inputs.make(5, n=n_sample, m=m)
    t0 = time.perf_counter()
    S.sor_bbmm_inference(w.kernel, w.X, w.Uind, w.y, w.lengthscale, w.outputscale, w.noise, w.jitter_rel,
                         w.E1, w.E2, w.k, w.iters)
    dt = time.perf_counter() - t0
    return {"value": dt * 1e3 * (n_full / n_sample), "unit": "ms", "cores": _cores(),
            "kind": "oracle",
            "sample": "fp64 numpy SGPR oracle, full call (m=%d, k=10, t=10, 50 iterations) on n=%d points of "
                      "the same recipe: %.1f s measured, scaled by n/n_sample = %.0f"
                      % (m, n_sample, dt, n_full / n_sample)}


TRAFFIC_NOTE = ("HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this kernel on this "
                "workload (profiles/%s), not counted in this run")


def roofline_sym(n, c, mm_ms, launches, config):
    """Product from the stored upper triangle.  The triangle is read once (2 n^2 + 4 n W bytes,
    W = 1024: the diagonal blocks are whole), which no longer binds; every stored 16 x 16 tile still
    takes its fp64 MFMAs for both of its uses, so the product is bound by the fp64 matrix rate.
    Algorithmic flops of one product: 2 c per pair of points (c = t + 1 columns really used).
    Executed: per pair 16 columns on the row-side use and 12 or 16 on the column-side use (12 when at
    most 12 columns of a 16-column group are in use), each on half the pairs; reported beside it."""
    alg_flops = 2.0 * c * n * n
    achieved = alg_flops / (mm_ms * 1e-3) / 1e12
    wide = sum(16 + (12 if min(16, c - 16 * q) <= 12 else 16) for q in range((c + 15) // 16))
    executed = wide * n * n / (mm_ms * 1e-3) / 1e12
    return {"bound": "mfma", "achieved": achieved, "peak": MFMA_F64_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": achieved / MFMA_F64_PEAK_TFLOPS,
            "traffic": MEASURED_TRAFFIC_SYM_N50000 if (n, config) == (50000, 3) else None,
            "traffic_source": TRAFFIC_NOTE % "k_mm_sym_cfg3_n50000_counters.txt" if (n, config) == (50000, 3) else None,
            "kernel": "k_mm_sym (one launch per product for c <= 12, else a second one for the diagonal blocks)",
            "avg_launch_ms": mm_ms, "launches": launches,
            "executed_TFLOPs_with_padding": executed,
            "executed_frac": executed / MFMA_F64_PEAK_TFLOPS}


def roofline_mat(n, c, mm_ms, launches, config):
    """Whole K_hat streamed once per product: algorithmic bytes 4 n^2 (K_hat) + 8 n c (block in and out)."""
    alg_bytes = 4.0 * n * n + 8.0 * n * c
    achieved = alg_bytes / (mm_ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_MAT_N50000 if (n, config) == (50000, 3) else None,
            "traffic_source": TRAFFIC_NOTE % "k_mm_mat_cfg3_n50000_hbm_counters.txt" if (n, config) == (50000, 3) else None,
            "kernel": "k_mm_mat", "avg_launch_ms": mm_ms, "launches": launches}


def roofline_otf(n, c, d, mm_ms, launches):
    """Tiles rebuilt from X in every product.  Algorithmic flops per pair: 2 d (distance contraction)
    + 2 c (multiply by the block).  `frac` prices all of them at the fp32 matrix rate; the second
    contraction is carried out in fp64, at half that rate on the same pipe, so the floor of the two
    together is n^2 (2 d / peak32 + 2 c / peak64): `frac_of_mixed_floor` is that floor over the
    launch time."""
    alg_flops = (2.0 * d + 2.0 * c) * n * n
    achieved = alg_flops / (mm_ms * 1e-3) / 1e12
    mixed_floor_ms = n * n * (2.0 * d / MFMA_F32_PEAK_TFLOPS + 2.0 * c / MFMA_F64_PEAK_TFLOPS) * 1e-9
    return {"bound": "mfma", "achieved": achieved, "peak": MFMA_F32_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": achieved / MFMA_F32_PEAK_TFLOPS, "traffic": None,
            "kernel": "k_mm_otf_tri (tiles on and above the diagonal, each used twice; two launches per product)"
                      if (c <= 16 and d <= 32 and -(-n // 256) * 256 >= 12288) else "k_mm_otf",
            "avg_launch_ms": mm_ms, "launches": launches,
            "pairs_per_s": n * n / (mm_ms * 1e-3),
            "mixed_floor_ms": mixed_floor_ms, "frac_of_mixed_floor": mixed_floor_ms / mm_ms}


def time_calls(ctx, prob, warmup, steps):
    """(ms per call, mean ms per K_hat.M product from HIP events on the library's stream, launches, last result)"""
    import torch
    res = None
    for _ in range(warmup):
        res = ctx.bbmm_solve_logdet_grad(prob, want_U=False)
    torch.cuda.synchronize()
    mm_avgs, launches = [], 0
    t0 = time.perf_counter()
    for _ in range(steps):
        res = ctx.bbmm_solve_logdet_grad(prob, want_U=False)
        avg, tot, cnt = ctx.bbmm_mm_timing()
        mm_avgs.append(avg)
        launches += cnt
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt * 1e3 / steps, float(np.mean(mm_avgs)), launches, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--mode", choices=["sym", "mat", "otf", "sgpr"], default=None,
                    help="default: sym (mat for --config 2, otf for --config 4)")
    ap.add_argument("--config", type=int, choices=[2, 3, 4], default=3,
                    help="exact-GP workload: 3 (default, the headline), 2 (n = 10000, RBF, tolerance stop) "
                         "or 4 (n = 200000, RBF, 17 columns, 100 iterations)")
    ap.add_argument("--n", type=int, default=None,
                    help="points (default 50000; 10000 for --config 2; 200000 for --config 4; 500000 for --mode sgpr)")
    ap.add_argument("--m", type=int, default=1024, help="inducing inputs (--mode sgpr)")
    ap.add_argument("--cpu-sample", type=int, default=10000)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-other-modes", action="store_true",
                    help="default run only: skip the whole-matrix and on-the-fly legs (roofline_mat, roofline_otf)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)")
    if args.mode is None:
        # the fastest storage of each configuration: the triangle at n = 50,000; the whole matrix at
        # n = 10,000 (short runs per workgroup favour the simpler product); tiles on the fly at n = 200,000
        args.mode = {3: "sym", 2: "mat", 4: "otf"}[args.config]

    import torch
    from paper_1809_11165_amd import binding, inputs

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU: the path runs only in the HIP library")
    mode = {"mat": inputs.MATERIALISED, "sym": inputs.MATERIALISED, "otf": inputs.ONTHEFLY,
            "sgpr": inputs.SGPR}[args.mode]
    if args.n is None:
        args.n = 500000 if mode == inputs.SGPR else {3: 50000, 2: 10000, 4: 200000}[args.config]
    w = inputs.make(5, n=args.n, m=args.m) if mode == inputs.SGPR else inputs.make(args.config, n=args.n)
    prob = binding.problem_from_workload(w, mode)
    ctx = binding.Context(0)
    ctx.bbmm_tune("time_mm", 1)
    if args.mode == "sym":
        ctx.bbmm_tune("khat_sym", 1)        # keep the upper triangle of K_hat only

    ms_per_step, mm_ms, mm_launches, res = time_calls(ctx, prob, args.warmup, args.steps)

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    n, c, d = w.n, w.t + 1, w.d
    workload = "config3: exact GP, Matern-5/2 ARD, n=%d, d=16, t=10, k=20, 50 mBCG iterations" % n
    metric = "mBCG solve+logdet+grad ms at n=50k,t=10"
    if args.config == 2:
        workload = ("config2: exact GP, RBF, n=%d, d=8, t=10, k=10, mBCG to a relative residual of 1e-2 or "
                    "50 iterations" % n)
        metric = "mBCG solve+logdet+grad ms at n=10k,t=10 (config 2)"
    if args.config == 4:
        workload = ("config4: exact GP, RBF, 20 Gaussian clusters, n=%d, d=8, t=16, k=20, 100 mBCG iterations" % n)
        metric = "mBCG solve+logdet+grad ms at n=200k,t=16 (config 4)"
    mode_name = "materialised fp32 K_hat" if mode == inputs.MATERIALISED else "on-the-fly tiles"
    if mode == inputs.SGPR:
        # one product = the root A (n x m fp32) streamed once in each layout, the block in and out,
        # the m x c middle result out and in: 8 n m + 16 n c + 16 m c bytes
        m = args.m
        alg_bytes = 8.0 * n * m + 16.0 * n * c + 16.0 * m * c
        achieved = alg_bytes / (mm_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS,
                    "traffic": MEASURED_TRAFFIC_SGPR_N500000_M1024 if (n, m) == (500000, 1024) else None,
                    "traffic_source": (TRAFFIC_NOTE % "k_mm_mat_cfg5_n500000_sgpr_hbm_counters.txt"
                                       if (n, m) == (500000, 1024) else None),
                    "kernel": "k_mm_mat (two launches per product: A^T D, then A T)",
                    "avg_launch_ms": mm_ms / 2.0, "avg_product_ms": mm_ms, "launches": 2 * mm_launches}
        workload = ("config5: SGPR (subset of regressors), RBF, n=%d, m=%d, d=8, t=10, k=10, 50 mBCG "
                    "iterations" % (n, m))
        metric = "mBCG solve+logdet+grad ms at n=500k,m=1024,t=10 (SGPR)"
        mode_name = "fp32 root A = K_XU G^-T in both layouts"
    elif args.mode == "sym":
        roofline = roofline_sym(n, c, mm_ms, mm_launches, args.config)
        mode_name = "materialised fp32 K_hat, upper triangle only (khat_sym)"
    elif mode == inputs.MATERIALISED:
        roofline = roofline_mat(n, c, mm_ms, mm_launches, args.config)
    else:
        roofline = roofline_otf(n, c, d, mm_ms, mm_launches)

    out = {
        "metric": metric,
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": workload,
                   "mode": mode_name,
                   "arithmetic": "kernel-matrix entries fp32 (stored or generated), products, sums and all "
                                 "n x c blocks fp64",
                   "iters_run": res.iters_run, "ms_per_iteration": ms_per_step / max(res.iters_run, 1),
                   "mm_ms_per_iteration": mm_ms,
                   "logdet": res.logdet, "nlml": res.nlml},
        "roofline": roofline,
    }
    if args.config == 3 and args.mode == "sym" and not args.no_other_modes:
        # the same workload in the other two product modes, in the same run (1 warm-up + 3 timed calls
        # each): the HBM-bound whole-matrix product and the on-the-fly product
        # (a failure of one of these legs -- say the whole matrix does not fit next to other tenants of
        # the GPU -- is reported in its place and leaves the headline line intact)
        ctx.bbmm_tune("khat_sym", 0)
        try:
            ms_mat, mm_mat, l_mat, r_mat = time_calls(ctx, prob, 1, 3)
            out["roofline_mat"] = dict(roofline_mat(n, c, mm_mat, l_mat, args.config), ms_per_call=ms_mat,
                                       mode="materialised fp32 K_hat, whole matrix", logdet=r_mat.logdet)
        except binding.BbmmError as e:
            out["roofline_mat"] = {"error": str(e)}
        try:
            prob_otf = binding.problem_from_workload(w, inputs.ONTHEFLY)
            ms_otf, mm_otf, l_otf, r_otf = time_calls(ctx, prob_otf, 1, 3)
            out["roofline_otf"] = dict(roofline_otf(n, c, d, mm_otf, l_otf), ms_per_call=ms_otf,
                                       mode="on-the-fly tiles", logdet=r_otf.logdet)
        except binding.BbmmError as e:
            out["roofline_otf"] = {"error": str(e)}
    if not args.no_cpu:
        out["cpu_baseline"] = (cpu_baseline_sgpr(min(n, 5 * args.cpu_sample), n, args.m)
                               if mode == inputs.SGPR
                               else cpu_baseline(args.config, min(n, args.cpu_sample), n, res.iters_run))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
