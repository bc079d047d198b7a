#!/usr/bin/env python3
"""Benchmark of the ALS hot path on one MI355X: seconds per sweep (X-update + Theta-update) at f = 100
on the Netflix-shaped synthetic workload, with the get_hermitian roofline and the CPU oracle beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mid] [--solver cg|cholesky]

Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_16BIT_MFMA_TFLOPS = 2500.0   # dense bf16 / fp16 MFMA
PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline_implicit(w, a_host, alpha):
    """The implicit-feedback oracle (the sum over all m*n pairs, as the cost is defined) on a sample of rows and
    columns; every row costs the same there (n f^2), so the sample is scaled by the number of rows."""
    import numpy as np
    import oracle
    import workload as W
    _, T0 = W.init_factors(w)
    rows = np.linspace(0, w.m - 1, num=min(w.m, 6000), dtype=np.int64)
    t0 = time.perf_counter()
    oracle.implicit_update_selected(rows, a_host.ptr, a_host.idx, a_host.val, T0, w.lam, alpha)
    t_rows = time.perf_counter() - t0
    c = W.transpose(a_host)
    cols = np.linspace(0, w.n - 1, num=min(w.n, 200), dtype=np.int64)
    Xs = W.random_factors(w.m, w.f, seed=9, scale=0.5)
    t0 = time.perf_counter()
    oracle.implicit_update_selected(cols, c.ptr, c.idx, c.val, Xs, w.lam, alpha)
    t_cols = time.perf_counter() - t0
    est = t_rows * (w.m / len(rows)) + t_cols * (w.n / len(cols))
    return {"value": est, "unit": "s/sweep", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": (f"exact fp64 all-pairs oracle on {len(rows)} evenly spaced rows ({t_rows:.2f} s) and {len(cols)} columns "
                       f"({t_cols:.2f} s), scaled by the numbers of rows and columns")}


def cpu_baseline(w, a_host, stride):
    """The oracle's exact sweep timed on every `stride`-th row and column, scaled by stored entries."""
    import numpy as np
    import oracle
    import workload as W
    _, T0 = W.init_factors(w)
    rows = np.arange(0, w.m, stride, dtype=np.int64)
    nnz_rows = int((a_host.ptr[rows + 1] - a_host.ptr[rows]).sum())
    t0 = time.perf_counter()
    oracle.update_selected(rows, a_host.ptr, a_host.idx, a_host.val, T0, w.lam)
    t_rows = time.perf_counter() - t0
    # column side: the same kernel of work on a CSC slice; build it from the sampled columns only
    c = W.transpose(a_host)
    cols = np.arange(0, w.n, stride, dtype=np.int64)
    nnz_cols = int((c.ptr[cols + 1] - c.ptr[cols]).sum())
    Xs = W.random_factors(w.m, w.f, seed=9, scale=0.5)
    t0 = time.perf_counter()
    oracle.update_selected(cols, c.ptr, c.idx, c.val, Xs, w.lam)
    t_cols = time.perf_counter() - t0
    est = t_rows * (a_host.nnz / max(nnz_rows, 1)) + t_cols * (a_host.nnz / max(nnz_cols, 1))
    return {"value": est, "unit": "s/sweep", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": (f"one whole exact fp64 sweep: all rows ({t_rows:.2f} s), then all columns ({t_cols:.2f} s)" if stride == 1
                       else f"exact fp64 oracle on every {stride}th row ({nnz_rows} entries, {t_rows:.2f} s) and every "
                            f"{stride}th column ({nnz_cols} entries, {t_cols:.2f} s), scaled by stored entries")}


# HBM bytes moved per launch by each get_hermitian kernel, from the rocprofv3 counter runs summarised in the file
# named here: FETCH_SIZE and WRITE_SIZE summed over the kernel's dispatches of one sweep, scaled by what the same
# counters read for a copy of known size (2 KiB and 1 KiB per count), divided by its launches.  Counters cannot be
# read from inside this process, so the figure is only reported for the configuration it was measured on;
# tests/test_host_logic.py checks the numbers against the file.
TRAFFIC_SOURCE = "profiles/k_hermitian_mid_f100_cg6_counters.txt"
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {
    ("mid", 100, "cg", 6, "f32", 4096): {
        "k_hermitian": ((3.282e5 + 1.043e7) * 2048 + (2.86e5 + 5.569e5) * 1024) / 2,
        "k_hermitian_cg": ((1.937e6 + 3.546e6) * 2048 + (4.125e4 + 5012) * 1024) / 2,
    },
}


def measured_traffic(w, args, chunk, kernel):
    """(HBM bytes per launch of `kernel`, where the figure comes from), or (None, None)."""
    if args.implicit is not None or args.batch_slots != 0 or args.herm_dtype != "f32":
        return None, None
    key = (w.name, w.f, args.solver, args.cg_iters if args.solver == "cg" else 0, args.factor_dtype, chunk)
    per_kernel = MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(key)
    if per_kernel is None or kernel not in per_kernel:
        return None, None
    return per_kernel[kernel], TRAFFIC_SOURCE


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="mid")
    ap.add_argument("--solver", default="cg", choices=["cg", "cholesky"])
    ap.add_argument("--herm-dtype", default="f32", choices=["f32", "bf16"],
                    help="storage of the partial Gram matrices that go through slots (Section 4.2); bf16 needs --solver cg")
    ap.add_argument("--no-reduced", action="store_true", help="skip the extra timings in the other input modes")
    ap.add_argument("--dense-short-rows", action="store_true",
                    help="rows with fewer than 64 entries build A_u too (the paper's route for every row) instead of "
                         "running Algorithm 1 on their gathered rows")
    ap.add_argument("--test-frac", type=float, default=0.0,
                    help="hold out this fraction of the entries (seeded), fit on the rest and report the held-out RMSE "
                         "per sweep and the time to come within 0.2 %% of its best value (protocol of Section 5.2)")
    ap.add_argument("--implicit", type=float, default=None, metavar="ALPHA",
                    help="time implicit-feedback sweeps (Section 5.6) with this confidence scale instead")
    ap.add_argument("--cg-iters", type=int, default=6)
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--batch-slots", type=int, default=0)
    ap.add_argument("--cpu-stride", type=int, default=1, help="oracle baseline on every k-th row/column (1 = one whole exact sweep, about 20 s on 16 host threads); 0 = skip")
    ap.add_argument("--f", type=int, default=0, help="override the workload's factor width (factor-width sweep)")
    ap.add_argument("--factor-dtype", default="f32", choices=["f32", "bf16", "f16", "f32x3", "f32x2"],
                    help="element type of the gathered factor matrix (16-bit: multiplied on the 16-bit matrix cores, fp32 accumulate; "
                         "f32x3: fp32 in memory, cut into three bf16 parts and multiplied on the 16-bit matrix cores at fp32 accuracy; "
                         "f32x2: fp32 in memory, scaled and cut into two fp16 parts, three products per pair)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device copy five times (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1.0, out=dst)      # an elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": "5 x (read 1 GiB, write 1 GiB), torch elementwise add kernel"}))
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (rows are independent, so the path shards by rows; "
                 "no collective is built). Run with --gpus 1.")

    import numpy as np
    import torch
    import paper_1808_03843_amd as P
    import workload as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    w = W.CONFIGS[args.workload]
    if args.f:
        w = w.with_f(args.f)
    dev = "cuda:0"
    t0 = time.perf_counter()
    a = W.generate(w)
    log(f"[bench] generated {w.name}: {w.m} x {w.n}, {a.nnz} stored entries in {time.perf_counter() - t0:.1f} s")
    held_out = None
    if args.test_frac > 0:
        a, held_out = W.split(a, args.test_frac, seed=w.seed)
        log(f"[bench] held out {held_out.nnz} entries, fitting on {a.nnz}")
    solver = P.SOLVER_CG if args.solver == "cg" else P.SOLVER_CHOLESKY
    fcode = {"f32": P.F32, "bf16": P.BF16, "f16": P.F16, "f32x3": P.F32X3, "f32x2": P.F32X2}[args.factor_dtype]
    ftorch = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16, "f32x3": torch.float32, "f32x2": torch.float32}[args.factor_dtype]
    in_fp32 = args.factor_dtype in ("f32", "f32x3", "f32x2")   # the gathered factor is the fp32 matrix itself
    als = P.Als(w.f, solver=solver, cg_iters=args.cg_iters, chunk=args.chunk, batch_slots=args.batch_slots,
                profile=True, factor_dtype=fcode, herm_dtype=P.BF16 if args.herm_dtype == "bf16" else P.F32,
                dense_short_rows=args.dense_short_rows)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val, device=dev)
    csc = als.csr_to_csc(csr)
    X0, T0 = W.init_factors(w)
    X, T = torch.from_numpy(X0).to(dev), torch.from_numpy(T0).to(dev)
    del X0

    def sweep():
        if args.implicit is not None:
            als.update_rows_implicit(csr, T, w.lam, args.implicit, X)
            als.update_cols_implicit(csc, X, w.lam, args.implicit, T)
            return
        # 16-bit modes: the gathered factor is converted by torch inside the timed region (part of the sweep)
        als.update_rows(csr, T if in_fp32 else T.to(ftorch), w.lam, X)
        als.update_cols(csc, X if in_fp32 else X.to(ftorch), w.lam, T)

    for _ in range(args.warmup):
        sweep()
    torch.cuda.synchronize()
    als.profile_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sweep()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sec_per_sweep = elapsed / args.steps
    herm_ms, herm_n = als.kernel_time(P.K_HERMITIAN)
    fused_ms, fused_n = als.kernel_time(P.K_FUSED)
    solve_ms, solve_n = als.kernel_time(P.K_SOLVE)
    gram_ms, gram_n = als.kernel_time(P.K_GRAM)
    short_ms, short_n = als.kernel_time(P.K_SHORT)
    als.synchronize()
    ev = P.Als(w.f, profile=True)
    ev.rmse(csr, X, T)                       # first call builds the plan of the matrix
    ev.profile_reset()
    rmse = ev.rmse(csr, X, T)
    rmse_ms, _ = ev.kernel_time(P.K_RMSE)
    ev.close()
    # batched RMSE (Section 5.2): gathered bytes per entry = 4 f (theta row) + 8 (column id, rating)
    rmse_gbps = a.nnz * (4.0 * w.f + 8.0) / max(rmse_ms * 1e-3, 1e-12) / 1e9
    K = args.steps
    log(f"[bench] {K} sweeps in {elapsed:.3f} s; rmse {rmse:.5f}; per sweep: k_hermitian {herm_ms / K:.2f} ms "
        f"({herm_n // K} launches), k_hermitian_cg {fused_ms / K:.2f} ms ({fused_n // K}), "
        f"k_cg_gathered {short_ms / K:.2f} ms ({short_n // K}), slot solve {solve_ms / K:.2f} ms ({solve_n // K}); rmse kernel {rmse_ms:.2f} ms ({rmse_gbps:.0f} GB/s gathered)"
        + (f", gram {gram_ms / K:.2f} ms ({gram_n // K}); implicit cost {als.implicit_loss(csr, X, T, w.lam, args.implicit):.6e}"
           if args.implicit is not None else ""))

    # get_hermitian roofline.  Algorithmic flops = f*(f+1) per stored entry and half-sweep (lower triangle
    # of theta theta^T, FMA = 2).  Rows with >= chunk entries are built by k_hermitian into slots, shorter
    # rows by k_hermitian_cg (which also runs the solver: its time is charged to get_hermitian in full).
    chunk = als.cfg.chunk or 4096
    deg_r = np.diff(a.ptr)
    deg_c = np.bincount(a.idx, minlength=w.n)
    nnz_fit = int(a.nnz)   # entries the factors are fitted on (all of them unless --test-frac)
    nnz_slot = int(deg_r[deg_r >= chunk].sum() + deg_c[deg_c >= chunk].sum()) if (fused_n > 0 or short_n > 0) else 2 * nnz_fit
    # short rows run Algorithm 1 on their gathered rows and never form A_u (k_cg_gathered): their
    # entries are no get_hermitian work and are left out of its flops
    short_limit = als.short_row_limit()   # 64, or 128 on the fp32 MFMA path at f = 100 / 128; 0: no such rows
    short_rows = int((deg_r < short_limit).sum() + (deg_c < short_limit).sum()) if short_n > 0 else 0
    nnz_short = int(deg_r[deg_r < short_limit].sum() + deg_c[deg_c < short_limit].sum()) if short_n > 0 else 0
    per_entry = w.f * (w.f + 1)
    flops_sweep = (2.0 * nnz_fit - nnz_short) * per_entry
    herm_s = (herm_ms + fused_ms) * 1e-3 / K
    achieved = flops_sweep / herm_s / 1e12          # all get_hermitian launches of a sweep together
    launches = (herm_n + fused_n) // K
    # The two get_hermitian kernels, each with its own launches: entries (the unit of work), flops and time per launch.
    kernels = {}
    for name, what, ms, n, entries in (
            ("k_hermitian", "get_hermitian of the work items of rows with >= chunk entries, into slots", herm_ms, herm_n, nnz_slot),
            ("k_hermitian_cg", "get_hermitian fused with the solver (rows shorter than a chunk); its whole time is charged "
                               "to get_hermitian", fused_ms, fused_n, 2 * nnz_fit - nnz_slot - nnz_short)):
        if n <= 0:
            continue
        per_launch = entries / (n / K)
        avg_ms = ms / n
        tf = per_launch * per_entry / (avg_ms * 1e-3) / 1e12
        kernels[name] = {"what": what, "tflops": tf, "frac": tf / PEAK_FP32_MFMA_TFLOPS, "ms_per_sweep": ms / K,
                         "launches_per_sweep": n // K, "avg_launch_ms": avg_ms, "entries_per_launch": per_launch,
                         "entries_per_sweep": entries}
    short = None
    if short_n > 0:
        # Algorithm 1 on the gathered rows: per row (f_s + 1) products of 4 n_u f + 2 f flops and b_u (2 n_u f), on the
        # vector ALUs
        fl = (args.cg_iters + 1) * (4.0 * nnz_short * w.f + 2.0 * w.f * short_rows) + 2.0 * nnz_short * w.f
        short = {"what": f"Algorithm 1 on the gathered rows of rows with fewer than {short_limit} entries, A_u never formed "
                         "(A_u p = G^T (G p) + lambda n_u p)", "bound": "alu", "ms_per_sweep": short_ms / K,
                 "launches_per_sweep": short_n // K, "rows_per_sweep": short_rows, "entries_per_sweep": nnz_short,
                 "systems_per_s": short_rows / (short_ms / K * 1e-3), "tflops": fl / (short_ms / K * 1e-3) / 1e12,
                 "frac_of_fp32_vector_peak": fl / (short_ms / K * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_sweep"])   # the kernel that takes most of the sweep
    d = kernels[dom]
    traffic, traffic_source = measured_traffic(w, args, chunk, dom)
    roofline = {"bound": "mfma", "achieved": d["tflops"], "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": d["frac"], "traffic": traffic, "traffic_source": traffic_source,
                "kernel": dom, "avg_launch_ms": d["avg_launch_ms"], "units_per_launch": d["entries_per_launch"],
                "unit_of_work": f"stored entry: f(f+1) = {per_entry} flops (lower triangle of theta theta^T, FMA = 2), "
                                f"{4 * w.f + 8} gathered bytes",
                "flops_per_launch": d["entries_per_launch"] * per_entry,
                "dominant_kernel": {"name": dom, "avg_launch_ms": d["avg_launch_ms"],
                                    "units_per_launch": d["entries_per_launch"], "frac": d["frac"]},
                "all_get_hermitian": {"achieved": achieved, "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                                      "ms_per_sweep": (herm_ms + fused_ms) / K, "launches_per_sweep": launches,
                                      "flops_per_sweep": flops_sweep},
                **kernels, **({"k_cg_gathered": short} if short else {})}
    if args.factor_dtype in ("f32x3", "f32x2"):
        # fp32 values as 16-bit parts on the 16-bit matrix cores: the numerator stays the algorithmic flops of the
        # fp32 Gram matrix, the denominator is the peak of the instruction that runs, the 16-bit dense MFMA peak
        for k in kernels.values():
            k["frac"] = k["tflops"] / PEAK_16BIT_MFMA_TFLOPS
            k["frac_of_fp32_mfma_peak"] = k["tflops"] / PEAK_FP32_MFMA_TFLOPS
        roofline.update({"peak": PEAK_16BIT_MFMA_TFLOPS, "frac": d["frac"],
                         "note": "algorithmic fp32 flops against the 16-bit MFMA peak: six bf16 (f32x3) or three fp16 (f32x2) "
                                 "products per fp32 product, so the ceiling of the mode is 1/6 (1/3) of the 16-bit peak = "
                                 "417 (833) TFLOP/s of Gram work"})
        roofline["dominant_kernel"]["frac"] = d["frac"]
        roofline["all_get_hermitian"]["frac"] = achieved / PEAK_16BIT_MFMA_TFLOPS
        roofline["all_get_hermitian"]["frac_of_fp32_mfma_peak"] = achieved / PEAK_FP32_MFMA_TFLOPS
    elif args.factor_dtype != "f32":
        # 16-bit factor inputs run on the 16-bit matrix cores (16x the fp32 rate): the gathers bound the kernel.
        # Algorithmic bytes per stored entry and half-sweep: one 16-bit factor row + column id + rating.
        per_entry_b = 2.0 * w.f + 8.0
        for k in kernels.values():
            k["gathered_GBps"] = k["entries_per_launch"] * per_entry_b / (k["avg_launch_ms"] * 1e-3) / 1e9
            k["frac"] = k["gathered_GBps"] / 8000.0
            k["frac_of_16bit_mfma_peak"] = k["tflops"] / PEAK_16BIT_MFMA_TFLOPS
        gbps_all = 2.0 * nnz_fit * per_entry_b / herm_s / 1e9
        roofline.update({"bound": "hbm", "achieved": d["gathered_GBps"], "peak": 8000.0, "unit": "GB/s",
                         "frac": d["frac"], "traffic": None, "traffic_source": None,
                         "unit_of_work": f"stored entry: {per_entry_b:.0f} gathered bytes (16-bit factor row, column id, rating)",
                         "bytes_per_launch": d["entries_per_launch"] * per_entry_b,
                         "dominant_kernel": {"name": dom, "avg_launch_ms": d["avg_launch_ms"],
                                             "units_per_launch": d["entries_per_launch"], "frac": d["frac"]},
                         "all_get_hermitian": {"achieved": gbps_all, "frac": gbps_all / 8000.0,
                                               "ms_per_sweep": (herm_ms + fused_ms) / K, "launches_per_sweep": launches},
                         "mfma": {"achieved_tflops": achieved, "peak_tflops": PEAK_16BIT_MFMA_TFLOPS,
                                  "frac": achieved / PEAK_16BIT_MFMA_TFLOPS}})
        roofline.pop("flops_per_launch", None)
    out = {
        "metric": f"seconds per {'implicit-feedback ' if args.implicit is not None else ''}ALS sweep (X+Theta) at f={w.f}",
        "value": sec_per_sweep, "unit": "s/sweep",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec_per_sweep * 1e3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.factor_dtype in ("f32x3", "f32x2") else args.factor_dtype, "data": "synthetic",
        "factor_dtype": args.factor_dtype, "herm_dtype": args.herm_dtype,
        "config": {"workload": f"{w.name}: m={w.m} n={w.n} nnz={nnz_fit} f={w.f} lambda={w.lam}",
                   "solver": args.solver + (f"({args.cg_iters})" if args.solver == "cg" else ""),
                   **({"implicit_alpha": args.implicit} if args.implicit is not None else {}),
                   "chunk": chunk, "batch_slots": als.cfg.batch_slots or 131072},
        "hermitian_tflops": achieved, "hermitian_ms_per_sweep": (herm_ms + fused_ms) / K,
        # the paper counts N_z f^2 multiply-adds per update (the full square, Section 3): for comparison with its
        # figures only, never the roofline fraction
        "hermitian_tflops_paper_convention": 4.0 * nnz_fit * w.f * w.f / herm_s / 1e12,
        # the paper's own timings (Table 4), other hardware and the real datasets: context, not a target
        "paper_context": {"netflix_seconds_to_test_rmse_0.92": {"Maxwell Titan X": 6.5, "Pascal P100": 3.3},
                          "note": "whole training runs to a test RMSE on the Netflix data (same shape as this workload), "
                                  "CG f_s=6, FP16 storage of A; no per-sweep time is printed in the paper"},
        "solve_ms_per_sweep": solve_ms / K, "train_rmse": rmse,
        "rmse_kernel": {"ms": rmse_ms, "gathered_GBps": rmse_gbps, "hbm_peak_GBps": 8000.0,
                        "note": "gathered bytes; above the HBM rate when the gathered factor is cache-resident"},
        "roofline": roofline,
    }
    if args.factor_dtype == "f32" and args.implicit is None and not args.no_reduced:
        # The same sweeps in the two other input modes, continuing from the factors reached above; reported beside the
        # fp32 figure, never as `value`.  f32x3: the fp32 factor itself, multiplied on the 16-bit matrix cores as three
        # bf16 parts (fp32 accuracy, f <= 128).  bf16: the factor rounded to bf16 each half-sweep (Section 4.2 taken to
        # the matrix cores; reduced precision).
        modes = [("bf16_factor_inputs", P.BF16, torch.bfloat16,
                  "gathered factor rounded to bf16 each half-sweep (conversion timed), v_mfma_f32_16x16x32_bf16 with fp32 "
                  "accumulate, fp32 solver and output")]
        if solver == P.SOLVER_CG and w.f <= 128 and not args.dense_short_rows:
            modes.append(("every_row_builds_A_u", P.F32, None,
                          "dense_short_rows = 1: rows with fewer than 64 entries also go through get_hermitian and the "
                          "dense Algorithm 1, as in the paper"))
        if w.f <= 128:
            modes.insert(0, ("f32x3_factor_inputs", P.F32X3, None,
                             "fp32 factor cut into three bf16 parts in registers, six products per pair on "
                             "v_mfma_f32_16x16x32_bf16, fp32 accumulate: the tolerances of the fp32 path"))
            modes.insert(1, ("f32x2_factor_inputs", P.F32X2, None,
                             "fp32 factor scaled by a power of two and cut into two fp16 parts in registers (to nearest), "
                             "three products per pair on v_mfma_f32_16x16x32_f16, fp32 accumulate: held to the tolerances "
                             "of the fp32 path"))
        for key, code, tdt, note in modes:
            a2 = P.Als(w.f, solver=solver, cg_iters=args.cg_iters, chunk=args.chunk, batch_slots=args.batch_slots,
                       factor_dtype=code, dense_short_rows=key == "every_row_builds_A_u")
            X2, T2 = X.clone(), T.clone()

            def sweep2():
                a2.update_rows(csr, T2 if tdt is None else T2.to(tdt), w.lam, X2)
                a2.update_cols(csc, X2 if tdt is None else X2.to(tdt), w.lam, T2)
            sweep2()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                sweep2()
            torch.cuda.synchronize()
            ms2 = (time.perf_counter() - t1) / args.steps * 1e3
            a2.synchronize()
            ev = P.Als(w.f)
            rmse2 = ev.rmse(csr, X2, T2)
            ev.close()
            a2.close()
            del X2, T2
            out[key] = {"ms_per_step": ms2, "train_rmse": rmse2, "sweeps_after_fp32": args.steps + 1, "note": note}
            log(f"[bench] {key}: {ms2:.2f} ms per sweep, rmse {rmse2:.5f}")
    # what the machine sustains on the simplest kernels (back-to-back MFMAs, a streaming copy): the reachable
    # counterparts of the published peaks the roofline is quoted against
    pk = P.Als(w.f)
    mf32, mbf16, cp = (pk.measure_peak(k) for k in (P.PEAK_MFMA_F32, P.PEAK_MFMA_BF16, P.PEAK_COPY))
    pk.close()
    out["measured_peaks"] = {"mfma_f32_TFLOPs": mf32 / 1e12, "mfma_bf16_TFLOPs": mbf16 / 1e12, "copy_GBps": cp / 1e9,
                             "note": "8 wavefronts per SIMD issuing independent MFMAs; copy of 1 GiB, bytes read + written"}
    if roofline["bound"] == "mfma":
        reach = (mbf16 if args.factor_dtype in ("f32x3", "f32x2") else mf32) / 1e12
        roofline["frac_of_measured_peak"] = roofline["achieved"] / reach
        roofline["all_get_hermitian"]["frac_of_measured_peak"] = roofline["all_get_hermitian"]["achieved"] / reach
    else:
        roofline["frac_of_measured_copy"] = roofline["achieved"] / (cp / 1e9)
    log(f"[bench] sustained on this box: fp32 MFMA {mf32 / 1e12:.1f} TFLOP/s, bf16 MFMA {mbf16 / 1e12:.0f} TFLOP/s, "
        f"copy {cp / 1e9:.0f} GB/s")
    if held_out is not None and args.implicit is None:
        # convergence protocol, outside the timed region: restart from the initial factors, held-out RMSE after
        # every sweep, update time accumulated without the evaluations
        te = P.SparseMatrix.from_host(held_out.nrows, held_out.ncols, held_out.ptr, held_out.idx, held_out.val, device=dev)
        X0, T0 = W.init_factors(w)
        X.copy_(torch.from_numpy(X0)); T.copy_(torch.from_numpy(T0))
        ev = P.Als(w.f)
        rm, cum, tsum = [], [], 0.0
        for _ in range(max(args.steps, 1)):
            torch.cuda.synchronize(); t1 = time.perf_counter()
            sweep()
            torch.cuda.synchronize(); tsum += time.perf_counter() - t1
            rm.append(ev.rmse(te, X, T)); cum.append(tsum)
        ev.close()
        best = min(rm)
        hit = next(i for i, r in enumerate(rm) if r <= 1.002 * best)
        out["held_out"] = {"test_frac": args.test_frac, "entries": int(held_out.nnz), "rmse_per_sweep": rm,
                           "seconds_cumulative": cum, "best_rmse": best,
                           "seconds_to_within_0.2pct_of_best": cum[hit], "sweeps_to_within_0.2pct_of_best": hit + 1}
        log(f"[bench] held-out rmse per sweep: " + " ".join(f"{r:.5f}" for r in rm)
            + f"; within 0.2% of the best after {hit + 1} sweeps = {cum[hit] * 1e3:.1f} ms")
    if args.cpu_stride > 0:
        log("[bench] timing the CPU oracle on a sample ...")
        out["cpu_baseline"] = (cpu_baseline_implicit(w, a, args.implicit) if args.implicit is not None
                               else cpu_baseline(w, a, args.cpu_stride))
    else:
        out["cpu_baseline"] = None
    als.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
