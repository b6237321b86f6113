#!/usr/bin/env python3
"""Benchmark of the CAT hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|cfg1..cfg5|cfg2u] [--no-cpu]

One step = one pass of the whole hot path over one synthetic batch that is
already resident in HBM: cat_fit (seeded init, `iters` Lloyd iterations, final
assignment, per-cluster affine fit) followed by cat_apply on the same rows
(inference-only workload cfg5: cat_apply alone).  Prints ONE JSON line.

With no --workload (or "all") the five workloads, and cfg2u (cfg2 with one more
channel: rows that are not whole 16-byte groups, so the fit's Lloyd loop runs on a
zero-padded copy and the inference pass reads and writes word by word), run one
after the other in this process.  The top-level fields are those of cfg3, the largest fitting workload
(1 GiB of rows like cfg4, and the most rows: the metric counts rows); `configs`
holds, for every workload, the same figures: value, ms_per_step, roofline (the
assignment pass), apply_roofline (the fused inference pass), the whole Lloyd
iteration as a fraction of the roofline, and cpu_baseline.  --workload cfgN runs
that workload alone and prints its figures at the top level.  `detail` carries the
rows beside the two calls: the fit with distance bounds (fit_bounds_ms,
lloyd_iter_frac_hbm_bounds: same outputs, its average iteration against the same
algorithmic bytes), the low-precision inference (apply_lp_bf16_*), and on cfg2 the
PCA front-end, the sweep of the blending coefficient, the seeding, the early stop,
the fits for a grid of cluster counts and a shape on the LDS streaming kernel.

value        rows x Lloyd-iterations per second of whole-step time (cfg5: GB/s of
             cat_apply, read + write)
roofline     (traffic: measured HBM bytes per launch from hardware counters, null when the
             kernel source has changed since they were taken or --rows overrides the size)
             the dominant kernel, k_tile (the assignment pass of a Lloyd iteration;
             cfg5: the fused inference pass): algorithmic bytes per launch (one read
             of lq; inference: one read + one write + the assignments) over its mean
             launch duration, measured with HIP events that the library records
             around every k_tile launch on the launch stream, against 8 TB/s.
             detail.lloyd_iter_us is the whole iteration (k_tile_prep + k_tile +
             amortised first-pass sums), detail.lloyd_iter_frac_hbm its fraction
cpu_baseline the CPU oracle timed on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM-side traffic of one launch of the two dominant kernels, from rocprofv3 --pmc runs of this file (FETCH_SIZE,
# then WRITE_SIZE; profiles/k_tile_hbm_traffic.md and profiles/k_infer_hbm_traffic.md have the commands and the raw
# figures).  Each counter is scaled by what it reads for the plain device copy of the same matrix that this script
# also times (a copy reads and writes exactly N*D*b bytes).  Per entry: (FETCH_SIZE of the kernel, FETCH_SIZE of the
# copy, WRITE_SIZE of the kernel, WRITE_SIZE of the copy), counter units, mean per dispatch.  The figures belong to
# one version of a kernel's source file: `traffic` is reported only while the hash of that file still matches, and the
# line says that it comes from profiles/, not from this run.
TRAFFIC_SOURCES = {
    "k_tile": ("cat_tile_kernel.h", "f7df3b216487c7955991ad77a448159b9bc0e66c1d4168af298b081d3a85d32d"),
    "k_infer": ("cat_infer_kernel.h", "d243d921fdcd31650ab229d15f5f562a3fb2bcae57aa0e239eb2055818ac6c93"),
}
TRAFFIC_COUNTERS = {
    "cfg2": ("k_tile", (133499.5, 128011.7, 302.6, 256000.0)),
    "cfg2_apply": ("k_infer", (129304.7, 128011.7, 265969.1, 256000.0)),
    "cfg3": ("k_tile", (526984.8, 524299.7, 4747.4, 1048576.0)),
    "cfg3_apply": ("k_infer", (524886.7, 524299.7, 1054738.2, 1048576.0)),
    "cfg4": ("k_tile", (551642.5, 524299.7, 1273.3, 1048576.0)),
    "cfg4_apply": ("k_tile", (1141365.2, 524299.7, 1049665.2, 1048576.0)),
    "cfg5_apply": ("k_infer", (4197668.4, 4194317.9, 8413243.7, 8388608.0)),
}


def _traffic_bytes(key, copy_bytes):
    """measured HBM bytes per launch, or None (no counters for this workload and kernel / its source changed)"""
    import hashlib
    if key not in TRAFFIC_COUNTERS:
        return None
    kernel, (fk, fc, wk, wc) = TRAFFIC_COUNTERS[key]
    fname, sha = TRAFFIC_SOURCES[kernel]
    try:
        with open(os.path.join(ROOT, "paper_2509_26277_amd", "csrc", fname), "rb") as f:
            if hashlib.sha256(f.read()).hexdigest() != sha:
                return None
    except OSError:
        return None
    return fk * (copy_bytes / fc) + wk * (copy_bytes / wc)


def _traffic_source(key):
    kernel = TRAFFIC_COUNTERS[key][0] if key in TRAFFIC_COUNTERS else "k_tile"
    return f"profiles/{kernel}_hbm_traffic.md (hardware counters of an earlier run of this kernel, not this run)"


def _events(fn, reps, torch):
    """mean milliseconds of fn() over reps calls, HIP events on the current stream"""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    fn()  # untimed: the first launch of a kernel loads its code object
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def _run_workload(name, args, torch, np, cpu_budget_s, extras):
    """All figures of one workload: a dict with the fields of the JSON line."""
    from paper_2509_26277_amd import binding, cat_apply, cat_fit, workloads
    w = workloads.make(name, n_rows=args.rows)
    N, D, K, iters, dt = w["N"], w["D"], w["K"], w["iters"], w["dtype"]
    esize = 4 if dt == "f32" else 2
    fit_kind = w["kind"] == "fit"
    dtc = binding.CAT_F32 if dt == "f32" else binding.CAT_BF16

    def dev(x):
        if dt == "f32":
            return torch.from_numpy(x).cuda()
        bits = workloads.f32_to_bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    lq = dev(w["lq"])
    out = torch.empty_like(lq)
    if fit_kind:
        fp = dev(w["fp"])
        ws_fit = torch.empty(binding.cat_fit_workspace_bytes(N, D, K, dtc), dtype=torch.uint8, device="cuda")
    else:
        cent, gamma, beta = (torch.from_numpy(w[k]).cuda() for k in ("centroids", "gamma", "beta"))
    ws_apply = torch.empty(max(256, binding.cat_apply_workspace_bytes(N, D, K, dtc)), dtype=torch.uint8, device="cuda")
    state = {}

    def step():
        if fit_kind:
            r = cat_fit(lq, fp, K, iters, seed=w["seed"], workspace=ws_fit)
            cat_apply(lq, r["centroids"], r["gamma"], r["beta"], out=out, workspace=ws_apply)
            state["fit"] = r
        else:
            cat_apply(lq, cent, gamma, beta, out=out, workspace=ws_apply)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # ---- per-launch figures, HIP events on the launch stream (torch's current stream) ----
    detail = {}
    apply_bytes = N * D * esize * 2 + 4 * N
    reps = max(5, args.steps)
    if fit_kind:
        r = state["fit"]
        apply_args = (r["centroids"], r["gamma"], r["beta"])
        t_fit = _events(lambda: cat_fit(lq, fp, K, iters, seed=w["seed"], workspace=ws_fit), reps, torch)
        t_fit0 = _events(lambda: cat_fit(lq, fp, K, 0, seed=w["seed"], workspace=ws_fit), reps, torch)
        t_iter = (t_fit - t_fit0) / iters  # one Lloyd iteration
        alg_bytes = N * D * esize
        detail.update(fit_ms=t_fit, fit_iters0_ms=t_fit0, lloyd_iter_us=1e3 * t_iter,
                      lloyd_iters_per_s=1e3 / t_iter, lloyd_rows_per_s=N * 1e3 / t_iter,
                      lloyd_iter_frac_hbm=alg_bytes / t_iter / 1e6 / HBM_PEAK_GBPS)
        # the two segmented-sum steps as calls of their own (the ordering of the rows, the zeroing and the finishing
        # kernels included): the statistics read lq and fp once, the centroid update lq once
        from paper_2509_26277_amd import cat_stats, cat_update
        t_stats = _events(lambda: cat_stats(lq, fp, r["assignments"], K, centroids=r["centroids"], workspace=ws_fit), reps, torch)
        t_upd = _events(lambda: cat_update(lq, r["assignments"], r["centroids"], workspace=ws_fit), reps, torch)
        detail.update(stats_call_us=1e3 * t_stats, stats_call_frac_hbm=2 * alg_bytes / t_stats / 1e6 / HBM_PEAK_GBPS,
                      update_call_us=1e3 * t_upd, update_call_frac_hbm=alg_bytes / t_upd / 1e6 / HBM_PEAK_GBPS)
        # the dominant kernel by itself: events around every k_tile launch of `reps` fits
        binding.profile_enable(True)
        for _ in range(reps):
            cat_fit(lq, fp, K, iters, seed=w["seed"], workspace=ws_fit)
        ms = binding.profile_read()
        binding.profile_enable(False)
        assert len(ms) == reps * (iters + 1), "expected one k_tile launch per assignment pass"
        t_k = sum(ms) / len(ms)
        achieved = alg_bytes / t_k / 1e6
        roof = dict(bound="hbm", kernel="k_tile (assignment pass of a Lloyd iteration)", achieved=achieved,
                    peak=HBM_PEAK_GBPS, unit="GB/s", frac=achieved / HBM_PEAK_GBPS,
                    traffic=None if args.rows else _traffic_bytes(w["name"], N * D * esize),
                    traffic_source=_traffic_source(w["name"]),
                    bytes_per_launch=alg_bytes, us_per_launch=1e3 * t_k, launches=len(ms))
        metric, unit = "cat_fit_lloyd_rows_per_s", "rows/s"
        value = N * iters / (ms_per_step * 1e-3)
    if fit_kind and not args.hot_path_only:
        # the same fit with rows left out by distance bounds (same outputs; a separate figure, never the headline):
        # its average iteration against the same algorithmic bytes, and the share of the rows its passes evaluate
        ws_b = torch.empty(binding.load_library().cat_fit_bounds_workspace_bytes(N, D, K, iters, dtc), dtype=torch.uint8, device="cuda")
        fb = lambda: cat_fit(lq, fp, K, iters, seed=w["seed"], workspace=ws_b, bounds=True)
        ev = fb()["rows_evaluated"].cpu().numpy()
        t_fb = _events(fb, reps, torch)
        t_iter_b = (t_fb - t_fit0) / iters
        detail.update(fit_bounds_ms=t_fb, lloyd_iter_us_bounds=1e3 * t_iter_b,
                      lloyd_iter_frac_hbm_bounds=alg_bytes / t_iter_b / 1e6 / HBM_PEAK_GBPS,
                      bounds_rows_evaluated_frac=float(ev.mean()) / N)
        del ws_b
    if not fit_kind:
        apply_args = (cent, gamma, beta)
        roof = None
        metric, unit = "cat_apply_GBps", "GB/s"
        value = apply_bytes / (ms_per_step * 1e-3) / 1e9
    # the fused inference pass: whole call, and its kernel by itself
    t_apply = _events(lambda: cat_apply(lq, *apply_args, out=out, workspace=ws_apply), reps, torch)
    binding.profile_enable(True)
    for _ in range(reps):
        cat_apply(lq, *apply_args, out=out, workspace=ws_apply)
    ms = binding.profile_read()
    binding.profile_enable(False)
    t_ka = sum(ms) / len(ms)
    apply_roof = dict(bound="hbm", kernel="fused inference pass (assign + gather + affine)", achieved=apply_bytes / t_ka / 1e6,
                      peak=HBM_PEAK_GBPS, unit="GB/s", frac=apply_bytes / t_ka / 1e6 / HBM_PEAK_GBPS,
                      traffic=None if args.rows else _traffic_bytes(w["name"] + "_apply", N * D * esize),
                      traffic_source=_traffic_source(w["name"] + "_apply"),
                      bytes_per_launch=apply_bytes, us_per_launch=1e3 * t_ka, launches=len(ms))
    detail.update(apply_ms=t_apply, apply_GBps=apply_bytes / t_apply / 1e6, apply_frac_hbm=apply_bytes / t_apply / 1e6 / HBM_PEAK_GBPS,
                  apply_rows_per_s=N * 1e3 / t_apply)
    if roof is None:
        roof = apply_roof
    # low-precision deployment of the same transformation: bfloat16 parameters, bfloat16 corrected rows (fp32 rows only)
    if dt == "f32" and not args.hot_path_only:
        from paper_2509_26277_amd import cat_apply_lp, cat_params_to_bf16
        cq, gq, bq = (cat_params_to_bf16(t) for t in apply_args)
        out16 = torch.empty((N, D), dtype=torch.bfloat16, device="cuda")
        ws_lp = torch.empty(binding.load_library().cat_apply_lp_workspace_bytes(N, D, K, dtc), dtype=torch.uint8, device="cuda")
        t_lp = _events(lambda: cat_apply_lp(lq, cq, gq, bq, bf16_out=True, out=out16, workspace=ws_lp), reps, torch)
        lp_bytes = N * D * (esize + 2) + 4 * N
        detail.update(apply_lp_bf16_ms=t_lp, apply_lp_bf16_GBps=lp_bytes / t_lp / 1e6,
                      apply_lp_bf16_frac_hbm=lp_bytes / t_lp / 1e6 / HBM_PEAK_GBPS)
        del out16, ws_lp

    # ---- the PCA front-end (a separate row of the method: not part of `value` or `roofline`) ----
    if extras and fit_kind and args.pca_dim > 0 and D <= 2048:
        from paper_2509_26277_amd import cat_apply_assigned, cat_apply_pca, cat_fit_pca, cat_pca_fit, cat_pca_project
        pdim = min(args.pca_dim, D)
        ws_pca = torch.empty(binding.load_library().cat_pca_workspace_bytes(N, D, pdim, dtc), dtype=torch.uint8, device="cuda")
        mean_p, comps_p, _ = cat_pca_fit(lq, pdim, workspace=ws_pca)
        t_pfit = _events(lambda: cat_pca_fit(lq, pdim, workspace=ws_pca), 2, torch)
        t_proj = _events(lambda: cat_pca_project(lq, mean_p, comps_p), 5, torch)
        r = state["fit"]
        t_lab = _events(lambda: cat_apply_assigned(lq, r["assignments"], r["gamma"], r["beta"], out=out), 5, torch)
        # Algorithm 1 / Algorithm 2 with pca_dim = pdim as single calls
        ws_fp = torch.empty(binding.load_library().cat_fit_pca_workspace_bytes(N, D, K, pdim, dtc), dtype=torch.uint8, device="cuda")
        ws_ap = torch.empty(binding.load_library().cat_apply_pca_workspace_bytes(N, D, K, pdim, dtc), dtype=torch.uint8, device="cuda")
        rp = cat_fit_pca(lq, fp, K, pdim, iters, seed=w["seed"], workspace=ws_fp)
        t_fpca = _events(lambda: cat_fit_pca(lq, fp, K, pdim, iters, seed=w["seed"], workspace=ws_fp), 2, torch)
        t_apca = _events(lambda: cat_apply_pca(lq, rp["mean"], rp["components"], rp["centroids_z"], rp["gamma"], rp["beta"],
                                                out=out, workspace=ws_ap), 5, torch)
        detail.update(fit_pca_ms=t_fpca, apply_pca_ms=t_apca, apply_pca_GBps=apply_bytes / t_apca / 1e6)
        detail.update(pca_dim=pdim, pca_fit_ms=t_pfit, pca_project_us=1e3 * t_proj,
                      pca_project_GBps=N * D * esize / t_proj / 1e6,
                      pca_project_TFLOPs=2.0 * N * D * (16 * ((pdim + 15) // 16)) / t_proj / 1e9,
                      apply_assigned_us=1e3 * t_lab, apply_assigned_GBps=2 * N * D * esize / t_lab / 1e6)

    # ---- the sweep of the blending coefficient (another separate row: the ablation grid of ten values in one pass) ----
    if extras and fit_kind and args.alpha_grid > 0:
        from paper_2509_26277_amd import cat_alpha_sweep, cat_top1
        r = state["fit"]
        grid = [(k + 1) / args.alpha_grid for k in range(args.alpha_grid)]
        ws_sw = torch.empty(binding.load_library().cat_alpha_sweep_workspace_bytes(), dtype=torch.uint8, device="cuda")
        lab = cat_top1(fp)
        t_top = _events(lambda: cat_top1(fp, out=lab), 5, torch)
        sweep = lambda: cat_alpha_sweep(lq, r["assignments"], r["gamma"], r["beta"], grid, fp=fp, labels=lab, workspace=ws_sw)
        res = sweep()
        t_sw = _events(sweep, 5, torch)
        hits = res["hits"].cpu().tolist()
        detail.update(alpha_grid=args.alpha_grid, alpha_sweep_us=1e3 * t_sw, alpha_sweep_GBps=2 * N * D * esize / t_sw / 1e6,
                      alpha_sweep_top1_agreement=[h / N for h in hits], top1_us=1e3 * t_top,
                      top1_GBps=N * D * esize / t_top / 1e6)

    # ---- D^2-weighted seeding (another separate row): K - 1 reads of the rows ----
    if extras and fit_kind and not args.no_seeding:
        from paper_2509_26277_amd import cat_init_kmeanspp
        ws_pp = torch.empty(binding.load_library().cat_init_kmeanspp_workspace_bytes(N, K), dtype=torch.uint8, device="cuda")
        t_pp = _events(lambda: cat_init_kmeanspp(lq, K, seed=w["seed"], workspace=ws_pp), 3, torch)
        detail.update(kmeanspp_ms=t_pp, kmeanspp_GBps=(K - 1) * N * D * esize / t_pp / 1e6)

    # ---- the same fit with the early stop allowed (a separate row: the headline runs every pass) ----
    if extras and fit_kind and not args.no_seeding:
        es = lambda: cat_fit(lq, fp, K, iters, seed=w["seed"], workspace=ws_fit, early_stop=True)
        skipped = int(es()["passes_skipped"].item())
        detail.update(fit_early_stop_ms=_events(es, 5, torch), passes_skipped=skipped)

    # ---- fits for the grid of cluster counts of the paper's ablation, one call against eleven (another separate row) ----
    if extras and fit_kind and not args.no_seeding:
        from paper_2509_26277_amd import cat_fit_multi_k
        grid_k = [k for k in (1, 8, 16, 24, 32, 48, 64, 96, 128, 192, 256) if k <= N]
        t_sep = {k: _events(lambda: cat_fit(lq, fp, k, iters, seed=w["seed"]), 2, torch) for k in grid_k}
        t_multi = _events(lambda: cat_fit_multi_k(lq, fp, grid_k, iters, seed=w["seed"]), 2, torch)
        small = [k for k in grid_k if k <= 32]
        t_small = _events(lambda: cat_fit_multi_k(lq, fp, small, iters, seed=w["seed"]), 2, torch)
        detail.update(multi_k_grid=grid_k, multi_k_ms=t_multi, multi_k_separate_ms=sum(t_sep.values()),
                      multi_k_ratio=t_multi / sum(t_sep.values()), multi_k_upto32_ms=t_small,
                      multi_k_upto32_separate_ms=sum(t_sep[k] for k in small))

    # ---- a shape outside the matrix-core tile kernels (one more channel: rows are no longer whole 16-byte groups): single
    # passes take the row-tile kernel's word-by-word form, fits a zero-padded copy; beside them the same calls on the
    # workload's own, aligned shape and on the LDS streaming kernel ----
    if extras and fit_kind and dt == "f32" and not args.no_seeding:
        from paper_2509_26277_amd import cat_assign
        r = state["fit"]
        pad = lambda t: torch.cat([t, t[:, :1]], dim=1).contiguous()
        lq_o, cent_o, g_o, b_o = pad(lq), pad(r["centroids"]), pad(r["gamma"]), pad(r["beta"])
        out_o = torch.empty_like(lq_o)
        ws_o = torch.empty(binding.cat_fit_workspace_bytes(N, D + 1, K, dtc), dtype=torch.uint8, device="cuda")
        t_as = _events(lambda: cat_assign(lq_o, cent_o, workspace=ws_o), 5, torch)
        t_ap = _events(lambda: cat_apply(lq_o, cent_o, g_o, b_o, out=out_o, workspace=ws_o), 5, torch)
        binding.debug_apply_kernel(1)  # the same calls on the LDS streaming kernel (the shapes without a row-tile instance)
        try:
            t_as_lds = _events(lambda: cat_assign(lq_o, cent_o, workspace=ws_o), 5, torch)
            t_ap_lds = _events(lambda: cat_apply(lq_o, cent_o, g_o, b_o, out=out_o, workspace=ws_o), 5, torch)
        finally:
            binding.debug_apply_kernel(0)
        t_as0 = _events(lambda: cat_assign(lq, r["centroids"], workspace=ws_fit), 5, torch)
        # the whole fit of those rows: its Lloyd loop runs on a zero-padded copy (the default), or on the LDS kernel
        fp_o = pad(fp)
        fit_o = lambda: cat_fit(lq_o, fp_o, K, iters, seed=w["seed"], workspace=ws_o)
        t_fit_pad = _events(fit_o, 3, torch)
        binding.debug_padded_fit(False)
        try:
            t_fit_lds = _events(fit_o, 3, torch)
        finally:
            binding.debug_padded_fit(True)
        detail.update(stream_shape=f"N={N} D={D + 1} K={K}", stream_assign_us=1e3 * t_as,
                      stream_assign_GBps=N * (D + 1) * esize / t_as / 1e6, stream_apply_us=1e3 * t_ap,
                      stream_apply_GBps=(2 * N * (D + 1) * esize + 4 * N) / t_ap / 1e6,
                      aligned_assign_us=1e3 * t_as0, stream_shape_fit_ms=t_fit_pad, stream_shape_fit_lds_kernel_ms=t_fit_lds,
                      stream_assign_lds_kernel_us=1e3 * t_as_lds, stream_apply_lds_kernel_us=1e3 * t_ap_lds)
        del lq_o, out_o, ws_o, fp_o

    # context: plain device copy of the same matrix, and what a kernel that only streams it reaches (one read; a read and a write)
    t_copy = _events(lambda: out.copy_(lq), 5, torch)
    detail["device_copy_GBps"] = 2 * N * D * esize / t_copy / 1e6
    if (N * D * esize) % 16 == 0:
        t_rd = _events(lambda: binding.stream_probe(lq), 5, torch)
        t_cp = _events(lambda: binding.stream_probe(lq, out), 5, torch)
        detail.update(stream_read_GBps=N * D * esize / t_rd / 1e6, stream_read_frac_hbm=N * D * esize / t_rd / 1e6 / HBM_PEAK_GBPS,
                      stream_copy_GBps=2 * N * D * esize / t_cp / 1e6, stream_copy_frac_hbm=2 * N * D * esize / t_cp / 1e6 / HBM_PEAK_GBPS)
        # beside each kernel's fraction of the peak: the fraction a kernel that only streams the same bytes reaches
        if roof is not None and roof is not apply_roof:
            roof["stream_probe_frac"] = detail["stream_read_frac_hbm"]
        apply_roof["stream_probe_frac"] = detail["stream_copy_frac_hbm"]

    # ---- the oracle on the host cores, bounded sample ----
    cpu = None
    if not args.no_cpu and cpu_budget_s > 0:
        import oracle
        probe = min(N, max(K, 4096))
        t = time.perf_counter()
        if fit_kind:
            oracle.fit(w["lq"][:probe], w["fp"][:probe], K, 1, seed=1)
        else:
            oracle.apply(w["lq"][:probe], w["centroids"], w["gamma"], w["beta"], 1.0)
        per_row_pass = (time.perf_counter() - t) / (probe * (3 if fit_kind else 1))
        budget = float(cpu_budget_s)  # seconds of oracle time
        if fit_kind:
            # passes of a fit: iters + 1 assignments, iters updates (cheap), 2 for the affine fit
            it_s = iters if per_row_pass * N * (iters + 3) <= budget else max(1, int(budget / (per_row_pass * N)) - 3)
            rows_s = N if per_row_pass * N * (it_s + 3) <= 1.5 * budget else max(K, int(budget / (per_row_pass * (it_s + 3))))
            t = time.perf_counter()
            oracle.fit(w["lq"][:rows_s], w["fp"][:rows_s], K, it_s, seed=w["seed"])
            sec = time.perf_counter() - t
            cpu = dict(value=rows_s * it_s / sec, unit="rows/s", cores=oracle.threads(), kind="oracle",
                       sample=f"oracle.fit on {'all' if rows_s == N else 'the first'} {rows_s} rows of {w['name']}, {it_s} Lloyd "
                              f"iterations + final assign + affine fit, {sec:.1f} s; rows x iterations / whole time")
        else:
            rows_s = int(min(N, max(K, budget / max(per_row_pass, 1e-12))))
            t = time.perf_counter()
            oracle.apply(w["lq"][:rows_s], w["centroids"], w["gamma"], w["beta"], 1.0)
            sec = time.perf_counter() - t
            cpu = dict(value=rows_s * D * esize * 2 / sec / 1e9, unit="GB/s", cores=oracle.threads(), kind="oracle",
                       sample=f"oracle.apply on the first {rows_s} rows of {w['name']}, {sec:.1f} s; bytes read + written / time")

    return {
        "metric": metric, "value": value, "unit": unit, "ms_per_step": ms_per_step,
        "dtype": "f32" if dt == "f32" else "bf16",
        "config": {"workload": f"{w['name']}: N={N} D={D} K={K} {dt} iters={iters}", "N": N, "D": D, "K": K,
                   "iters": iters, "step": "cat_fit + cat_apply" if fit_kind else "cat_apply"},
        "roofline": roof, "apply_roofline": apply_roof,
        "lloyd_iter_frac_hbm": detail.get("lloyd_iter_frac_hbm"), "cpu_baseline": cpu, "detail": detail,
    }


HEADLINE = "cfg3"  # the largest fitting workload: 1 GiB of rows like cfg4, and the most rows (the metric counts rows)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="all", choices=["all", "cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg2u"])
    ap.add_argument("--rows", type=int, default=None, help="override N (debugging; the result is then not the named workload)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--hot-path-only", action="store_true",
                    help="only cat_fit and cat_apply: none of the rows beside them (bound-based fit, low-precision inference, "
                         "PCA, sweeps, seeding, grid of cluster counts); the profile commands use it so that every launch of a "
                         "kernel in the trace belongs to the two calls")
    ap.add_argument("--no-seeding", action="store_true",
                    help="skip the timing of the D^2-weighted seeding (detail.kmeanspp_*; cfg2 only)")
    ap.add_argument("--alpha-grid", type=int, default=10,
                    help="also time one pass that evaluates the fitted transformation at this many blending coefficients "
                         "(1/n .. 1): Top-1 agreement with the FP rows and squared error; reported under detail.alpha_*; "
                         "0 skips it, at most 16 (cfg2, or the workload named with --workload)")
    ap.add_argument("--pca-dim", type=int, default=50,
                    help="also time the PCA front-end (fit, projection, labelled affine map) with this many "
                         "components; reported under detail.pca_*; 0 skips it (cfg2, or the workload named with --workload)")
    args = ap.parse_args()
    if args.hot_path_only:
        args.no_seeding, args.pca_dim, args.alpha_grid = True, 0, 0
    if args.gpus != 1:
        sys.exit("bench.py: this library is single-GPU; run with --gpus 1 (rows shard trivially: one all-reduce of K x D sums per iteration)")

    import numpy as np
    import torch

    from paper_2509_26277_amd import binding

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    binding.load_library()  # no fallback: fails here if the HIP library is missing

    if args.workload != "all":
        top = _run_workload(args.workload, args, torch, np, 20.0, extras=True)
        configs = None
    else:
        # the oracle's time is shared out: most of it to the headline workload, a few seconds to each of the others
        per = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg2u"):
            per[name] = _run_workload(name, args, torch, np, 12.0 if name == HEADLINE else 4.0, extras=(name == "cfg2"))
            torch.cuda.empty_cache()
        top = per[HEADLINE]
        configs = [dict(name=k, **{f: v[f] for f in ("metric", "value", "unit", "ms_per_step", "dtype", "config", "roofline",
                                                     "apply_roofline", "lloyd_iter_frac_hbm", "cpu_baseline", "detail")})
                   for k, v in per.items()]
    line = {
        "metric": top["metric"], "value": top["value"], "unit": top["unit"], "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": top["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": top["dtype"], "data": "synthetic", "config": top["config"],
        "roofline": top["roofline"], "apply_roofline": top["apply_roofline"],
        "lloyd_iter_frac_hbm": top["lloyd_iter_frac_hbm"], "cpu_baseline": top["cpu_baseline"], "detail": top["detail"],
    }
    if configs is not None:
        line["configs"] = configs
    print(json.dumps(line))


if __name__ == "__main__":
    main()
