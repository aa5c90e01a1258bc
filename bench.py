#!/usr/bin/env python3
"""Benchmark of the row-structured hybrid SpMM hot path on one MI355X.

One "step" is one rsh_spmm call: tile kernel + irregular kernel + combine over the
whole matrix, with the plan, B and C already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak
# What a gather of 256-byte rows from a table of 67-537 MB sustained on this part in a microbenchmark
# (8 loads in flight per 16-lane team): the rate a kernel bound by random row fetches can be held to.
GATHER_CEILING_GBPS = 7200.0


ABLATIONS = {
    # Section 4.3.2: the row-length threshold of Algorithm 1 decides what leaves for the residual path
    "thresholds": [dict(tau_nnz=t) for t in (0, 1, 2, 4, 6, 8, 12, 16)] + [dict(min_reuse=m) for m in (0.0, 1.0, 1.25, 1.5, 2.0, 3.0)],
    # Section 4.3.3: identity -> spanning-tree walk -> + 2-opt -> + relocation of isolated rows
    "reorder": [dict(reorder=0), dict(reorder=2), dict(reorder=3), dict(reorder=1)],
    # window height and fragment width (the paper fixes 16 x 8 for its MMA shape)
    "shape": [dict(window_rows=w, tile_k=k) for w in (16, 32, 64) for k in (16, 32)] + [dict(window_rows=w) for w in (128, 256)],
}


def ablation(args, A, N, B_np) -> int:
    """One plan + timed SpMM per setting; everything else at its default."""
    import numpy as np
    import torch
    from paper_2603_08734_amd import Plan

    B = torch.from_numpy(B_np.view(np.int16)).cuda().view(torch.float16)
    C = torch.empty((A.n_rows, N), dtype=torch.float32, device="cuda")
    rows = []
    for setting in ABLATIONS[args.ablation]:
        t0 = time.perf_counter()
        plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **setting)
        plan_s = time.perf_counter() - t0
        st = plan.stats()
        for _ in range(args.warmup):
            plan.spmm(B, C)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            plan.spmm(B, C)
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        rows.append({
            "setting": setting, "ms_per_step": round(ms, 4), "gflops": round(2.0 * A.nnz * N / ms / 1e6, 1),
            "plan_s": round(plan_s, 2), "window_rows": st["window_rows"], "tile_k": st["tile_k"],
            "tau_nnz": st["tau_nnz"], "windows": st["n_windows"], "fragments": st["n_tiles"],
            "nnz_tile_share": round(st["nnz_tile"] / max(1, A.nnz), 4),
            "mean_nnz_per_fragment": round(st["nnz_tile"] / max(1, st["n_tiles"]), 2),
            "mean_nnz_per_window": round(st["nnz_tile"] / max(1, st["n_windows"]), 1),
            "distinct_columns_per_window": round(st["sum_window_cols"] / max(1, st["n_windows"]), 1),
            "objective_given": round(st["reorder_cost_given"], 1), "objective_found": round(st["reorder_cost_found"], 1),
        })
        plan.destroy()
        print("ablation %s %s: %.4f ms" % (args.ablation, setting, ms), file=sys.stderr, flush=True)
    print(json.dumps({"ablation": args.ablation, "config": {"workload": A.meta["name"], "nnz": A.nnz, "N": N},
                      "steps": args.steps, "warmup": args.warmup, "rows": rows}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = the headline R-MAT graph)")
    ap.add_argument("--features", type=int, default=0,
                    help="override the configuration's feature width N (the paper sweeps 64..512); 0 = as configured")
    ap.add_argument("--reorder", type=int, default=-1, help="override the plan's reorder option")
    ap.add_argument("--opt", action="append", default=[], help="plan option override name=value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gcn-epoch", type=int, default=0, metavar="HIDDEN",
                    help="also time one training epoch (forward, backward, gradient step) of the 6-layer GCN of the "
                         "paper's case study with this hidden width on the workload's graph; adds a 'gcn_epoch' object")
    ap.add_argument("--epilogue", action="store_true",
                    help="also time rsh_spmm_f16 (bias + ReLU + binary16 output fused) against rsh_spmm followed by "
                         "the same epilogue as separate elementwise kernels; adds a 'fused_epilogue' object")
    ap.add_argument("--ablation", choices=["thresholds", "reorder", "shape"], default=None,
                    help="instead of the benchmark line: sweep one planning knob on --config and print one JSON "
                         "line with a row per setting (the paper's Sections 4.3.2 and 4.3.3 on synthetic data)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the library's plain copy kernel on 1 GiB (for scaling profiler traffic counters)")
    ap.add_argument("--summarize-profile", metavar="DIR", default=None,
                    help="no benchmark: turn the rocprofv3 output under DIR (sub-directories stats, pmc_fetch, pmc_write, "
                         "pmc_sq of the same bench.py command, each with its .log) into the summary --profile-out")
    ap.add_argument("--profile-out", default=None, help="summary file to write (under profiles/)")
    ap.add_argument("--profile-args", default="", help="the bench.py arguments the profiled command was run with")
    args = ap.parse_args()
    if args.summarize_profile:
        from paper_2603_08734_amd import profiles
        data = profiles.summarize(args.summarize_profile, args.profile_out, args.profile_args)
        print(json.dumps(data))
        return 0
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2603_08734_amd import Plan
    from workloads import dense_B, make_config

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    A, N, dist = make_config(args.config)
    if args.features:
        N = args.features
    B_np = dense_B(A.n_cols, N, dist, seed=1)
    gen_s = time.perf_counter() - t0

    if args.ablation:
        return ablation(args, A, N, B_np)

    opts = {}
    if args.reorder >= 0:
        opts["reorder"] = args.reorder
    for kv in args.opt:
        k, v = kv.split("=")
        opts[k] = float(v) if k in ("alpha", "min_reuse") else int(v)
    t0 = time.perf_counter()
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **opts)
    plan_s = time.perf_counter() - t0
    st = plan.stats()

    B = torch.from_numpy(B_np.view(np.int16)).cuda().view(torch.float16)
    C = torch.empty((A.n_rows, N), dtype=torch.float32, device="cuda")
    for _ in range(args.warmup):
        plan.spmm(B, C)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan.spmm(B, C)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    flops = 2.0 * A.nnz * N
    gflops = flops / (ms_per_step * 1e-3) / 1e9

    if args.calibrate_copy:
        from paper_2603_08734_amd.binding import rsh_copy_probe
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            rsh_copy_probe(src, dst, 1 << 30)
        torch.cuda.synchronize()
        del src, dst

    # per-kernel durations with HIP events on the launch stream
    acc = {"tile": 0.0, "irregular": 0.0, "combine": 0.0}
    n_prof = max(5, min(args.steps, 20))
    for _ in range(n_prof):
        t = plan.spmm_profile(B, C)
        for k in acc:
            acc[k] += t[k]
    kernel_ms = {k: v / n_prof for k, v in acc.items()}
    dominant = max(("tile", "irregular"), key=lambda k: kernel_ms[k])
    # the dense-fragment part runs in the panel kernel for windows of 128 rows and more
    kernel_name = "rsh_irregular_kernel" if dominant == "irregular" else ("rsh_panel_kernel" if st["window_rows"] >= 128 else "rsh_tile_kernel")
    if dominant == "irregular":
        alg_bytes = st["irregular_part_bytes"] + 2 * N * st["cols_irregular"] + 4 * N * st["rows_irregular"]
    else:
        alg_bytes = st["tile_part_bytes"] + 2 * N * st["cols_tile"] + 4 * N * st["rows_tile"]
    achieved = alg_bytes / (kernel_ms[dominant] * 1e-3) / 1e9 if kernel_ms[dominant] > 0 else 0.0
    bytes_min = st["plan_bytes"] + 2 * N * st["cols_all"] + 4 * N * A.n_rows
    # counter traffic per launch: only from a profile summary made for exactly this workload, width,
    # plan options and library build (profiles/*.md); otherwise null
    from paper_2603_08734_amd import build as lib_build, profiles
    measured = profiles.lookup(A.meta["name"], N, opts, kernel_name)
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": measured[0] if measured else None,
                "algorithmic_bytes": int(alg_bytes), "kernel_ms": round(kernel_ms[dominant], 4)}
    if measured and kernel_ms[dominant] > 0:
        # what the memory system moved per launch (counters) over this run's kernel time
        moved = measured[0] / (kernel_ms[dominant] * 1e-3) / 1e9
        roofline["traffic_source"] = "profiles/%s: %s" % (measured[1], measured[2])
        roofline["traffic_GBps"] = round(moved, 1)
        roofline["traffic_frac"] = round(moved / HBM_PEAK_GBPS, 4)
        if dominant == "irregular":
            # a kernel of random 256-byte row fetches: its moved bytes against what such fetches sustain
            roofline["gather_ceiling_GBps"] = GATHER_CEILING_GBPS
            roofline["traffic_over_gather_ceiling"] = round(moved / GATHER_CEILING_GBPS, 4)

    # work the matrix cores are given: every W x K fragment is multiplied out in full, zeros included
    mfma = None
    if kernel_ms["tile"] > 0:
        dense_flops = 2.0 * st["window_rows"] * st["tile_k"] * N * st["n_tiles"]
        tf = dense_flops / (kernel_ms["tile"] * 1e-3) / 1e12
        mfma = {"dense_equivalent_TFLOPs": round(tf, 1), "peak_TFLOPs": 2500.0, "frac": round(tf / 2500.0, 4),
                "useful_share": round(2.0 * st["nnz_tile"] * N / dense_flops, 4)}

    out = {
        "metric": "SpMM GFLOP/s (2*nnz*N/t), N=%d, 1 MI355X" % N, "value": round(gflops, 1), "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16*f16+f32",
        "data": "synthetic",
        "config": {"workload": A.meta["name"], "rows": A.n_rows, "cols": A.n_cols, "nnz": A.nnz, "N": N,
                   "seed": 0, "csr_checksum": A.checksum(), "plan_options": opts},
        "roofline": roofline,
        "library_sources": lib_build.source_digest(),
        "tile_mfma": mfma,
        "hbm_useful_GBps": round(bytes_min / (ms_per_step * 1e-3) / 1e9, 1),
        "bytes_min": int(bytes_min),
        "kernel_ms": {k: round(v, 4) for k, v in kernel_ms.items()},
        "plan": {"build_s": round(plan_s, 3), "stage_ms": {k[3:]: round(st[k], 1) for k in st if k.startswith("ms_")},
                 "windows": st["n_windows"], "tiles": st["n_tiles"], "nnz_tile": st["nnz_tile"],
                 "nnz_irregular": st["nnz_irregular"], "tile_items": st["n_tile_items"],
                 "irregular_waves": st["n_irregular_waves"], "split_rows": st["n_split_rows"],
                 "split_windows": st["n_split_windows"], "plan_bytes": st["plan_bytes"], "csr_bytes": st["csr_bytes"],
                 "mean_nnz_per_tile": round(st["nnz_tile"] / max(1, st["n_tiles"]), 2),
                 "mean_nnz_per_window": round(st["nnz_tile"] / max(1, st["n_windows"]), 1)},
        "gen_s": round(gen_s, 2),
    }

    if args.epilogue:
        def timed(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t0) / args.steps

        bias = torch.from_numpy(np.random.default_rng(2).normal(scale=0.1, size=N).astype(np.float32)).cuda()
        C16 = torch.empty((A.n_rows, N), dtype=torch.float16, device="cuda")
        fused_ms = timed(lambda: plan.spmm_f16(B, C16, bias, True))

        def unfused():
            plan.spmm(B, C)
            torch.relu(C + bias).to(torch.float16)

        unfused_ms = timed(unfused)
        out["fused_epilogue"] = {"op": "binary16(relu(A*B + bias))", "ms_per_step": round(fused_ms, 4),
                                 "separate_kernels_ms_per_step": round(unfused_ms, 4)}
        del C16

    if args.gcn_epoch:
        from paper_2603_08734_amd.gcn import Adjacency, GCNLayer
        assert A.n_rows == A.n_cols, "a GCN needs a square adjacency"
        d, n_layers = args.gcn_epoch, 6
        adj = Adjacency(A.row_ptr, A.col_idx, A.val, A.n_cols, **opts)
        layers = [GCNLayer(adj, d, d) for _ in range(n_layers)]      # A (H W): bias/ReLU/rounding fused
        g = torch.Generator(device="cuda").manual_seed(0)
        X = torch.randn((A.n_cols, d), device="cuda", generator=g).to(torch.float16)
        T = torch.randn((A.n_rows, d), device="cuda", generator=g)
        Ws = [(torch.randn((d, d), device="cuda", generator=g) / d ** 0.5).requires_grad_(True) for _ in range(n_layers)]

        def epoch():
            h = X
            for i, (layer, w) in enumerate(zip(layers, Ws)):
                h = layer(h, w.to(torch.float16), None, i + 1 < n_layers)
            loss = ((h.float() - T) ** 2).sum() / A.n_rows
            loss.backward()
            with torch.no_grad():
                for w in Ws:
                    w -= 1e-3 * w.grad
                    w.grad = None

        for _ in range(3):
            epoch()                      # the first backward pass also builds the plan of the transpose
        torch.cuda.synchronize()
        n_ep = max(3, min(args.steps, 10))
        t0 = time.perf_counter()
        for _ in range(n_ep):
            epoch()
        torch.cuda.synchronize()
        ep_ms = 1e3 * (time.perf_counter() - t0) / n_ep
        Y16 = torch.empty((A.n_rows, d), dtype=torch.float16, device="cuda")
        pf, pb = adj.plan(d), adj.plan(d, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_ep):
            for _ in range(n_layers):
                pf.spmm_f16(X, Y16, None, False)
                pb.spmm_f16(X, Y16, None, False)
        torch.cuda.synchronize()
        sp_ms = 1e3 * (time.perf_counter() - t0) / n_ep
        out["gcn_epoch"] = {"layers": n_layers, "hidden": d, "order": "A (H W)", "ms_per_epoch": round(ep_ms, 3),
                            "sparse_products_ms": round(sp_ms, 3), "epochs_timed": n_ep}
        adj.destroy()

    if not args.no_cpu_baseline:
        # the oracle as it stands, on this machine's host cores, whole matrix, one run
        from oracle import spmm as oracle_spmm
        cores = len(os.sched_getaffinity(0))
        threads = min(cores, 16)
        t0 = time.perf_counter()
        C_ref, S, used = oracle_spmm.spmm(A.row_ptr, A.col_idx, A.val, B_np, threads=threads)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(flops / cpu_s / 1e9, 2), "unit": "GFLOP/s", "cores": used,
                               "kind": "oracle", "sample": "whole matrix, one run, %.2f s" % cpu_s}
        C_host = C.cpu().numpy().astype(np.float64)
        err = np.abs(C_host - C_ref)
        ok = bool(np.all(err <= 1e-4 * S))
        out["parity"] = {"ok": ok, "max_err_over_S": float((err / np.where(S > 0, S, 1.0)).max())}
        del C_ref, S, C_host, err
    print(json.dumps(out), flush=True)
    plan.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
