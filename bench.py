#!/usr/bin/env python3
"""Benchmark of the single-linkage hot path on one MI355X.

A step is one pass of the whole path (half norms, fused MFMA k-NN sweep, Boruvka forest with
cross-component 1-NN connection, edge sort, host dendrogram) over one synthetic workload that is
already resident in HBM.  Prints ONE JSON line:

  value      fused k-NN distance pairs per second = N^2 / (norm kernel + k-NN sweep kernel time),
             kernel times taken with HIP events on the launch stream inside every timed step
  ms_per_step   wall time of the whole step (the end-to-end single-linkage seconds x 1000)
  roofline   the fused k-NN sweep against the fp32 MFMA peak (2*d FLOP per ordered pair); also against
             the rate a register-only fp32 MFMA loop sustains in the same run (empirical_peak)
  roofline_connect / roofline_forest   the connection sweeps (MFMA) and the Boruvka rounds (HBM)
  cpu_baseline  the CPU oracle's brute-force k-NN on a bounded sample of query rows, and its dense Prim +
             dendrogram on the small workload and on a scaled-down copy of this one, next to the GPU
             path's seconds on the same inputs
  pruned     the same workload through the default entry point (tile pruning on), outside the
             timed region: end-to-end seconds, stage times and the share of tile steps multiplied

The timed step multiplies every (query panel, candidate tile) pair, as the paper's method does, so
that pairs/s and the roofline fraction count real multiply-adds only.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X published dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X published dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--rows", type=int, default=None, help="scale the workload to this many rows")
    ap.add_argument("--k", type=int, default=None, help="override the workload's k (kernel studies)")
    ap.add_argument("--knn-only", action="store_true", help="time slhc_knn_graph alone (kernel study)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pruned-leg", action="store_true", help="skip the extra runs with tile pruning")
    ap.add_argument("--no-fp32-leg", action="store_true",
                    help="skip the extra k-NN launches with float32 tile products (roofline_fp32_products)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy three times and exit (reference for HBM counters)")
    ap.add_argument("--loop-study", action="store_true",
                    help="run the panel-loop probe (multiplies with the loop's ingredients added one by one) and exit")
    ap.add_argument("--cpu-sample-rows", type=int, default=None)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (nothing here shards across GPUs; "
              "the path would shard by query rows with one all-gather of the neighbour lists)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2306_16354_amd as slhc
    import slhc_inputs as gen

    if not os.path.exists(slhc.library_path()):
        from paper_2306_16354_amd import build as libbuild
        libbuild.build_library(verbose=False)
    slhc.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": a.numel() * 4, "bytes_written": a.numel() * 4, "repeats": 3}))
        return

    if args.loop_study:
        ws_probe = torch.zeros(1 << 27, dtype=torch.float32, device=dev)        # 512 MB to stream from
        names = ["operands in registers", "+ barrier per chunk, A operands from LDS",
                 "+ next chunk: global loads, LDS stores", "+ filter compares per tile",
                 "as 2, chunk loaded straight into LDS", "as 3, chunk loaded straight into LDS",
                 "as 2, unequal wavefront priorities", "as 3, unequal wavefront priorities",
                 "bf16 multiplies of the split-product sweeps (v_mfma_f32_32x32x16_bf16), operands in registers",
                 "bf16: + barrier per chunk of 24 multiplies, hi and lo fragments from LDS",
                 "bf16: + next chunk: global loads, LDS stores", "bf16: + filter compares per tile"]
        out_rows = []
        for rep in range(2):                                                    # second pass reported
            out_rows = [{"steps": st, "what": names[st], "tflops": slhc.probe_panel_loop(st, ws_probe)} for st in range(12)]
        for r in out_rows:
            r["frac_of_peak"] = r["tflops"] / (PEAK_BF16_MFMA_TFLOPS if r["steps"] >= 8 else PEAK_FP32_MFMA_TFLOPS)
        print(json.dumps({"loop_study": out_rows, "peak": PEAK_FP32_MFMA_TFLOPS, "peak_bf16": PEAK_BF16_MFMA_TFLOPS}))
        return

    t0 = time.time()
    X, _, k = gen.make(args.workload, n=args.rows)
    N, d = X.shape
    if args.k is not None:
        k = args.k
    gen_s = time.time() - t0
    Xd = torch.from_numpy(X).to(dev)
    torch.cuda.synchronize()

    ws = torch.empty(slhc.slhc_workspace_bytes(N, d, k), dtype=torch.uint8, device=dev)
    out = None
    knn_out = None

    def step():
        nonlocal out, knn_out
        if args.knn_only:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            knn_out = slhc.knn_graph(Xd, k, out=knn_out, workspace=ws)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            return dict(ms_knn_kernel=ms, ms_norm_kernel=0.0)
        out = slhc.slhc(Xd, k, workspace=ws, out=out, prune=False)
        return out["stats"]

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    stats = []
    for _ in range(args.steps):
        stats.append(step())
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_begin) * 1e3 / max(1, args.steps)

    def mean(name):
        return float(np.mean([s[name] for s in stats]))

    empirical_tflops = slhc.probe_fp32_mfma(dev)       # register-only MFMA loop, same process, right after the steps
    empirical_bf16_tflops = slhc.probe_bf16_mfma(dev)  # the same for v_mfma_f32_32x32x16_bf16

    # Which products the timed sweeps formed: float32 on the fp32 MFMA, or (64 to 128 features, the library's
    # default) split bfloat16 halves hi*hi + hi*lo + lo*hi on the bf16 MFMA.  Either way every pair that can
    # enter a list is re-evaluated in float32, so the outputs are the same bits.
    split = (not args.knn_only and bool(stats[-1].get("split_products", 0))) or \
            (args.knn_only and ((d % 32 == 0 and 64 <= d <= 128) or (d > 128 and d % 4 == 0)))
    peak_tflops = PEAK_BF16_MFMA_TFLOPS if split else PEAK_FP32_MFMA_TFLOPS
    # the float32-product variant of the same sweep, once, outside the timed region (the kernel earlier
    # reports quote)
    fp32_ms = None
    leg_errors = {}            # a failing side leg is reported in the line; it never costs the main measurement
    if split and not args.no_fp32_leg:
        try:
            for rep_ in range(2):                                   # second pass reported
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                knn_out = slhc.knn_graph(Xd, k, out=knn_out, workspace=ws, fp32_filter=True)
                e1.record()
                torch.cuda.synchronize()
                fp32_ms = e0.elapsed_time(e1)
        except Exception as exc:                                    # noqa: BLE001
            leg_errors["fp32_products"] = repr(exc)
            fp32_ms = None

    knn_kernel_ms = mean("ms_knn_kernel")
    knn_ms = knn_kernel_ms + mean("ms_norm_kernel")
    pairs = float(N) * float(N)
    value = pairs / (knn_ms * 1e-3)
    flops = 2.0 * d * pairs
    achieved_tflops = flops / (knn_kernel_ms * 1e-3) / 1e12

    line = {
        "metric": "fused kNN distance pairs/s (+ % FP32-MFMA peak; end-to-end SLHC seconds in slhc_seconds)",
        "value": value,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 (tile products from split bf16 halves on the bf16 MFMA, accumulated in f32; every listed pair "
                 "re-evaluated in f32)" if split else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}: N={N} d={d} k={k} squared-L2 "
                        + ("fused k-NN graph only" if args.knn_only else
                           "k-NN graph + Boruvka/connect MST + sort + dendrogram"),
            "step": "slhc_knn_graph" if args.knn_only else "slhc_slhc (whole hot path)",
            "N": N, "d": d, "k": k,
        },
        "slhc_seconds": None if args.knn_only else ms_per_step / 1e3,
        "pct_fp32_mfma_peak": None if split else 100.0 * achieved_tflops / PEAK_FP32_MFMA_TFLOPS,
        "roofline": {
            "kernel": "sweep_kernel (fused distance tile + filter + top-k)" +
                      (", products from split bf16 halves" if split else ""),
            "bound": "mfma",
            "achieved": achieved_tflops,
            "peak": peak_tflops,
            "unit": "TFLOP/s",
            "frac": achieved_tflops / peak_tflops,
            "traffic": None,
            "launch_ms": knn_kernel_ms,
            "algorithmic_flop_per_launch": flops,
            "executed_mfma_flop_per_launch": 3.0 * flops if split else flops,
            "frac_executed": (3.0 if split else 1.0) * achieved_tflops / peak_tflops,
            "note": ("achieved counts the algorithmic 2 d N^2 against the bf16 MFMA peak; the kernel executes three "
                     "bf16 products per multiply-add (frac_executed) and is bound by LDS operand reads, the "
                     "candidate stream and the exact re-evaluation of the pairs that pass, not by the MFMA pipe")
                    if split else "",
            "empirical_peak": empirical_bf16_tflops if split else empirical_tflops,
            "frac_of_empirical_peak": achieved_tflops / (empirical_bf16_tflops if split else empirical_tflops),
            "frac_executed_of_empirical_peak": (3.0 * achieved_tflops / empirical_bf16_tflops) if split
                                               else achieved_tflops / empirical_tflops,
            "empirical_peak_note": "TFLOP/s of a register-only loop of the sweep's own multiply ("
                                   + ("v_mfma_f32_32x32x16_bf16" if split else "v_mfma_f32_32x32x2_f32") +
                                   ", 4 accumulator blocks per wavefront, 8 wavefronts per CU) measured in this run: "
                                   "what the chip sustains at the clocks it holds under MFMA load",
            "empirical_peak_fp32_mfma": empirical_tflops,
        },
        "input_generation_s": gen_s,
    }
    if fp32_ms is not None:
        ft = flops / (fp32_ms * 1e-3) / 1e12
        line["roofline_fp32_products"] = {
            "kernel": "sweep_kernel with float32 products (SLHC_FP32_FILTER): norms + sweep, one launch outside the timed region",
            "bound": "mfma", "achieved": ft, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": ft / PEAK_FP32_MFMA_TFLOPS, "launch_ms": fp32_ms, "pairs_per_s": pairs / (fp32_ms * 1e-3),
            "frac_of_empirical_peak": ft / empirical_tflops}
        # the metric's "% FP32-MFMA peak" belongs to the sweep that multiplies on the fp32 MFMA
        line["pct_fp32_mfma_peak"] = 100.0 * ft / PEAK_FP32_MFMA_TFLOPS
        line["pct_fp32_mfma_peak_note"] = ("of the k-NN sweep with float32 tile products (roofline_fp32_products); the timed "
                                           "default forms its products from split bf16 halves and is priced in `roofline`")
    # HBM traffic is not measurable from inside the run; it comes from the committed rocprofv3 counter runs
    # of this same workload (profiles/traffic.json: one entry per kernel, keyed by workload and kernel name,
    # FETCH_SIZE + WRITE_SIZE scaled by what the same counters read for a plain copy of known size)
    traffic_table = {}
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            for ent in json.load(f).get("entries", []):
                if ent.get("workload") == args.workload and ent["N"] == N and ent["d"] == d and ent["k"] == k:
                    traffic_table[ent["role"]] = ent
    except (OSError, ValueError, KeyError):
        pass

    def attach_traffic(obj, role):
        ent = traffic_table.get(role)
        if ent:
            obj["traffic"] = ent["fetch_bytes"] + ent["write_bytes"]
            obj["traffic_unit"] = ent["per"]
            obj["traffic_kernel"] = ent["kernel"]

    attach_traffic(line["roofline"], "knn_sweep_split" if split else "knn_sweep")
    if "roofline_fp32_products" in line:
        attach_traffic(line["roofline_fp32_products"], "knn_sweep")
    if not args.knn_only:
        line["stages_ms"] = {n: mean(n) for n in ("ms_knn", "ms_norm_kernel", "ms_knn_kernel", "ms_boruvka",
                                                  "ms_connect", "ms_connect_kernels", "ms_sort",
                                                  "ms_dendrogram", "ms_total")}
        s0 = stats[-1]
        line["counters"] = {n: int(s0[n]) for n in ("boruvka_rounds", "connect_rounds", "components_after_knn",
                                                    "knn_filter_survivors", "connect_query_rows",
                                                    "connect_filter_survivors")}
        cq = float(s0["connect_query_rows"])
        if cq > 0 and mean("ms_connect_kernels") > 0:
            ct = 2.0 * d * cq * N / (mean("ms_connect_kernels") * 1e-3) / 1e12
            line["roofline_connect"] = {"kernel": "sweep_kernel (cross-component 1-NN)", "bound": "mfma",
                                        "achieved": ct, "peak": peak_tflops, "unit": "TFLOP/s",
                                        "frac": ct / peak_tflops, "traffic": None,
                                        "frac_executed": (3.0 if split else 1.0) * ct / peak_tflops}
            attach_traffic(line["roofline_connect"], "connect_sweeps_split" if split else "connect_sweeps")

    if not args.knn_only:
        # graph / Boruvka stage against the HBM roofline: per round every list entry (4 B index) and the
        # colour it points to (4 B gather) may be read once, one distance per vertex, and ~40 B of
        # per-vertex state are rewritten; ms_boruvka is host time including the per-round readbacks
        rounds = float(stats[-1]["boruvka_rounds"])
        forest_bytes = rounds * N * (8.0 * k + 44.0)
        fms = mean("ms_boruvka")
        if fms > 0:
            gbs = forest_bytes / (fms * 1e-3) / 1e9
            line["roofline_forest"] = {"kernel": "Boruvka rounds (scan lists, classify, select, commit, relabel)",
                                       "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                       "frac": gbs / PEAK_HBM_GBS, "traffic": None,
                                       "algorithmic_bytes": forest_bytes, "ms": fms, "rounds": int(rounds)}
            attach_traffic(line["roofline_forest"], "forest_rounds")

    pr = None
    if not args.knn_only and not args.no_pruned_leg:
        # the default entry point (slhc_slhc: tile pruning from 24 576 rows on) on the same input, outside the
        # timed region
        try:
            for _ in range(max(1, args.warmup)):
                pr = slhc.slhc(Xd, k, workspace=ws, out=out, prune=None)
            torch.cuda.synchronize()
            p0 = time.perf_counter()
            reps = max(1, args.steps)
            for _ in range(reps):
                pr = slhc.slhc(Xd, k, workspace=ws, out=out, prune=None)
            torch.cuda.synchronize()
            p_ms = (time.perf_counter() - p0) * 1e3 / reps
        except Exception as exc:                                    # noqa: BLE001
            leg_errors["default_entry_point"] = repr(exc)
            pr = None
    if pr is not None:
        line["default_entry_point_seconds"] = p_ms / 1e3
        ps = pr["stats"]
        if ps["pruned"]:
            tiles_all = ((N + 127) // 128) ** 2
            knn_eff_ms = ps["ms_norm_kernel"] + ps["ms_order"] + ps["ms_knn_kernel"]
            line["pruned"] = {
                "slhc_seconds": p_ms / 1e3,
                "effective_knn_pairs_per_s": pairs / (knn_eff_ms * 1e-3),
                "note": "same outputs bit for bit; effective pairs/s = N^2 / (norms + row order + pruned sweep), "
                        "not comparable with the roofline (skipped tiles are not multiplied)",
                "knn_tile_steps": int(ps["knn_tile_steps"]),
                "knn_tile_steps_unpruned": int(tiles_all),
                "connect_tile_steps": int(ps["connect_tile_steps"]),
                "order_pivots": int(ps["order_pivots"]),
                "order_padded_rows": int(ps["order_padded_rows"]),
                "mfma_tflops_on_multiplied_tiles":
                    2.0 * d * 128.0 * 128.0 * ps["knn_tile_steps"] / (ps["ms_knn_kernel"] * 1e-3) / 1e12,
                "stages_ms": {n: float(ps[n]) for n in ("ms_norm_kernel", "ms_order", "ms_knn_kernel", "ms_boruvka",
                                                        "ms_connect", "ms_connect_kernels", "ms_sort",
                                                        "ms_dendrogram", "ms_total")},
            }
            for role in ("pruned_knn_sweep", "pruned_connect_sweeps"):
                ent = traffic_table.get(role)
                if ent:
                    line["pruned"].setdefault("traffic", {})[role] = {
                        "bytes": ent["fetch_bytes"] + ent["write_bytes"], "per": ent["per"], "kernel": ent["kernel"]}

    if not args.no_cpu_baseline:
        import oracle                                     # cpu_baseline leg only
        oracle.build()
        rng = np.random.default_rng(12345)
        m = args.cpu_sample_rows
        if m is None:                                     # size the sample for about 12 s of CPU work
            probe = rng.choice(N, size=min(N, 64), replace=False).astype(np.int64)
            p0 = time.perf_counter()
            oracle.knn_rows(X, probe, k)
            per_row = (time.perf_counter() - p0) / probe.size
            m = int(max(64, min(N, 12.0 / max(per_row, 1e-9))))
        rows = rng.choice(N, size=min(m, N), replace=False).astype(np.int64)
        c0 = time.perf_counter()
        oracle.knn_rows(X, rows, k)
        c1 = time.perf_counter()
        line["cpu_baseline"] = {
            "value": rows.size * float(N) / (c1 - c0),
            "unit": "pairs/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"fp64 brute-force k-NN of {rows.size} seeded query rows against all {N} rows "
                      f"of the same workload ({c1 - c0:.1f} s)",
        }
        if not args.knn_only:
            # the oracle's whole tree (dense Prim + sort + union-find dendrogram) beside the GPU path on the
            # same inputs: the small workload in full, and this workload scaled down to what Prim
            # finishes in a few seconds (its cost grows with N^2 d)
            tree = []
            scaled_rows = int(min(N, max(2000, (2.5e11 / d) ** 0.5)))
            for wname, rows_ in (("c1", None), (args.workload, scaled_rows)):
                Xs, _, ks = gen.make(wname, n=rows_)
                if args.k is not None and wname == args.workload:
                    ks = min(args.k, Xs.shape[0] - 1)
                Xsd = torch.from_numpy(Xs).to(dev)
                slhc.slhc(Xsd, ks)
                torch.cuda.synchronize()
                g0 = time.perf_counter()
                slhc.slhc(Xsd, ks)
                torch.cuda.synchronize()
                g1 = time.perf_counter()
                o0 = time.perf_counter()
                oracle.slhc(Xs)
                o1 = time.perf_counter()
                tree.append({"workload": f"{wname}: N={Xs.shape[0]} d={Xs.shape[1]} k={ks}",
                             "oracle_seconds": o1 - o0, "gpu_slhc_seconds": g1 - g0})
            line["cpu_baseline"]["tree"] = tree
            line["cpu_baseline"]["tree_note"] = ("oracle = dense Prim + sort + union-find on the host cores; the full "
                                                 "workload would cost the oracle about (N / scaled N)^2 times its scaled time")
    if leg_errors:
        line["side_leg_errors"] = leg_errors
    print(json.dumps(line))


if __name__ == "__main__":
    main()
