#!/usr/bin/env python3
"""Benchmark of the quantized-GBDT hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: quantize
(g, h), root histogram, then for every split partition -> histogram of the smaller
child -> sibling subtraction -> split scan, and the final leaf refit, i.e. one call
of grow_tree.  The (g, h) of step i are those of boosting iteration i of a real
boosting run on the synthetic data (computed before the timed region and kept in
HBM), so the timed trees are exactly the trees of that run.

Prints ONE JSON line.  `value` = rows*features accumulated into histograms per
second of whole-step time.  `roofline` is the histogram kernel (all its launches in
the timed region, timed with HIP events on the library's stream).  `cpu_baseline`
times the CPU oracle on the same inputs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="index into workloads.CONFIGS (default: 10.5M x 28)")
    ap.add_argument("--rows", type=int, default=0, help="override the row count (testing only)")
    ap.add_argument("--bits", type=int, default=3)
    ap.add_argument("--acc-width", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--root-reps", type=int, default=20)
    ap.add_argument("--no-bind", action="store_true",
                    help="do not bind the bin matrix to the context (no feature-major copy for the partitions)")
    ap.add_argument("--root-only", action="store_true",
                    help="only the full-size root-pass histogram build (3 warm-up + --root-reps launches); prints "
                         "the root_pass object alone (used for the per-kernel rocprofv3 summaries)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="counter collection run: 5 root-pass builds, one tree, then three plain 256 MiB copies "
                         "(the last dispatches of the process) that calibrate FETCH_SIZE / WRITE_SIZE; no timing")
    return ap.parse_args()


def root_pass(ctx, torch, bins, g, h, bits_g, bits_h, cfg, args, iteration, N, F, nb, copies=1):
    """Times the histogram build of all rows (quantized (g, h) of one iteration) with HIP events.

    copies = 1: the same matrix and gradients every repetition (a warm figure when they fit the memory-side
    cache).  copies > 1: the repetitions rotate over that many distinct copies of the matrix and of the packed
    gradients, so that a repetition finds nothing of its input in the 256 MB memory-side cache (cold figure)."""
    gh, _ = ctx.quantize_gradients(g, h, bits_g, bits_h, cfg.seed, iteration)
    hist = torch.empty(F * nb, dtype=torch.int64, device=bins.device)
    mats = [(bins, gh)] + [(bins.clone(), gh.clone()) for _ in range(copies - 1)]
    for k in range(3):
        b_, g_ = mats[k % copies]
        ctx.build_histograms(b_, g_, bits_g=bits_g, bits_h=bits_h, acc_width=args.acc_width, hist_out=hist)
    torch.cuda.synchronize()
    ctx.set_profiling(True)
    ctx.read_profile()
    for k in range(args.root_reps):
        b_, g_ = mats[k % copies]
        ctx.build_histograms(b_, g_, bits_g=bits_g, bits_h=bits_h, acc_width=args.acc_width, hist_out=hist)
    root_ms, root_n, root_bytes = ctx.read_profile()
    ctx.set_profiling(False)
    avg_ms = root_ms / max(root_n, 1)
    gbs = root_bytes / max(root_n, 1) / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    return {"avg_launch_us": avg_ms * 1e3, "achieved_GBps": gbs, "frac": gbs / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": root_bytes / max(root_n, 1),
            "rows_x_features_per_s": N * F / (avg_ms * 1e-3) if avg_ms > 0 else 0.0, "reps": root_n,
            "distinct_input_copies": copies,
            "input_bytes_rotated": copies * (bins.numel() * bins.element_size() + gh.numel() * 2)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import workloads
    from paper_2207_09682_amd import Context
    from paper_2207_09682_amd import binding as qb

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    cfg = workloads.CONFIGS[args.config]
    bits_g = args.bits if cfg.loss == "logistic" else cfg.bits_g
    bits_h = args.bits if cfg.loss == "logistic" else cfg.bits_h
    N = args.rows or cfg.n_rows
    t0 = time.time()
    wl = workloads.make_workload(cfg, n_rows=N, device=dev)
    N = wl.n_rows
    F, nb, L = cfg.n_features, cfg.n_bins, cfg.num_leaves
    bins = wl.bins.contiguous()
    # one workspace block, owned here (a torch tensor inside Context): the sections this run uses
    ws_flags = qb.WS_BOOST | (qb.WS_ROW_COPIES if args.no_bind else qb.WS_BIND)
    ctx = Context(N, F, nb, max_leaves=L, workspace_flags=ws_flags)
    K, W = args.steps, args.warmup
    sys.stderr.write(f"[bench] workload {cfg.name}: {N} x {F}, {nb} bins, generated in {time.time() - t0:.1f}s\n")

    # the matrix of all trees of the run: bound once, like binning part of the set-up (no effect for narrow rows)
    bind_ms = None
    if not args.no_bind:
        torch.cuda.synchronize()
        tb = time.perf_counter()
        ctx.bind_bins(bins)
        torch.cuda.synchronize()
        bind_ms = (time.perf_counter() - tb) * 1e3

    if args.pmc_probe:
        g, h = workloads.gradients(wl, torch.zeros(N, device=dev))
        tree = ctx.new_tree()
        ctx.grow_tree(bins, g, h, bits_g, bits_h, cfg.seed, 0, L, cfg.min_data_in_leaf, acc_width=args.acc_width, tree=tree)
        upd = torch.zeros(N, device=dev)
        g, h = workloads.gradients(wl, upd.normal_(0.0, 0.5))  # spread gradients, like a later iteration
        gh, _ = ctx.quantize_gradients(g, h, bits_g, bits_h, cfg.seed, 1)
        hist = torch.empty(F * nb, dtype=torch.int64, device=dev)
        for _ in range(5):
            ctx.build_histograms(bins, gh, bits_g=bits_g, bits_h=bits_h, acc_width=args.acc_width, hist_out=hist)
        torch.cuda.synchronize()
        n_copy = 256 * 1024 * 1024
        src = torch.zeros(n_copy, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "root_pass_algorithmic_bytes": N * (F + 2) + F * nb * 8,
                          "copy_bytes_read": n_copy, "copy_bytes_written": n_copy}))
        return

    if args.root_only:
        g, h = workloads.gradients(wl, torch.zeros(N, device=dev).normal_(0.0, 0.5))
        print(json.dumps({"root_pass": root_pass(ctx, torch, bins, g, h, bits_g, bits_h, cfg, args, 1, N, F, nb)}))
        return

    # ---- set-up (untimed): a real boosting run that records (g, h) of every iteration --------
    score = torch.zeros(N, device=dev)
    gs, hs = [], []
    tree = ctx.new_tree()
    for it in range(W + K):
        g, h = workloads.gradients(wl, score)
        gs.append(g); hs.append(h)
        ctx.grow_tree(bins, g, h, bits_g, bits_h, cfg.seed, it, L, cfg.min_data_in_leaf, acc_width=args.acc_width, tree=tree)
        order = torch.argsort(tree.leaf_begin[: int(tree.n_leaves.item())])
        cnt = tree.leaf_count[order]
        leaf_at_pos = torch.repeat_interleave(order, cnt)
        upd = (cfg.learning_rate * tree.leaf_value[leaf_at_pos]).float()
        score.index_add_(0, tree.row_idx.long(), upd)
    torch.cuda.synchronize()

    # ---- timed region: W warm-up steps, then exactly K steps ---------------------------------
    units = torch.zeros(1, dtype=torch.int64, device=dev)
    stats = []
    for it in range(W):
        ctx.grow_tree(bins, gs[it], hs[it], bits_g, bits_h, cfg.seed, it, L, cfg.min_data_in_leaf,
                      acc_width=args.acc_width, tree=tree)
    torch.cuda.synchronize()
    ctx.set_profiling(True)
    ctx.read_profile()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for it in range(W, W + K):
        ctx.grow_tree(bins, gs[it], hs[it], bits_g, bits_h, cfg.seed, it, L, cfg.min_data_in_leaf,
                      acc_width=args.acc_width, tree=tree)
        units += tree.hist_units
        stats.append(ctx.tree_stats())
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    in_tree_root_ms, in_tree_root_n = ctx.read_profile_roots()
    hist_ms, hist_launches, hist_bytes = ctx.read_profile()
    ctx.set_profiling(False)
    total_units = int(units.item())
    n_leaves_last = int(tree.n_leaves.item())

    # ---- the first tree of a run (every |g| = 1/2, h = 1/4 for the logistic loss: all rows carry the extreme
    # quantized values, the tightest case of the accumulator bounds), which the timed steps above leave out
    # when there is a warm-up step ----
    first_tree = None
    if W > 0:
        ctx.grow_tree(bins, gs[0], hs[0], bits_g, bits_h, cfg.seed, 0, L, cfg.min_data_in_leaf, acc_width=args.acc_width, tree=tree)
        torch.cuda.synchronize()
        f0 = time.perf_counter()
        for _ in range(3):
            ctx.grow_tree(bins, gs[0], hs[0], bits_g, bits_h, cfg.seed, 0, L, cfg.min_data_in_leaf, acc_width=args.acc_width, tree=tree)
        torch.cuda.synchronize()
        first_tree = {"ms_per_tree": (time.perf_counter() - f0) / 3 * 1e3, "repetitions": 3,
                      "leaves": int(tree.n_leaves.item()), "hist_units": int(tree.hist_units.item()),
                      "what": "iteration 0 (scores all zero), timed apart: the timed steps are iterations "
                              f"{W}..{W + K - 1} of the same boosting run"}

    # ---- whole boosting iterations on the device (derivatives + tree + score update) ----
    sc = torch.zeros(N, device=dev)
    label = wl.label.to(dev).float().contiguous()
    gs_rank = wl.extra.get("group_size", 0) if cfg.loss == "lambdarank" else 0
    for it in range(W):
        ctx.boost_iteration(bins, label, sc, bits_g, bits_h, cfg.seed, it, L, cfg.learning_rate,
                            min_data_in_leaf=cfg.min_data_in_leaf, acc_width=args.acc_width, tree=tree, group_size=gs_rank)
    torch.cuda.synchronize()
    b0 = time.perf_counter()
    for it in range(W, W + K):
        ctx.boost_iteration(bins, label, sc, bits_g, bits_h, cfg.seed, it, L, cfg.learning_rate,
                            min_data_in_leaf=cfg.min_data_in_leaf, acc_width=args.acc_width, tree=tree, group_size=gs_rank)
    torch.cuda.synchronize()
    boost = {"ms_per_iteration": (time.perf_counter() - b0) / K * 1e3, "iterations": K,
             "what": f"qgbdt_boost_iteration ({cfg.loss}): loss derivatives + grow_tree + score update, no host arithmetic"}

    # ---- root pass alone (contiguous rows): the kernel at its full-size launch -----------------
    root = root_pass(ctx, torch, bins, gs[W], hs[W], bits_g, bits_h, cfg, args, W, N, F, nb)
    root["what"] = ("back-to-back repetitions over ONE matrix: a warm figure when matrix + gradients "
                    f"({(bins.numel() * bins.element_size() + 2 * N) / 1e6:.0f} MB) fit the 256 MB memory-side cache")
    # the same launch with nothing of its input left in the memory-side cache: rotate over enough distinct copies
    # of matrix + packed gradients that at least 1.2 GB pass between two reads of the same copy
    one = bins.numel() * bins.element_size() + 2 * N
    n_copies = max(2, min(8, -(-1_300_000_000 // one)))
    root_cold = root_pass(ctx, torch, bins, gs[W], hs[W], bits_g, bits_h, cfg, args, W, N, F, nb, copies=n_copies)
    root_cold["what"] = f"repetitions rotate over {n_copies} distinct copies of matrix + packed gradients (cold input)"
    # the root build as it runs inside grow_tree (first histogram launch of every timed tree)
    root_bytes_alg = N * (F * bins.element_size() + 2) + F * nb * 8
    rit_us = in_tree_root_ms / max(in_tree_root_n, 1) * 1e3
    root_in_tree = {"avg_launch_us": rit_us, "launches": in_tree_root_n,
                    "achieved_GBps": root_bytes_alg / (rit_us * 1e-6) / 1e9 if rit_us > 0 else 0.0,
                    "algorithmic_bytes_per_launch": root_bytes_alg,
                    "what": "root build inside grow_tree: HIP events around the first histogram launch "
                            "(kernel + reduce) of every timed tree"}
    root_in_tree["frac"] = root_in_tree["achieved_GBps"] / HBM_PEAK_GBS

    # ---- measured streaming-read ceiling of this machine: a plain 16-byte-load kernel over 1 GiB ------
    probe = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    stream_read_gbps = ctx.measure_stream_read(probe, reps=10)
    del probe
    for r_ in (root, root_cold, root_in_tree):
        r_["frac_of_measured_stream_read"] = r_["achieved_GBps"] / stream_read_gbps if stream_read_gbps > 0 else None

    # ---- CPU oracle on the same inputs -----------------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        bins_h = bins.cpu().numpy()
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        # whole trees of the oracle on the (g, h) of the first timed iterations, until about 10 s are spent
        c_units, c_trees, c_el, c_match = 0, 0, 0.0, True
        c0 = time.perf_counter()
        while c_trees < K and time.perf_counter() - c0 < 10.0:
            it = W + c_trees
            g_h = gs[it].cpu().numpy(); h_h = hs[it].cpu().numpy()
            c1 = time.perf_counter()
            tr = oracle.grow_tree(bins_h, nb, g_h, h_h, bits_g, bits_h, cfg.seed, it, L, cfg.min_data_in_leaf)
            c_el += time.perf_counter() - c1
            c_units += int(tr.hist_units); c_trees += 1
            # the same tree from the library, in the launch configuration that was timed (untimed check)
            ctx.grow_tree(bins, gs[it], hs[it], bits_g, bits_h, cfg.seed, it, L, cfg.min_data_in_leaf,
                          acc_width=args.acc_width, tree=tree)
            ns = int(tree.n_leaves.item()) - 1
            c_match = c_match and ns == tr.n_leaves - 1 \
                and np.array_equal(tree.split_feature[:ns].cpu().numpy(), tr.split_feature[:ns]) \
                and np.array_equal(tree.split_bin[:ns].cpu().numpy(), tr.split_bin[:ns]) \
                and np.array_equal(tree.split_leaf[:ns].cpu().numpy(), tr.split_leaf[:ns]) \
                and np.array_equal(tree.row_idx.cpu().numpy(), tr.row_idx)
        cpu = {"value": c_units / c_el, "unit": "rows*features/s", "cores": threads, "kind": "oracle",
               "sample": f"{c_trees} whole tree(s) of the oracle (quantize, histograms, subtraction, scan, partition, "
                         f"refit) on all {N} rows x {F} features, the (g, h) of timed step(s) 0..{c_trees - 1}, "
                         f"{c_el:.1f} s", "s_per_tree": c_el / c_trees,
               "library_tree_equals_oracle_tree": bool(c_match)}

    # Algorithmic bytes of the timed launches.  The launches also serve speculative builds (nodes expanded ahead of
    # the sequential order that never become part of the tree); `achieved` counts only the builds the sequential
    # algorithm performs (the work unit of `value`): the root and the smaller child of every committed split.
    esz = bins.element_size()
    committed_builds = sum(x[2] for x in stats) + K
    rows_committed = total_units // F
    bytes_committed = K * N * (F * esz + 2) + (rows_committed - K * N) * (F * esz + 2 + 4) + committed_builds * F * nb * 8
    achieved_all = (hist_bytes / hist_launches) / (hist_ms / hist_launches * 1e-3) / 1e9 if hist_launches and hist_ms > 0 else 0.0
    achieved = bytes_committed / (hist_ms * 1e-3) / 1e9 if hist_ms > 0 else 0.0
    # HBM bytes per histogram launch from the rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE scaled by a plain
    # copy; see profiles/): measured offline on this workload, so only reported for it
    traffic, root_traffic = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_cfg3.json")
    if args.config == 2 and not args.rows and args.bits == 3 and os.path.exists(tpath):
        with open(tpath) as fh:
            tj = json.load(fh)
        traffic, root_traffic = tj.get("tree_launch_traffic_bytes"), tj.get("root_pass_traffic_bytes")
    root["traffic"] = root_traffic
    root["traffic_source"] = "rocprofv3 counter runs of another process (profiles/hbm_traffic_cfg3.json), not this run"
    out = {
        "metric": "histogram build rows*features/s over whole trees (quantize+hist+subtract+scan+partition+refit), "
                  f"{bits_g}-bit gradients",
        "value": total_units / elapsed,
        "unit": "rows*features/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": elapsed / K * 1e3,
        "s_per_tree": elapsed / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {N} rows x {F} features, {nb} bins (uint8), {cfg.loss} loss, "
                               f"{bits_g}-bit g / {bits_h}-bit h, {L} leaves/tree, leaf-wise",
                   "acc_width": args.acc_width or "auto", "leaves_last_tree": n_leaves_last,
                   "hist_units_per_tree": total_units / K,
                   "bins_bound": bind_ms is not None, "bind_ms_once": bind_ms,
                   "rows": ("in place: row ids (and, for matrices beyond the caches, the packed gradients) move, the bin rows of the "
                            "smaller children are gathered (the faster of the two layouts for whole trees)") if (bind_ms is not None or F > 64 or F % 4 or F < 16)
                           else "kept in leaf order: every level moves the rows, builds stream contiguous memory"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": "rocprofv3 FETCH_SIZE + WRITE_SIZE runs of another process on this workload "
                                       "(profiles/hbm_traffic_cfg3.json): an offline counter value, bytes per launch "
                                       "of one tree; FETCH_SIZE counts L2 misses, which the memory-side cache may serve",
                     "achieved_incl_speculative_builds": achieved_all,
                     "frac_incl_speculative_builds": achieved_all / HBM_PEAK_GBS,
                     "kernel": "histogram build = hist_*_kernel + hist_reduce_kernel (all launches of the timed trees)",
                     "launches": hist_launches, "avg_launch_us": hist_ms / max(hist_launches, 1) * 1e3,
                     "algorithmic_bytes_per_launch": bytes_committed / max(hist_launches, 1),
                     "algorithmic_bytes_per_launch_incl_speculative_builds": hist_bytes / max(hist_launches, 1),
                     "measured_stream_read_GBps": stream_read_gbps,
                     "measured_stream_read_variant": getattr(ctx, "stream_read_variant", None),
                     # rate of the bytes that actually cross the HBM interface (counter runs): what the gathered
                     # builds are bound by -- a 128-byte line per sparse 28-byte row
                     "offline_traffic_over_this_runs_launch_time_GBps": (traffic / (hist_ms / hist_launches * 1e-3) / 1e9) if (traffic and hist_launches and hist_ms > 0) else None},
        "root_pass": root,
        "root_pass_cold": root_cold,
        "root_pass_in_tree": root_in_tree,
        "hist_time_share": hist_ms / (elapsed * 1e3),
        "growth": {"rounds_per_tree": sum(x[0] for x in stats) / K, "expanded_per_tree": sum(x[1] for x in stats) / K,
                   "committed_per_tree": sum(x[2] for x in stats) / K},
        "boost_iteration": boost,
        "first_tree": first_tree,
        "cpu_baseline": cpu,
        "paper_context": "paper: V100, Higgs 10.5M x 28, 3-bit: 4.74 s histogram time / 500 trees = 9.5 ms per tree "
                         "(another machine; context, not the target)",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
