#!/usr/bin/env python3
"""Benchmark of the quantised-histogram tree-construction path on one MI355X.

Headline workload: the 115,000,000 x 13 "large tabular" configuration (8-bit packing, 256 bins, depth 8,
lambda 1, logistic objective) on seeded synthetic data of that shape.  One step is one boosting iteration
of the whole hot path with all inputs resident in HBM: gradients (Eq. 1-2) -> grow one tree (root
histogram, per level: split evaluation, row partition, histograms of the smaller children, sibling
subtraction) -> margin update by prediction.  Quantisation and compression run once before the loop, as in
the paper's pipeline, and are reported separately.

Prints ONE JSON line.  `value` = rows*features per second of a whole step on the headline workload.
Every `roofline*` object is stated on the bytes the METHOD needs (`algorithmic_bytes_per_launch`: a
histogram rows_built * (F*bits/8 + 8 [+ 4 with a row id]), a repartition 4 + 4 + bits/8 per row and level -- a pass
that leaves the rows where they are counts the symbol alone, the move that later puts them in order over L levels of
splits at once counts the id traffic of those L levels, 8 L + bits/8 per row), divided
by the launch time measured with HIP events on the library's stream inside the timed region; the bytes this
library's design moves (whole records read and written) are given beside it as `design_bytes_per_launch`.
`roofline` is the kernel the step spends most time in, `roofline_hist_root` the root-node launch (the
figure the 60 %-of-peak target names), `hist_depth4` the launches that build the depth-4 nodes,
`stream_read_ceiling_GBps` what a kernel that only reads gets from HBM in this very run, `workloads` the
other four configurations at full size, `cpu_baseline` the CPU oracle's tree on a bounded row sample.
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

HBM_PEAK_GBPS = 8000.0


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def load_workload(cfg, rows, cache_dir):
    import numpy as np
    import synth
    if cache_dir:
        os.makedirs(cache_dir, exist_ok=True)
        fx = os.path.join(cache_dir, f"c{cfg}_{rows}_X.npy")
        fy = os.path.join(cache_dir, f"c{cfg}_{rows}_y.npy")
        if os.path.exists(fx) and os.path.exists(fy):
            try:
                d = synth.make(cfg, 1)
                d["X"], d["y"] = np.load(fx), np.load(fy)
                if d["X"].ndim == 2 and d["y"].shape == (d["X"].shape[0],):
                    return d
            except (ValueError, OSError):
                pass   # not a cache this version wrote: make the workload again
    d = synth.make(cfg, rows)
    if cache_dir and d.get("y") is not None:   # (a workload with given gradient pairs has more than X and y: not cached)
        np.save(fx, d["X"])
        np.save(fy, d["y"])
    return d


def committed_traffic(cfg):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this command and committed
    under profiles/ (the file gives the commands): NOT measured in this run.  None when no summary exists."""
    path = os.path.join(ROOT, "profiles", f"hist_kernel_c{cfg}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    out = {}
    for line in open(path):
        if line.startswith("@"):
            k, v = line[1:].split("=", 1)
            out[k.strip()] = float(v)
    return out or None


def cpu_baseline(d, sample_rows):
    """The oracle's tree (its own quantisation, fp64 histograms, exhaustive split search) on the first
    `sample_rows` rows, timed on the host cores."""
    import numpy as np
    import oracle
    p = d["params"]
    X = np.ascontiguousarray(d["X"][:sample_rows])
    y = None if d["y"] is None else d["y"][:sample_rows]
    n, F = X.shape
    t0 = time.time()
    cuts, nb = oracle.cuts(X, p["max_bins"])
    sym, missing, _ = oracle.bin_matrix(X, cuts, nb)
    t_q = time.time() - t0
    gp = (np.stack([d["g"][:sample_rows], d["h"][:sample_rows]], 1) if p["objective"] == "given"
          else oracle.gradients(p["objective"], np.zeros(n, np.float32), y))
    t0 = time.time()
    oracle.hist(sym, p["max_bins"], missing, None, gp)
    t_hist = time.time() - t0
    t0 = time.time()
    tree, _, _ = oracle.grow_tree(sym, nb, cuts, missing, gp, max_depth=p["max_depth"], max_bins=p["max_bins"],
                                  lam=p["lam"], gamma=p["gamma"], min_child_weight=p["min_child_weight"])
    t_tree = time.time() - t0
    threads = min(F, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    return {"value": n * F / t_tree, "unit": "rows*features/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n} rows of the workload: one depth-{p['max_depth']} tree in {t_tree:.2f} s "
                      f"(root histogram alone {t_hist:.3f} s = {n * F / t_hist:.3g} rows*features/s; "
                      f"quantisation {t_q:.2f} s not included)",
            "seconds_per_tree": t_tree, "hist_root_rows_features_per_s": n * F / t_hist}


def roof(prof, classes, kernel):
    ms_ = sum(prof[c]["ms"] for c in classes)
    alg = sum(prof[c]["alg_bytes"] for c in classes)
    des = sum(prof[c]["bytes"] for c in classes)
    launches = sum(prof[c]["launches"] for c in classes)
    if ms_ <= 0 or launches == 0:
        return None
    ach = alg / (ms_ * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBPS,
            "traffic": None, "traffic_source": None, "traffic_ratio": None, "kernel": kernel, "launches": launches,
            "avg_launch_ms": ms_ / launches, "algorithmic_bytes_per_launch": alg / launches,
            "design_bytes_per_launch": des / launches, "design_frac": des / (ms_ * 1e-3) / 1e9 / HBM_PEAK_GBPS}


def run_workload(g, a, cfg, rows, steps, warmup, layout="dense", policy="depthwise", max_leaves_arg=0, headline=False):
    import numpy as np
    import torch
    t0 = time.time()
    d = load_workload(cfg, rows, a.data_cache)
    p = d["params"]
    X = d["X"]
    n, F = X.shape
    log(f"workload C{cfg} ({layout}, {policy}): {n} x {F}, generated in {time.time() - t0:.1f} s")
    given = p["objective"] == "given"   # workload 1 carries its own gradient pairs: a step is the tree alone

    ctx = g.Context(0)
    dev = ctx.device
    # ---- one-off preprocessing: quantise + compress (Sec. 2.1, 2.2)
    t0 = time.time()
    import synth
    if cfg == 3:   # the sparse workload enters as CSR
        csr = tuple(torch.from_numpy(v).to(dev) for v in synth.dense_to_csr(X))
        Xd = None
    else:
        Xd = torch.from_numpy(X).to(dev)
    torch.cuda.synchronize()
    t_h2d = time.time() - t0
    t0 = time.time()
    if Xd is None:
        cuts, nb, sym, mv, ms = ctx.quantise(csr=csr, max_bins=p["max_bins"], n=n, F=F)
        del csr
    else:
        cuts, nb, sym, mv, ms = ctx.quantise(Xd, max_bins=p["max_bins"])
    torch.cuda.synchronize()
    t_quant = time.time() - t0
    t0 = time.time()
    packed, bits = ctx.compress(sym, mv)
    torch.cuda.synchronize()
    t_comp = time.time() - t0
    # the same two steps as one call that never stores the symbol matrix (same cuts, same bit stream)
    t0 = time.time()
    if Xd is None:
        csr = tuple(torch.from_numpy(v).to(dev) for v in synth.dense_to_csr(X))
        torch.cuda.synchronize()
        t0 = time.time()
        _, _, packed_1, bits_1, _, _ = ctx.quantise_packed(csr=csr, max_bins=p["max_bins"], n=n, F=F)
        del csr
    else:
        _, _, packed_1, bits_1, _, _ = ctx.quantise_packed(Xd, max_bins=p["max_bins"])
    torch.cuda.synchronize()
    t_fused = time.time() - t0
    if bits_1 != bits or not torch.equal(packed_1, packed):
        raise SystemExit("bench.py: gbt_quantise_packed and gbt_quantise + gbt_compress disagree")
    del packed_1
    sparse = layout == "sparse"
    t_sparse = None
    if sparse:
        t0 = time.time()
        rowptr, ent, nnz = ctx.compress_sparse(sym, p["max_bins"], ms)
        torch.cuda.synchronize()
        t_sparse = time.time() - t0
        log(f"sparse rows: {nnz} present elements ({nnz / (n * F):.1%}), {t_sparse * 1e3:.1f} ms")
    del Xd, sym
    torch.cuda.empty_cache()
    log(f"H2D {t_h2d:.2f} s, quantise {t_quant * 1e3:.1f} ms, compress {t_comp * 1e3:.1f} ms, both in one call "
        f"{t_fused * 1e3:.1f} ms, bits={bits}")

    y = None if given else torch.from_numpy(d["y"]).to(dev)
    margin = torch.zeros(n, dtype=torch.float32, device=dev)
    gp = (torch.from_numpy(np.stack([d["g"], d["h"]], 1)).to(dev) if given
          else torch.empty((n, 2), dtype=torch.float32, device=dev))
    params = g.make_params(max_depth=p["max_depth"], max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"], eta=p["eta"], objective=p["objective"])
    lossguide = policy == "lossguide"
    max_leaves = max_leaves_arg or 2 ** p["max_depth"]
    lg_params = g.make_params(max_depth=64, max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                              min_child_weight=p["min_child_weight"], eta=p["eta"], objective=p["objective"])
    # A one-round workload is ONE tree from margin 0, and every step repeats exactly that: the gradients are taken
    # from a margin that stays zero, and the step's margin update goes to an array of its own (what it holds
    # is never read), so that no reset of the margin sits inside the timed step.
    single_tree = p["rounds"] == 1
    margin_in = torch.zeros_like(margin) if (single_tree and not given) else margin
    eta = p["eta"]
    trees = []

    one_call = not (given or sparse or lossguide)   # gbt_boost_round: the three steps of an iteration in one call

    def step(outputs=False, three_calls=False):
        # outputs: also the final row order and each row's leaf (nothing in the boosting loop reads them)
        if one_call and not outputs and not three_calls:
            trees.append(ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y, margin_in, margin, gp, params))
            return
        if not given:
            ctx.gradients(p["objective"], margin_in, y, out=gp)
        if sparse:
            if lossguide:
                tree, _, _ = ctx.grow_tree_sparse_lossguide(rowptr, ent, n, nnz, F, nb, cuts, gp, lg_params, max_leaves,
                                                            want_rows=outputs, want_leaf=outputs)
            else:
                tree, _, _ = ctx.grow_tree_sparse(rowptr, ent, n, nnz, F, nb, cuts, gp, params, want_rows=outputs,
                                                  want_leaf=outputs)
            ctx.predict_sparse([tree], margin, eta, rowptr, ent, n, F, p["max_bins"])
            trees.append(tree)
            return
        if lossguide:
            tree, _, _ = ctx.grow_tree_lossguide(packed, bits, n, F, ms, nb, cuts, gp, lg_params, max_leaves,
                                                 want_rows=outputs, want_leaf=outputs)
        else:
            tree, _, _ = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp, params, want_rows=outputs,
                                       want_leaf=outputs)
        ctx.predict([tree], margin, eta, packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
        trees.append(tree)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if headline and a.copy_calibration:
        scratch = torch.empty_like(packed)
        scratch.copy_(packed)
        torch.cuda.synchronize()
        log(f"copy calibration: one device copy of {packed.numel() * 4} bytes")
        del scratch
    # ---- the timed region: exactly `steps` steps, the library's HIP events around every launch group
    ctx.profile_enable(True)
    ctx.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_read()
    levels = ctx.last_profile_levels
    ctx.profile_enable(False)
    ms_per_step = dt * 1e3 / steps
    margin_keep = None if single_tree else margin.clone()
    n_trees_timed = len(trees)
    # the same steps without the event records (for information: `value` is from the region above)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_plain = (time.perf_counter() - t0) * 1e3 / steps
    # ... as three calls (gbt_gradients, gbt_grow_tree, gbt_predict) where the step above is gbt_boost_round
    ms_per_step_three = None
    if one_call:
        keep = None if single_tree else margin.clone()
        step(three_calls=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(three_calls=True)
        torch.cuda.synchronize()
        ms_per_step_three = (time.perf_counter() - t0) * 1e3 / steps
        if keep is not None:
            margin.copy_(keep)
    # ... and when the caller also asks for the row order and the leaf of every row
    ms_per_step_outputs = None
    if headline and not a.no_outputs_leg:
        step(outputs=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(outputs=True)
        torch.cuda.synchronize()
        ms_per_step_outputs = (time.perf_counter() - t0) * 1e3 / steps
    del trees[n_trees_timed:]
    if margin_keep is not None:
        margin.copy_(margin_keep)
    log("per-class device ms per step: " + ", ".join(f"{k}={v['ms'] / steps:.3f}" for k, v in prof.items()))
    log(f"nodes per tree: {[t['n_nodes'] for t in trees[-steps:]]}; step {ms_per_step:.3f} ms "
        f"({ms_per_step_plain:.3f} ms without event records)")

    # which kernels the classes of the library's profile stand for on this shape
    path = ctx.grow_tree_path(F, bits, p["max_bins"], track_rows=False)
    root8 = bits == 8 and F <= 16
    hist_kernel = ("hist8_kernel" if root8 else "hist_b8_kernel") if bits == 8 else "hist_bits_kernel"
    node_hist_kernel = "hist_b8_kernel" if bits == 8 else "hist_bits_kernel"
    # path 2, depth-wise: which levels a class covers depends on the depth (see gbt_grow_tree): with depth 8 the
    # rows stay in place at levels 1, 3, 4, 6, 7 and are moved over several levels of splits at levels 2 and 5
    node_kernel = ("part_hist_kernel (partition + one child's histogram in one pass) where rows move at every level; "
                   "hist8_kernel over the built children's records behind a move over several levels"
                   if path == 2 else node_hist_kernel)
    part_kernel = ("move_levels_kernel (rows moved over two or three levels of splits at once)"
                   + ("" if one_call else " + count2_kernel (row counts of the leaves)") if path == 2 and not lossguide else
                   "part_flag_kernel + part_scan_kernel (row counts of the last level)" if path == 2 else
                   ("part_fused_kernel" if (F * bits + 31) // 32 == 4 else "part_staged_kernel") if path == 1 else
                   "part_flag_kernel + part_scan_kernel + part_scatter_kernel (row-id lists)" if path == 3 else
                   "part_flag_kernel + part_scan_kernel + part_move_kernel")
    if sparse:
        hist_kernel = node_kernel = "sparse_hist_kernel"
        part_kernel = "sparse_part_kernel"
    r_root = roof(prof, ["hist_root"], hist_kernel)
    r_node = roof(prof, ["hist_node"], node_kernel)
    r_first = roof(prof, ["hist_first"], "the pass at level 1, from the packed matrix: where the rows stay in place (depth 5, 6, 8, 9, ...) "
                                        "hist8_kernel adding one side of the root's split, else part_hist_first_kernel")
    r_inplace = roof(prof, ["hist_inplace"], "hist_keep_kernel + hist2_kernel (passes over records that stay in place: one and two "
                                            "histograms per workgroup)")
    r_part = roof(prof, ["partition"], part_kernel)
    traffic = None if sparse else committed_traffic(cfg)
    if traffic:
        for obj, key in ((r_root, "hist_root_launch_bytes"), (r_node, "hist_node_launch_avg_bytes"),
                         (r_first, "hist_first_launch_bytes"), (r_inplace, "hist_inplace_launch_avg_bytes"),
                         (r_part, "partition_launch_avg_bytes")):
            if obj and traffic.get(key):
                obj["traffic"] = traffic[key]
                obj["traffic_source"] = f"profiles/hist_kernel_c{cfg}_hbm_traffic.txt (rocprofv3 --pmc, committed; not measured in this run)"
                obj["traffic_ratio"] = traffic[key] / obj["algorithmic_bytes_per_launch"]
    # the top-level roofline is the kernel class the step spends most of its time in
    dominant = max((r for r in (r_root, r_node, r_first, r_inplace, r_part) if r),
                   key=lambda r: r["avg_launch_ms"] * r["launches"], default=None)
    root_ms = prof["hist_root"]["ms"] / max(prof["hist_root"]["launches"], 1)

    def level_obj(k):
        for lv in levels:
            if lv["level"] == k and lv["ms"] > 0:
                ms_ = lv["ms"] / lv["launches"]
                ach = lv["alg_bytes"] / (lv["ms"] * 1e-3) / 1e9
                return {"depth_of_nodes_built": k, "avg_launch_ms": ms_, "launches": lv["launches"],
                        "rows_features_per_s": lv["row_features"] / (lv["ms"] * 1e-3),
                        "algorithmic_bytes_per_launch": lv["alg_bytes"] / lv["launches"],
                        "achieved_GBps": ach, "frac": ach / HBM_PEAK_GBPS}
        return None

    out = {
        "config": {"workload": f"C{cfg}: {n} rows x {F} features, {p['max_bins']} bins, {bits}-bit packing, "
                               f"depth {p['max_depth']}, lambda {p['lam']}, {p['objective']} objective",
                   "rows": n, "features": F, "bits": bits, "max_depth": p["max_depth"],
                   "policy": policy, **({"max_leaves": max_leaves} if lossguide else {}),
                   "layout": layout, **({"present_elements": nnz} if sparse else {})},
        "steps": steps, "ms_per_step": ms_per_step, "value": n * F / (ms_per_step * 1e-3),
        "seconds_per_tree": ms_per_step * 1e-3,
        "ms_per_step_without_event_records": ms_per_step_plain,
        "step_entry_point": "gbt_boost_round" if one_call else "gbt_gradients + gbt_grow_tree* + gbt_predict*",
        **({"ms_per_step_as_three_calls": ms_per_step_three} if ms_per_step_three is not None else {}),
        "device_ms_sum_per_step": sum(v["ms"] for v in prof.values()) / steps,
        "hist_root_ms": root_ms,
        "hist_root_rows_features_per_s": (n * F / (root_ms * 1e-3)) if root_ms > 0 else None,
        "roofline": dominant,
        "roofline_hist_root": r_root,
        "roofline_hist_node": r_node,
        "roofline_hist_first_level": r_first,
        "roofline_hist_in_place": r_inplace,
        "roofline_partition": r_part,
        "hist_by_depth": [level_obj(lv["level"]) for lv in levels],
        "hist_depth4": level_obj(4),
        "grow_tree_path": path,
        "device_ms_per_step": {k: v["ms"] / steps for k, v in prof.items()},
        "preprocess_ms": {"quantise": t_quant * 1e3, "compress": t_comp * 1e3,
                          "quantise_packed_one_call": t_fused * 1e3, "h2d_raw_matrix": t_h2d * 1e3,
                          **({"compress_sparse": t_sparse * 1e3} if sparse else {})},
        "given": given, "lossguide": lossguide, "max_leaves": max_leaves,
    }
    if ms_per_step_outputs is not None:
        out["with_row_order_and_leaf_ids"] = {"ms_per_step": ms_per_step_outputs,
                                              "value": n * F / (ms_per_step_outputs * 1e-3)}
    if headline:
        # what a kernel that only reads gets from HBM here and now: a buffer of 6 GB, many times the 256 MB the
        # memory-side cache holds, so that a repetition finds nothing of the one before (on the 1.5 GB packed matrix
        # the same call reads 6 TB/s, a tenth of it from that cache)
        big = torch.empty(6 * 1024 ** 3 // 4, dtype=torch.int32, device=dev)
        big.fill_(1)
        out["stream_read_ceiling_GBps"] = ctx.measure_stream_read(big, reps=5)
        out["stream_read_ceiling_bytes"] = big.numel() * 4
        del big
        log(f"streaming-read ceiling: {out['stream_read_ceiling_GBps']:.0f} GB/s")
        if not given and not sparse:
            # the root histogram again with gradient pairs of a boosted model (every row its own hessian): the first
            # tree of a logistic model has ONE hessian value for all rows, which the kernel exploits
            m2 = torch.zeros(n, dtype=torch.float32, device=dev)
            ctx.predict([trees[-1]], m2, eta, packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
            gp2 = ctx.gradients(p["objective"], m2, y)
            p1 = g.make_params(max_depth=1, max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                               min_child_weight=p["min_child_weight"])
            ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp2, p1, want_rows=False, want_leaf=False)
            ctx.profile_enable(True)
            ctx.profile_read()
            for _ in range(max(steps, 5)):
                ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp2, p1, want_rows=False, want_leaf=False)
            pr2 = ctx.profile_read()
            ctx.profile_enable(False)
            out["roofline_hist_root_second_tree"] = roof(pr2, ["hist_root"], hist_kernel + " (pairs of the second boosting round: no common hessian)")
            if one_call:
                # ... and the whole step on those pairs: the second round of the same model, repeated (margins in: after
                # one tree; out: an array of its own), so every launch takes its general form
                m3 = torch.empty_like(m2)
                ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y, m2, m3, gp2, params)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y, m2, m3, gp2, params)
                torch.cuda.synchronize()
                out["ms_per_step_second_round"] = (time.perf_counter() - t0) * 1e3 / steps
                log(f"second boosting round (no common hessian): {out['ms_per_step_second_round']:.3f} ms per step")
                del m3
            del m2, gp2
    if a.predict_trees > 0 and not given and headline:
        # Sec. 2.4 with many trees: boost (untimed), then one gbt_predict call over the raw floats
        Xraw = torch.from_numpy(X).to(dev)
        bm = torch.zeros(n, dtype=torch.float32, device=dev)
        many = []
        for _ in range(a.predict_trees):
            ctx.gradients(p["objective"], bm, y, out=gp)
            t_, _, _ = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp, params, want_rows=False, want_leaf=False)
            ctx.predict([t_], bm, eta, packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
            many.append(t_)
        pm = torch.zeros(n, dtype=torch.float32, device=dev)
        ctx.predict(many, pm, eta, X=Xraw)
        same = bool(torch.equal(pm, bm))     # the margins the boosting loop built tree by tree
        ctx.profile_enable(True)
        ctx.profile_read()
        reps = 5
        for _ in range(reps):
            ctx.predict(many, pm, eta, X=Xraw)
        torch.cuda.synchronize()
        pp = ctx.profile_read()["other"]
        ctx.profile_enable(False)
        k_ms = pp["ms"] / max(pp["launches"], 1)
        out["predict_many_trees"] = {
            "trees": len(many), "rows": n, "features": F, "input": "raw fp32 matrix, one pass",
            "kernel_ms": k_ms, "row_trees_per_s": n * len(many) / (k_ms * 1e-3),
            "hbm_GBps": (n * (F * 4 + 8)) / (k_ms * 1e-3) / 1e9,
            "equals_boosting_margins": same}
        del Xraw
    if headline and not a.no_cpu_baseline:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(d, min(a.cpu_sample_rows, n))
        log(f"cpu baseline in {time.time() - t0:.1f} s")
    ctx.close()
    del packed, gp, margin, margin_in, y, d, X
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4, help="headline workload 1..5 (default 4: 115M x 13)")
    ap.add_argument("--rows", type=int, default=None, help="fewer rows than the workload's own size")
    ap.add_argument("--data-cache", default=None, help="directory to keep the generated inputs in")
    ap.add_argument("--cpu-sample-rows", type=int, default=40_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-outputs-leg", action="store_true",
                    help="skip the extra timing of the steps with row order and leaf ids asked for")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the other four configurations (by default each is run at full size: 20 steps for C1 and C2, "
                         "5 for C3, packed and sparse, and C5)")
    ap.add_argument("--policy", choices=["depthwise", "lossguide"], default="depthwise",
                    help="node expansion order (Sec. 2.3); lossguide grows --max-leaves leaves, no depth cap")
    ap.add_argument("--max-leaves", type=int, default=0, help="lossguide: leaf budget (default 2^max_depth)")
    ap.add_argument("--layout", choices=["dense", "sparse"], default="dense",
                    help="sparse: rows keep only their present elements (global bin ids of 16 or 32 bits)")
    ap.add_argument("--predict-trees", type=int, default=0,
                    help="also boost this many rounds (untimed) and time gbt_predict with all those trees at once "
                         "on the raw float matrix (Sec. 2.4); reported as predict_many_trees")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of the packed matrix (a kernel of known size to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings by)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import paper_1806_11248_amd as g

    r = run_workload(g, a, a.config, a.rows, a.steps, a.warmup, layout=a.layout, policy=a.policy,
                     max_leaves_arg=a.max_leaves, headline=True)
    given, lossguide = r.pop("given"), r.pop("lossguide")
    max_leaves = r.pop("max_leaves")
    depth = r["config"]["max_depth"]
    out = {
        "metric": "histogram-tree build throughput: rows*features/s of one boosting step "
                  "(%sone %s tree%s)" % ("" if given else "gradients + ",
                                         ("loss-guided %d-leaf" % max_leaves) if lossguide else ("depth-%d" % depth),
                                         "" if given else " + margin update"),
        "value": r["value"], "unit": "rows*features/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64",
        "dtype_note": "histogram sums are exact 64-bit integers of fixed-point (26/22-bit) roundings of the fp32 "
                      "gradient pairs; split gains fp64",
        "data": "synthetic",
    }
    for k, v in r.items():
        if k not in out and k != "steps":
            out[k] = v
    if not a.no_other_workloads and a.rows is None and a.config == 4 and a.layout == "dense" and a.policy == "depthwise":
        others = []
        for cfg, layout in ((1, "dense"), (2, "dense"), (3, "dense"), (3, "sparse"), (5, "dense")):
            # (the two small workloads take a millisecond per step: more steps, so that one slow step does not decide)
            w = run_workload(g, a, cfg, None, 20 if cfg <= 2 else 5, 3, layout=layout)
            others.append({k: w[k] for k in ("config", "steps", "ms_per_step", "seconds_per_tree", "value",
                                              "ms_per_step_without_event_records", "hist_root_ms",
                                              "hist_root_rows_features_per_s", "roofline_hist_root", "roofline",
                                              "hist_depth4", "grow_tree_path", "device_ms_per_step", "preprocess_ms")})
        out["workloads"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
