#!/usr/bin/env python3
"""Benchmark of the arrow SpMM hot path on one MI355X.

One "step" is one whole product Y = A.X = sum_i P_i^T B_i (P_i X) through
``arrow_spmm`` (all levels, all kernels) on the R-MAT scale-23, k = 128 workload
with inputs already resident in HBM.  Prints ONE JSON line.

Timing: W untimed warm-up steps, then K steps between two device synchronisations on the host
clock (``ms_per_step``, the figure ``value`` is computed from); after that the same K steps once
more, each bracketed by HIP events on the launch stream (``per_call_ms``: median, min, mean),
a pass with the library's per-launch events (``launch_ms``), and the bare row-gather yardstick
(``roofline.gather_yardstick``).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--shrink S]

``--op sddmm`` times the sampled dense-dense product S = A .* (U V^T) over the same arrow
layout instead (one step = one ``arrow_sddmm`` call); the default, and the headline, is the product.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E peak


def algorithmic_bytes_sddmm(levels, n, k):
    """Bytes one sampled product must move, per launch and for the whole path: per stored entry
    8 B (row id + value) + 4 B (entry map) read and 4 B of S written; the work-list words; every
    distinct V row a launch references and the U row of every row it handles, read once."""
    row = 4 * k
    per = {}
    for i, L in enumerate(levels):
        per[("rows", i)] = 16 * L["nnz_rows"] + 12 * L["short_rows"] + 4 + row * (L["x_rows_rows"] + L["short_rows"] - L["rows_partials"])
        per[("chunks", i)] = 16 * L["nnz_chunks"] + 12 * L["chunks"] + 4 + row * (L["x_rows_chunks"] + L["chunks"] - L["chunks_partials"] + L["split_rows"])
        per[("window", i)] = 16 * L["nnz_window"] + 16 * L["window_rows"] + row * 2 * L["window_rows"]
        per[("panel", i)] = 16 * L["nnz_panel"] + 4 * L["panel_bins"] + row * 2 * L["panel_rows"]
        per[("corner", i)] = 16 * L["nnz_corner"] + 4 * 67 * L["corner_tiles"] + row * 2 * L["corner"]
        per[("reduce", i)] = 0
        per[("stage", i)] = 0
    path = 16 * sum(L["nnz"] for L in levels) + 2 * row * n
    return per, path


def algorithmic_bytes(levels, n, k):
    """Bytes one product must move: per launch (kernel class, level) and for the whole path.

    Per level: 8 B per stored entry (X-row id + value) read once, the work-list words, and the
    dense rows: each distinct X row a launch references is read once, each Y row it produces is
    written once (levels >= 1 read it first), split rows write and re-read their partial vectors.
    Column slicing (kc) re-reads entries; that is the kernel's choice, not counted here.
    """
    row = 4 * k
    per = {}
    for i, L in enumerate(levels):
        rmw = 2 if i > 0 else 1
        whole = L["short_rows"] - L["rows_partials"]
        per[("rows", i)] = 8 * L["nnz_rows"] + 12 * L["short_rows"] + 4 + row * (L["x_rows_rows"] + rmw * whole + L["rows_partials"])
        whole = L["chunks"] - L["chunks_partials"]
        per[("chunks", i)] = 8 * L["nnz_chunks"] + 12 * L["chunks"] + 4 + row * (L["x_rows_chunks"] + rmw * whole + L["chunks_partials"])
        per[("reduce", i)] = 8 * L["split_rows"] + 4 + row * (L["partials"] + rmw * L["split_rows"])
        per[("window", i)] = 8 * L["nnz_window"] + 12 * L["window_rows"] + row * (1 + rmw) * L["window_rows"]
        per[("stage", i)] = 0
        # panels: entries, every staged head row once, the eight class results written and read,
        # Y read and written
        per[("panel", i)] = 8 * L["nnz_panel"] + 4 * L["panel_bins"] + row * (18 * L["panel_rows"]) if L["panel_rows"] else 0
        # dense corner: entries, tile words, each tile's 256 staged rows once per tile, the items'
        # result rows written and read, Y read and written
        per[("corner", i)] = (8 * L["nnz_corner"] + 4 * 67 * L["corner_tiles"] + row * 256 * L["corner_tiles"]
                              + row * (2 * 256 * L["corner_items"] + 2 * L["corner"])) if L["corner"] else 0
    # whole product, as the method defines it (independent of how the image executes the levels):
    # 8 B per stored entry and 12 B per work item, X read once and Y written once, and for every
    # later level its active rows gathered again and added to Y (read + write)
    path = sum(8 * L["nnz"] for L in levels) + 2 * row * n
    path += sum(12 * (L["short_rows"] + L["chunks"] + L["window_rows"]) for L in levels)
    path += sum(row * 3 * L["n_i"] for L in levels[1:])
    return per, path


def per_call_events(torch, fn, steps):
    """`steps` calls of fn, each bracketed by a pair of events on the current stream (the stream the
    library launches on); returns the per-call times in ms."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for a, b in pairs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in pairs]


def call_stats(ms):
    ms = sorted(ms)
    return {"median": round(ms[len(ms) // 2], 4), "min": round(ms[0], 4), "mean": round(sum(ms) / len(ms), 4),
            "max": round(ms[-1], 4), "calls": len(ms)}


def gather_yardstick(torch, binding, X, n, k, dev, gathers=1 << 26):
    """Bare gathers of whole rows of X (`arrow_probe_gather`), in G rows/s: rows drawn from an LDS
    window, from 2 MiB per accelerator die (L2 hits), from the first 128 MiB (the size of the staged
    head at the headline) and from all of X.  None where X is too small for a region."""
    if k < 4 or k > 256 or k & (k - 1):
        return None
    row = 4 * k
    out_bytes = binding.arrow_probe_gather_out_bytes(gathers)
    out = torch.empty(out_bytes // 4, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    cases = {"lds_64KiB": ((64 << 10) // row, True, True), "l2_hit_2MiB_per_die": ((2 << 20) // row, True, False),
             "shared_128MiB": ((128 << 20) // row, False, False), "all_of_X": (n, False, False)}
    res = {}
    for name, (rows, per_die, lds) in cases.items():
        if rows < 1 or rows * (8 if per_die else 1) > n:
            res[name] = None
            continue
        def run():
            binding.arrow_probe_gather(X.data_ptr(), n, k, rows, per_die, lds, gathers, out.data_ptr(), out_bytes, stream)
        run()
        ms = per_call_events(torch, run, 3)
        res[name] = round(gathers / (min(ms) * 1e-3) / 1e9, 2)
    res["unit"] = "G rows/s"
    res["row_bytes"] = row
    res["rows_gathered"] = gathers
    return res


def hit_path_rate(torch, binding, k, dev):
    """The product kernels' own rate when every gather hits the L2: a 4096 x 4096 operand with 2048
    random entries per row (8.4 M entries, all of them in the chunk list) times an X of 4096 x k
    (2 MiB at k = 128).  G rows/s of the whole product."""
    rng = np.random.default_rng(7)
    n, per_row = 4096, 2048
    cols = np.sort(np.stack([rng.choice(n, per_row, replace=False) for _ in range(n)]), axis=1)
    rowptr = np.arange(n + 1, dtype=np.int64) * per_row
    vals = rng.uniform(-1, 1, n * per_row).astype(np.float32)
    op = binding.ArrowSpMM(rowptr, cols.astype(np.int32).ravel(), vals, 512, device=dev)
    X = torch.randn((n, k), device=dev)
    Y = torch.empty_like(X)
    for _ in range(3):
        op.spmm(X, Y)
    ms = per_call_events(torch, lambda: op.spmm(X, Y), 10)
    op.close()
    return round(n * per_row / (min(ms) * 1e-3) / 1e9, 2)


def stored_traffic(path, launch_nnz, launch_items):
    """Counter bytes of a launch from a stored rocprofv3 summary, or None when there is none or when
    it was taken on another image (its entry / item counts differ from the live ones)."""
    if not os.path.exists(path):
        return None, None
    with open(path) as f:
        rec = json.load(f)
    src = os.path.relpath(path, ROOT)
    fp = rec.get("launch")
    if not fp or fp.get("nnz") != launch_nnz or fp.get("items") != launch_items:
        return None, src + " (stale: taken on another packed image; ignored)"
    return rec.get("hbm_bytes_per_launch"), src


def bench_mttkrp(args, torch, binding, synth, dev) -> int:
    """One step = one order-3 MTTKRP A = T x (B, C) through ``csf3_mttkrp`` (fibre kernel +
    reduction of split slices), tensor image and factor matrices resident in HBM."""
    cfg = args.config if args.config in (0, 1) else 0
    t0 = time.time()
    w = synth.make_tensor_config(cfg, args.shrink)
    t_gen = time.time() - t0
    t0 = time.time()
    op = binding.Csf3Mttkrp(w.dims, w.i, w.j, w.k, w.vals, device=dev)
    t_build = time.time() - t0
    info = op.info
    Bh, Ch = w.factors()
    B, C = torch.from_numpy(Bh).to(dev), torch.from_numpy(Ch).to(dev)
    A = torch.empty((w.dims[0], w.R), dtype=torch.float32, device=dev)
    for _ in range(args.warmup):
        op.mttkrp(B, C, A)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        op.mttkrp(B, C, A)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    per_call = call_stats(per_call_events(torch, lambda: op.mttkrp(B, C, A), args.steps))
    R, nnz = w.R, w.nnz
    # factorize-and-fuse operation count: 2 per entry and column for the fibre sums, 2 per fibre
    # and column for the products with B (the paper's "Pairwise Contraction" count)
    flops = 2.0 * nnz * R + 2.0 * info["fibers"] * R
    gflops = flops / (ms_per_step * 1e-3) / 1e9
    if args.calibrate_copy:
        # plain device copies of known size (1 GiB read + 1 GiB written each), the yardstick of counter runs
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.calibrate_copy):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    binding.csf3_set_profiling(op.h, True)
    runs = 1 if args.no_profile_pass else max(3, min(10, args.steps))
    k_ms = r_ms = 0.0
    for _ in range(runs):
        op.mttkrp(B, C, A)
        p = binding.csf3_get_profile(op.h)
        k_ms += p["kernel_ms"] / runs
        r_ms += p["reduce_ms"] / runs
    binding.csf3_set_profiling(op.h, False)
    row = 4 * R
    # bytes the fibre kernel must move: entries, segment and item words, every referenced row of B
    # and C once, every row of A or partial vector written once
    alg = (8 * nnz + 8 * info["segments"] + 8 * info["items"] + row * (info["distinct_j"] + info["distinct_k"])
           + row * info["items"])
    achieved = alg / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_mttkrp_kernel_{w.name}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
    roofline = {"bound": "hbm", "kernel": "mttkrp_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "avg_launch_ms": round(k_ms, 4), "launches_per_step": 1, "algorithmic_bytes_per_launch": int(alg),
                "traffic_source": os.path.relpath(tpath, ROOT) if traffic else None,
                # the HBM figure is the required one, but it is not what holds this kernel back: its
                # counter traffic is about its algorithmic bytes, the factor rows live in L2, and the
                # time goes into gathering them from there
                "limiter": "L2-to-L1 gather of factor rows (HBM traffic ~ algorithmic bytes)",
                "gathered_rows_per_launch": int(nnz + info["fibers"]), "row_bytes": row,
                "gather_Grows_per_s": round((nnz + info["fibers"]) / (k_ms * 1e-3) / 1e9, 2) if k_ms > 0 else None}
    cpu_baseline = None
    check = None
    if not args.no_cpu_baseline:
        import oracle
        op.mttkrp(B, C, A)
        torch.cuda.synchronize()
        # calibrate on the first slices, then size the sample (a prefix of whole slices) to --cpu-seconds
        cut = int(np.searchsorted(w.i, max(1, w.dims[0] // 256)))
        t0 = time.perf_counter()
        oracle.mttkrp(w.dims, w.i[:cut], w.j[:cut], w.k[:cut], w.vals[:cut], Bh, Ch)
        t_cal = time.perf_counter() - t0
        want = min(nnz, int(max(cut, 1) / max(t_cal, 1e-6) * args.cpu_seconds))
        last = int(w.i[min(want, nnz) - 1]) if nnz else 0
        cut = nnz if want >= nnz else int(np.searchsorted(w.i, last))          # whole slices only
        rows_done = w.dims[0] if cut == nnz else last
        t0 = time.perf_counter()
        Aref, E = oracle.mttkrp(w.dims, w.i[:cut], w.j[:cut], w.k[:cut], w.vals[:cut], Bh, Ch)
        t_cpu = time.perf_counter() - t0
        fib = len(np.unique(w.i[:cut].astype(np.int64) * w.dims[1] + w.j[:cut]))
        cpu_baseline = {"value": round((2.0 * cut * R + 2.0 * fib * R) / t_cpu / 1e9, 3), "unit": "GFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"slices 0..{rows_done - 1} of the same tensor, all R={R} columns: {cut} nonzeros, "
                                  f"{t_cpu:.1f} s (the oracle evaluates the unfactorized definition; the rate "
                                  f"uses the same operation count as the GPU line)"}
        got = A[:rows_done].cpu().numpy().astype(np.float64)
        ratio = np.abs(got - Aref[:rows_done]) / np.maximum(E[:rows_done], 1e-300)
        check = {"rows": int(rows_done), "max_err_over_bound": float(ratio.max()) if ratio.size else 0.0,
                 "tolerance": 1e-5, "ok": bool(ratio.size == 0 or ratio.max() <= 1e-5)}
    out = {
        "metric": "fp32 order-3 MTTKRP GFLOP/s (2*nnz*R + 2*fibres*R), factorize-and-fuse over compressed sparse fibres",
        "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": None, "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "dims": list(w.dims), "nnz": nnz, "R": R, "fibers": info["fibers"],
                   "items": info["items"], "op": "mttkrp"},
        "per_call_ms": per_call, "roofline": roofline, "cpu_baseline": cpu_baseline,
        "launch_ms": {"mttkrp_kernel": round(k_ms, 4), "reduce_kernel": round(r_ms, 4)},
        "host_seconds": {"generate": round(t_gen, 1), "build_upload": round(t_build, 1)},
        "check": check,
        "paper": "single-thread and multi-node CPU results on FROSTT tensors only (section \"Performance Evaluation\"); not comparable",
    }
    print(json.dumps(out))
    op.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload index 0..4 (3 = headline)")
    ap.add_argument("--shrink", type=int, default=0, help="halve n this many times (debugging only)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0,
                    help="also run this many plain device copies Y <- X (known HBM traffic: n*k*4 read + "
                         "n*k*4 written each) so that counter runs can be scaled")
    ap.add_argument("--no-profile-pass", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--no-gather-yardstick", action="store_true", help="skip the bare row-gather probes")
    ap.add_argument("--hit-path", action="store_true",
                    help="also time the product kernels on a small operand whose X fits the L2 (every gather a "
                         "hit) and report their rate against the L2-hit yardstick")
    ap.add_argument("--kc", type=int, default=None)
    ap.add_argument("--op", choices=("spmm", "sddmm", "mttkrp"), default="spmm",
                    help="spmm: Y = A.X (the headline); sddmm: S = A .* (U V^T) on the same layout; "
                         "mttkrp: order-3 MTTKRP on a synthetic tensor (--config 0 uniform, 1 skewed)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2307_05740_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    if args.op == "mttkrp":
        return bench_mttkrp(args, torch, binding, synth, dev)

    t0 = time.time()
    w = synth.make_config(args.config, args.shrink)
    t_gen = time.time() - t0
    t0 = time.time()
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, w.b, device=dev)
    t_dec = time.time() - t0
    if args.kc is not None:
        binding.arrow_set_option(op.h, "kc", args.kc)
    Xh = w.make_x()
    X = torch.from_numpy(Xh).to(dev)
    Y = torch.empty_like(X)
    k, n, nnz = w.k, w.n, w.nnz
    levels = op.levels()
    sampled = args.op == "sddmm"
    l = 1 if sampled else w.l
    if sampled:
        # U = the workload's X, V = a second seeded normal matrix of the same shape
        Vh = synth.normal_matrix(n, k, seed=w.seed_x + 1)
        V = torch.from_numpy(Vh).to(dev)
        S = torch.empty(nnz, dtype=torch.float32, device=dev)

    def run_once():
        if sampled:
            op.sddmm(X, V, S)
        else:
            op.spmm(X, Y)

    def step():
        if sampled or l == 1:
            run_once()
        else:
            Y.copy_(X)
            op.spmm_iter(Y, l)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    flops = 2.0 * nnz * k * l
    gflops = flops / (ms_per_step * 1e-3) / 1e9
    # the same K steps again, each bracketed by events on the launch stream
    per_call = call_stats(per_call_events(torch, step, args.steps))

    # ---- per-kernel time with HIP events on the launch stream (separate pass) --------------
    for _ in range(args.calibrate_copy):
        Y.copy_(X)
    torch.cuda.synchronize()
    binding.arrow_set_profiling(op.h, True)
    prof_runs = 1 if args.no_profile_pass else max(3, min(10, args.steps))
    acc = {}
    lev_acc = {}
    for _ in range(prof_runs):
        run_once()
        p = binding.arrow_get_profile(op.h)
        for key, v in p.items():
            acc[key] = acc.get(key, 0) + v
        for i in range(len(levels)):
            pl = binding.arrow_get_level_profile(op.h, i)
            for cls in ("rows", "chunks", "reduce", "stage", "window", "panel", "corner"):
                lev_acc[(cls, i)] = lev_acc.get((cls, i), 0.0) + pl[cls + "_ms"]
    binding.arrow_set_profiling(op.h, False)
    prof = {key: v / prof_runs for key, v in acc.items()}
    launch_ms = {key: v / prof_runs for key, v in lev_acc.items()}
    per_bytes, path_bytes = (algorithmic_bytes_sddmm if sampled else algorithmic_bytes)(levels, n, k)
    # the dominant kernel = the single launch (kernel class, level) that takes the most time;
    # at the headline workload that is the chunk kernel of level 0
    dom = max(launch_ms, key=launch_ms.get)
    avg_ms = launch_ms[dom]
    bytes_per_launch = per_bytes[dom]
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
    kname = ("sddmm_" if sampled else "") + dom[0]
    nnz_key = {"rows": "nnz_rows", "chunks": "nnz_chunks", "window": "nnz_window", "panel": "nnz_panel",
               "corner": "nnz_corner"}.get(dom[0])
    item_key = {"rows": "short_rows", "chunks": "chunks", "window": "window_rows", "panel": "panel_bins",
                "corner": "corner_tiles"}.get(dom[0])
    launch_nnz = levels[dom[1]][nnz_key] if nnz_key else 0
    launch_items = levels[dom[1]][item_key] if item_key else 0
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{kname}_kernel_level{dom[1]}_{w.name}.json")
    traffic, traffic_source = stored_traffic(tpath, launch_nnz, launch_items)
    roofline = {"bound": "hbm", "kernel": f"{kname}_kernel (level {dom[1]})", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_ms": round(avg_ms, 4), "launches_per_step": 1,
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "launch": {"nnz": int(launch_nnz), "items": int(launch_items)}}
    if traffic and avg_ms > 0:
        # the counter bytes over the live launch time, and how much of them the method asks for
        roofline["counter_GBps"] = round(traffic / (avg_ms * 1e-3) / 1e9, 1)
        roofline["useful_fraction"] = round(bytes_per_launch / traffic, 4)
    # the plain device-to-device copy Y <- X (n*k*4 bytes read and as many written): what a pure
    # stream reaches on this device, next to the 8 TB/s peak figure
    copy_ms = min(per_call_events(torch, lambda: Y.copy_(X), 5))
    roofline["copy_yardstick_GBps"] = round(2.0 * n * k * 4 / (copy_ms * 1e-3) / 1e9, 1)
    if not args.no_gather_yardstick:
        # every stored entry of the launch gathers one row of 4k bytes: its rate against the bare
        # gather of rows that all hit the L2 is how far the kernel is from the device's limit for
        # this access pattern
        yard = gather_yardstick(torch, binding, X, n, k, dev)
        roofline["gather_yardstick"] = yard
        if yard and avg_ms > 0 and launch_nnz:
            rate = launch_nnz / (avg_ms * 1e-3) / 1e9
            roofline["launch_Grows_per_s"] = round(rate, 2)
            if yard.get("l2_hit_2MiB_per_die"):
                roofline["frac_of_l2_hit_yardstick"] = round(rate / yard["l2_hit_2MiB_per_die"], 3)
            roofline["product_Grows_per_s"] = round(nnz * l / (ms_per_step * 1e-3) / 1e9, 2)
            if args.hit_path and not sampled:
                # the same kernels on an operand whose X fits the L2: what their hit path reaches
                hp = hit_path_rate(torch, binding, k, dev)
                roofline["hit_path_Grows_per_s"] = hp
                if yard.get("l2_hit_2MiB_per_die"):
                    roofline["hit_path_frac_of_l2_hit_yardstick"] = round(hp / yard["l2_hit_2MiB_per_die"], 3)

    # ---- quick correctness sanity + CPU baseline: the oracle on a bounded row sample ----------
    cpu_baseline = None
    check = None
    if not args.no_cpu_baseline and sampled:
        import oracle
        op.sddmm(X, V, S)
        torch.cuda.synchronize()

        def sample_rows(stride):            # the operand with only every stride-th row kept
            rows = np.arange(0, n, stride, dtype=np.int64)
            cnt = np.zeros(n, np.int64)
            cnt[rows] = w.rowptr[rows + 1] - w.rowptr[rows]
            rp = np.concatenate([[0], np.cumsum(cnt)])
            lens = cnt[rows]
            first = np.cumsum(lens) - lens                       # where each kept row starts in the sample
            idx = np.repeat(w.rowptr[rows] - first, lens) + np.arange(int(lens.sum()), dtype=np.int64)
            return rows, rp, idx

        rows, rp, idx = sample_rows(max(1, n // 4096))
        t0 = time.perf_counter()
        oracle.sddmm(rp, w.colidx[idx], w.vals[idx], Xh, Vh)
        t_cal = time.perf_counter() - t0
        rate = max(len(idx), 1) / max(t_cal, 1e-6)
        want = min(nnz, int(rate * args.cpu_seconds))
        stride = max(1, int(round(nnz / max(want, 1))))
        rows, rp, idx = sample_rows(stride)
        t0 = time.perf_counter()
        Sref, B = oracle.sddmm(rp, w.colidx[idx], w.vals[idx], Xh, Vh)
        t_cpu = time.perf_counter() - t0
        cpu_baseline = {"value": round(2.0 * len(idx) * k / t_cpu / 1e9, 3), "unit": "GFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"every {stride}th row of the same operand, all k={k} columns: "
                                  f"{len(rows)} rows, {len(idx)} nonzeros, {t_cpu:.1f} s"}
        Ss = S[torch.from_numpy(idx).to(dev)].cpu().numpy().astype(np.float64)
        ratio = np.abs(Ss - Sref) / np.maximum(B, 1e-300)
        check = {"entries": int(len(idx)), "max_err_over_bound": float(ratio.max()), "tolerance": 1e-5,
                 "ok": bool(ratio.max() <= 1e-5)}
    elif not args.no_cpu_baseline:
        import oracle
        op.spmm(X, Y)
        torch.cuda.synchronize()
        # calibrate on a small stride sample, then size the sample to about --cpu-seconds
        rows = np.arange(0, n, max(1, n // 4096), dtype=np.int64)
        t0 = time.perf_counter()
        oracle.spmm(w.rowptr, w.colidx, w.vals, Xh, rows=rows)
        t_cal = time.perf_counter() - t0
        nnz_cal = int(np.sum(w.rowptr[rows + 1] - w.rowptr[rows]))
        rate = max(nnz_cal, 1) / max(t_cal, 1e-6)              # nonzeros per second
        want = min(nnz, int(rate * args.cpu_seconds))
        stride = max(1, int(round(nnz / max(want, 1))))
        rows = np.arange(0, n, stride, dtype=np.int64)
        nnz_s = int(np.sum(w.rowptr[rows + 1] - w.rowptr[rows]))
        t0 = time.perf_counter()
        Yref, B = oracle.spmm(w.rowptr, w.colidx, w.vals, Xh, rows=rows)
        t_cpu = time.perf_counter() - t0
        cpu_baseline = {"value": round(2.0 * nnz_s * k / t_cpu / 1e9, 3), "unit": "GFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"every {stride}th row of the same operand, all k={k} columns: "
                                  f"{len(rows)} rows, {nnz_s} nonzeros, {t_cpu:.1f} s"}
        Ys = Y[torch.from_numpy(rows).to(dev)].cpu().numpy().astype(np.float64)
        ratio = np.abs(Ys - Yref) / np.maximum(B, 1e-300)
        check = {"rows": int(len(rows)), "max_err_over_bound": float(ratio.max()), "tolerance": 1e-5,
                 "ok": bool(ratio.max() <= 1e-5)}

    out = {
        "metric": ("fp32 A .* (U V^T) GFLOP/s (2*nnz*k), sampled dense-dense product on the arrow layout" if sampled
                   else "fp32 A.X GFLOP/s (2*nnz*k), arrow-decomposed SpMM"),
        "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": None, "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n": n, "nnz": nnz, "k": k, "b": w.b, "products": l,
                   "levels": op.info["levels"], "op": args.op, "tuning": {"kc": args.kc}},
        "per_call_ms": per_call,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "levels": [{"n_i": L["n_i"], "nnz": L["nnz"], "nnz_head_head": L["nnz_head_head"],
                    "nnz_head_row": L["nnz_head_row"], "nnz_head_col": L["nnz_head_col"], "nnz_diag": L["nnz_diag"],
                    "blocks": L["blocks"], "separator_rule": L["separator_rule"], "nnz_fused": L["nnz_fused"],
                    "nnz_corner": L["nnz_corner"]} for L in levels],
        "whole_path": {"algorithmic_GB": round(path_bytes / 1e9, 3),
                       "algorithmic_GBps": round(path_bytes * l / (ms_per_step * 1e-3) / 1e9, 1),
                       "frac_of_hbm_peak": round(path_bytes * l / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "kernel_ms": {key: round(v, 4) for key, v in prof.items()},
        "launch_ms": {f"{c}@{i}": round(v, 4) for (c, i), v in sorted(launch_ms.items(), key=lambda t: -t[1]) if v > 0},
        "host_seconds": {"generate": round(t_gen, 1), "decompose_pack_upload": round(t_dec, 1)},
        "check": check,
        "paper": "not reported (the paper measures other kernels on CPUs)",
    }
    print(json.dumps(out))
    op.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
