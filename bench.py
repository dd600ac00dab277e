#!/usr/bin/env python3
"""Throughput of the Local AdaAlter hot path on one MI355X.

A *step* is one iteration of Algorithm 3 (arXiv 1911.09030) for all W workers: the fused
gradient + parameter update + accumulator update and, on every H-th iteration, the averaging
of x and B^2 over the worker axis.  The default workload is the headline configuration
(d = 400M fp32 parameters, W = 8, H = 16, gradients fused in-kernel from a Philox seed).

Prints ONE JSON line: whole-job element-updates/s with inputs resident in HBM, the HBM roofline
of the dominant kernel (algorithmic bytes per launch / its average duration from HIP events on
the launch stream), and the CPU oracle timed on the host on a bounded sample of the same workload.
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

HBM_PEAK_GBS = 8000.0


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=None, help="timed iterations (default: the workload's own T; 1024 for c5)")
    p.add_argument("--warmup", type=int, default=16)
    p.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    p.add_argument("--H", type=int, default=0, help="override the sync period (c3 sweep)")
    p.add_argument("--algorithm", default="local_adaalter", choices=["local_adaalter", "dist_adagrad", "local_sgd"],
                   help="quadratic workloads: Algorithm 3 (the method), or one of the paper's two comparison methods on the same "
                        "inputs: Algorithm 1 (averages every iteration, H is ignored) or Algorithm 2 (no accumulator)")
    p.add_argument("--offsets", default="philox", choices=["philox", "array", "none"],
                   help="per-worker optimum offsets: regenerated in-kernel, read from HBM, or absent")
    p.add_argument("--row-distance", type=int, default=0,
                   help="elements between the arrays of the spread layout (default workloads.SPREAD_ROW_DISTANCE)")
    p.add_argument("--hold-gaps", action="store_true",
                   help="spread layout as one ordinary allocation that includes the gaps (instead of laa_spread_alloc)")
    p.add_argument("--unfused-sync", action="store_true", help="local step and laa_sync as two kernels")
    p.add_argument("--tile", type=int, default=None,
                   help="laa_set_tile: workers loaded per batch (1, 2, 4, 8), or 0 for one worker per thread block")
    p.add_argument("--pitch", type=int, default=0, help="row pitch of x/acc in elements (0: dense rows of d)")
    p.add_argument("--layout", default="tuned", choices=["tuned", "spread", "packed"],
                   help="tuned: the arrays' places inside a pool of most of the free memory are chosen by timing the "
                        "step on candidate placements (placement.tune), the rest of the pool is released; "
                        "spread: all [W][d] rows and [d] vectors up to 10 GB apart over the HBM address range "
                        "(binding.spread_arrays); packed: ordinary dense tensors")
    p.add_argument("--placements", type=int, default=48, help="random candidate placements of the tuned layout")
    p.add_argument("--no-lazy-replicas", action="store_true",
                   help="write the averaged state into all W rows at every sync (laa_set_lazy_replicas off)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-settle", action="store_true",
                   help="do not wait for the driver's clearing of released memory before timing (profiler counter runs)")
    p.add_argument("--graph", action="store_true",
                   help="quadratic workloads: run whole periods through laa_run_periods_gen (one HIP graph per period, "
                        "replayed) on a side stream; for sizes where the launches dominate")
    p.add_argument("--side-stream", action="store_true", help="run on a non-default stream (as --graph does)")
    p.add_argument("--sparse-repeats", action="store_true",
                   help="workload c4: draw each worker's rows independently (with repeats) and use the coalescing sparse step")
    p.add_argument("--calibrate-copy", type=int, default=0,
                   help="after the run, launch the plain copy kernel this many times over one row of d floats "
                        "(a known volume for scaling profiler byte counters)")
    p.add_argument("--reps", type=int, default=5,
                   help="repetitions of the timed region of --steps iterations; value is the median over them")
    p.add_argument("--no-packed-compare", action="store_true",
                   help="skip the short run in the packed layout that is reported next to the spread one (c5 default run)")
    p.add_argument("--cpu-reps", type=int, default=3, help="repetitions of the one-core CPU baseline (median reported)")
    p.add_argument("--cpu-sample-d", type=int, default=524_288)
    p.add_argument("--cpu-procs", type=int, default=min(16, os.cpu_count() or 1),
                   help="processes of the all-cores CPU baseline (1 switches it off)")
    p.add_argument("--cpu-slice", type=int, nargs=2, metavar=("LO", "N"), default=None,
                   help="internal: run the oracle on columns [LO, LO+N) and print the seconds")
    return p.parse_args()


def traffic_from_profile(kernel_tag: str):
    """HBM bytes per launch of the dominant kernel as last profiled (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a
    copy of known size) and the committed file it is read from; (None, None) if there is none.  A stored figure:
    counters cannot be collected from inside this run."""
    rel = os.path.join("profiles", f"hbm_traffic_{kernel_tag}.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("bytes_per_launch:"):
                return float(line.split(":")[1]), rel
    except OSError:
        pass
    return None, None


def valu_from_profile(kernel_tag: str):
    """Vector-ALU utilisation (per cent) and vector instructions per element-update of the dominant kernel as last
    profiled (rocprofv3 SQ counters) and the committed file they are read from; (None, None, None) if there is none."""
    import re
    rel = os.path.join("profiles", f"valu_{kernel_tag}.txt")
    try:
        text = open(os.path.join(ROOT, rel)).read()
    except OSError:
        return None, None, None
    busy = re.search(r"VALUBusy ([0-9.]+) %", text)           # the first block of the file is the plain step
    per = re.search(r"= ([0-9.]+) per element-update", text)
    return (float(busy.group(1)) if busy else None), (float(per.group(1)) if per else None), rel


def _oracle_period(c, lo, n, offsets):
    """One sync period of the fp64 oracle on the columns [lo, lo + n) of workload c; returns the seconds it took."""
    import numpy as np
    import oracle
    from paper_1911_09030_amd import workloads as wl
    cols = np.arange(lo, lo + n, dtype=np.int64)
    a = wl.curvature(lo + n, c.seed, c.a_dist)[lo:]
    xs = wl.optimum(lo + n, c.seed)[lo:]
    o = oracle.Oracle(n, c.W, c.H, c.eta, c.eps)
    o.set_columns(cols)
    o.init_state()
    om = {"philox": oracle.OFF_PHILOX, "none": oracle.OFF_NONE, "array": oracle.OFF_ARRAY}[offsets]
    off = wl.offsets(lo + n, c.W, c.seed, c.off_scale)[:, lo:] if offsets == "array" else None
    o.set_generator(oracle.GEN_QUADRATIC, c.seed, a, xs, off, om, c.noise_scale, c.off_scale)
    t0 = time.perf_counter()
    for _ in range(c.H):
        o.step_gen()
    return time.perf_counter() - t0


def cpu_baseline(c, sample_d, offsets, procs, reps):
    """The oracle as it stands (single thread, fp64) on a column slice of the same workload, one sync period, median of
    `reps` runs; then the same oracle once as `procs` independent single-threaded processes on disjoint column slices
    (columns are independent, so this is the same computation)."""
    import statistics
    import subprocess
    times = [_oracle_period(c, 0, sample_d, offsets) for _ in range(max(reps, 1))]
    dt = statistics.median(times)
    out = {"value": c.W * sample_d * c.H / dt, "unit": "element-updates/s", "cores": 1, "kind": "oracle",
           "columns": sample_d, "repetitions": len(times), "seconds": [round(t, 2) for t in times],
           "sample": f"first {sample_d} columns of {c.name}, W={c.W}, one sync period of H={c.H} steps, fp64, "
                     f"median of {len(times)} runs: {dt:.1f} s"}
    if procs > 1:
        kids = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--workload", c.name, "--offsets", offsets,
                                  "--cpu-slice", str(i * sample_d), str(sample_d)], stdout=subprocess.PIPE, text=True)
                for i in range(procs)]
        times = [float(k.communicate()[0].strip().splitlines()[-1]) for k in kids]
        if all(k.returncode == 0 for k in kids):
            out["all_cores"] = {"value": procs * c.W * sample_d * c.H / max(times), "unit": "element-updates/s",
                                "cores": procs, "kind": "oracle", "columns": procs * sample_d,
                                "sample": f"{procs} processes x {sample_d} disjoint columns, one run, slowest {max(times):.1f} s"}
    return out


def main():
    args = parse()
    if args.cpu_slice:                      # child of the all-cores CPU baseline: no GPU, no torch
        from paper_1911_09030_amd import workloads as wl
        print(_oracle_period(wl.WORKLOADS[args.workload], args.cpu_slice[0], args.cpu_slice[1], args.offsets))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the W workers are a worker axis in one GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1911_09030_amd import binding as B, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()
    dev = torch.device("cuda:0")
    c = wl.WORKLOADS[args.workload]
    if args.side_stream and not args.graph:
        torch.cuda.set_stream(torch.cuda.Stream(device=dev))
    if args.graph:
        if c.kind != "quadratic" or args.unfused_sync:
            print("bench.py: --graph replays whole periods of the fused generator step (workloads c1, c2, c5)", file=sys.stderr)
            sys.exit(2)
        torch.cuda.set_stream(torch.cuda.Stream(device=dev))     # the default stream cannot be captured
    H = args.H or c.H
    algo = args.algorithm
    if algo != "local_adaalter" and (c.kind != "quadratic" or args.graph or args.unfused_sync):
        print("bench.py: --algorithm runs the fused generator step of the quadratic workloads (c1, c2, c5)", file=sys.stderr)
        sys.exit(2)
    if algo == "dist_adagrad":
        H = 1
    K, Wm = (args.steps if args.steps is not None else c.T), args.warmup
    d, W = c.d, c.W

    pitch = args.pitch or None
    spread = args.layout != "packed"
    keep, layouts = [], []
    tuning = {}

    def alloc(dd, n_mat, n_vec, measure=None):
        """n_mat arrays [W][dd] and n_vec arrays [dd]: at measured places inside a pool (when a measure is given),
        spread over the address range, else ordinary tensors."""
        if args.layout == "tuned" and measure is not None:
            from paper_1911_09030_amd import placement
            pool = None
            try:
                free = torch.cuda.mem_get_info(dev)[0]
                t_tune = time.perf_counter()
                pool = B.Pool(int(free * 0.9), device=dev)
                best = placement.tune(pool, dd, W, n_mat, n_vec, measure, n_random=args.placements, seed=c.seed)
                mats, vecs = placement.views(pool, dd, W, best)
                pool.trim(best.ranges(dd, W))
                keep.append(pool)
                layouts.append(f"tuned(pitch {best.pitch})")
                tuning.setdefault("pools", []).append(
                    {"d": dd, "placements_timed": best.tried, "best_ms": best.ms, "median_ms": best.median_ms,
                     "slowest_ms": best.slowest_ms, "pool_gb": pool.nbytes / 1e9, "seconds": time.perf_counter() - t_tune,
                     "matrices_at_gb": [m * 4 / 1e9 for m in best.matrices], "vectors_at_gb": [v * 4 / 1e9 for v in best.vectors]})
                return mats, vecs, best.pitch
            except (B.LaaError, RuntimeError, ValueError) as e:
                print(f"bench.py: tuned layout unavailable for d={dd} ({e}); spread layout instead", file=sys.stderr)
                if pool is not None:
                    pool.close()
        if spread:
            try:
                backing, mats, vecs, rp = B.spread_arrays(dd, W, n_mat, n_vec, args.row_distance or wl.SPREAD_ROW_DISTANCE,
                                                          dev, hold_gaps=args.hold_gaps)
                keep.append(backing)
                layouts.append(f"spread({rp})")
                return mats, vecs, rp
            except (B.LaaError, RuntimeError, ValueError) as e:   # no memory / address space for it
                print(f"bench.py: spread layout unavailable for d={dd} ({e}); packed tensors instead", file=sys.stderr)
        rp = pitch or dd
        layouts.append(f"packed({rp})")
        mats = [torch.empty((W, rp), dtype=torch.float32, device=dev)[:, :dd] for _ in range(n_mat)]
        vecs = [torch.empty(dd, dtype=torch.float32, device=dev) for _ in range(n_vec)]
        return mats, vecs, rp

    if c.kind == "quadratic":
        with_off = args.offsets == "array"
        om = {"philox": B.OFF_PHILOX, "array": B.OFF_ARRAY, "none": B.OFF_NONE}[args.offsets]

        from paper_1911_09030_amd import placement
        algo_id = {"local_adaalter": None, "dist_adagrad": B.ALGO_DIST_ADAGRAD, "local_sgd": B.ALGO_LOCAL_SGD}[algo]
        measure = placement.quadratic_step_timer(d, W, c.eta, c.eps, c.seed, om, c.noise_scale, c.off_scale, args.tile,
                                                 algo_id, algo == "dist_adagrad" and not args.no_lazy_replicas)
        mats, (bsnap, a, xs), rp = alloc(d, 3 if with_off else 2, 3, measure)
        g = B.LocalAdaAlter(d, W, H, c.eta, c.eps, b0=0.0 if algo == "dist_adagrad" else None,
                            x=mats[0], acc=mats[1], snap=bsnap, pitch=rp)
        if algo_id is not None:
            g.set_algorithm(algo_id)
        a.copy_(torch.from_numpy(wl.curvature(d, c.seed, c.a_dist)))
        xs.copy_(torch.from_numpy(wl.optimum(d, c.seed)))
        g.init_state()
        off = None
        if with_off:
            off = mats[2]
            for w in range(W):      # inputs only: N(0, off_scale^2) drawn on the device, one worker row at a time
                off[w].normal_(0.0, c.off_scale)
        g.set_generator(B.GEN_QUADRATIC, c.seed, a, xs, off, om, c.noise_scale, c.off_scale)
        step_bytes = (16 * W + 12 + (4 * W if off is not None else 0)) * d
        kernel_tag = f"step_kernel_{c.name}"
        if algo != "local_adaalter":
            # Algorithm 1 reads every x row, a, x* and snap and writes every x and acc row and snap (with lazy replicas its
            # one iterate is row 0 of x and snap); Algorithm 2 reads and writes every x row and reads a, x*.  Every
            # iteration of Algorithm 1 is the same kernel, and Algorithm 2's averaging moves what its plain step moves.
            lazy_on = not args.no_lazy_replicas
            per_col = ((24 if lazy_on else 12 * W + 16) if algo == "dist_adagrad" else 8 * W + 8) + (4 * W if off is not None else 0)
            step_bytes = per_col * d
            kernel_tag = f"baseline_kernel_{algo}_{c.name}"
        if args.unfused_sync:
            def do_step(t):
                g.local_step_gen()
                if t % H == 0:
                    g.sync()
        else:
            def do_step(t):
                g.step_gen()
        updates_per_step = W * d
    elif c.kind == "explicit":
        P = 4

        def measure(mats, vecs, rp):
            """The explicit-gradient step streaming the pool of gradient tensors, arrays at a candidate placement."""
            for m in mats[2:]:
                m.zero_()
            h = B.LocalAdaAlter(d, W, 1 << 30, c.eta, c.eps, x=mats[0], acc=mats[1], snap=vecs[0], pitch=rp)
            h.init_state()
            if args.tile is not None:
                h.set_tile(args.tile)
            k = [0]

            def one():
                k[0] += 1
                h.step_dense(mats[2 + k[0] % P])
            one()
            from paper_1911_09030_amd.placement import event_median_ms
            ms = event_median_ms(one, n=2 * P + 1)
            h.close()
            return ms

        mats, (bsnap, sig), rp = alloc(d, 2 + P, 2, measure)
        g = B.LocalAdaAlter(d, W, H, c.eta, c.eps, x=mats[0], acc=mats[1], snap=bsnap, pitch=rp)
        g.init_state()
        sig.copy_(torch.from_numpy(wl.sigma(d, c.seed)))
        g.set_generator(B.GEN_NOISE, c.seed, sig)
        pool = mats[2:]
        for p in range(P):           # precompute the gradient pool in HBM; the timed loop streams it
            g.generate_gradient(pool[p])
            g.step_dense(pool[p])    # advance t so each pool entry uses another iteration's noise
        g.init_state()
        step_bytes = (20 * W + 4) * d
        kernel_tag = f"step_kernel_{c.name}"

        def do_step(t):
            g.step_dense(pool[t % P])
        updates_per_step = W * d
    else:  # embedding table with row-sparse gradients + dense LSTM blocks
        from paper_1911_09030_amd import placement
        mats, (bsnap,), rp = alloc(d, 2, 1, placement.averaging_timer(d, W, c.eta, c.eps))
        g = B.LocalAdaAlter(d, W, H, c.eta, c.eps, x=mats[0], acc=mats[1], snap=bsnap, pitch=rp)
        g.init_state()
        zipf = wl.ZipfRows(c.rows, c.zipf_s)
        P = 16
        if args.sparse_repeats:      # tokens drawn independently: popular rows repeat within a worker's list
            import numpy as np
            rng = np.random.default_rng(c.seed)
            idx_pool = [torch.from_numpy(np.minimum(np.searchsorted(zipf.cdf, rng.random((W, c.k))), c.rows - 1)
                                         .astype(np.int32)).to(dev) for t in range(P)]
            g.set_sparse_coalesce(True)
        else:
            idx_pool = [torch.from_numpy(wl.sparse_step(zipf, W, c.k, c.row_len, c.seed, t, with_vals=False)[0]).to(dev)
                        for t in range(P)]
        vals_pool = [torch.randn((W, c.k, c.row_len), dtype=torch.float32, device=dev) * c.val_sigma for _ in range(4)]
        dd = sum(r * q for r, q in c.dense_blocks)
        dmats, (dsnap, sigd), drp = alloc(dd, 2, 2, placement.generator_step_timer(dd, W, c.eta, c.eps, c.seed, B.GEN_NOISE, B.OFF_NONE,
                                                                                     c.noise_scale, c.off_scale))
        gd = B.LocalAdaAlter(dd, W, H, c.eta, c.eps, x=dmats[0], acc=dmats[1], snap=dsnap, pitch=drp)
        gd.init_state()
        sigd.copy_(torch.from_numpy(wl.sigma(dd, c.seed)))
        gd.set_generator(B.GEN_NOISE, c.seed, sigd)
        step_bytes = W * c.k * (c.row_len * 24 + 4)
        kernel_tag = f"sparse_step_kernel_{c.name}"

        mid = {}

        def do_step(t):
            g.step_sparse(idx_pool[t % P], vals_pool[t % 4], c.row_len)
            if t in mid:                      # timed region: split the iteration into its sparse and dense parts
                mid[t].record()
            gd.step_gen()
        updates_per_step = W * c.k * c.row_len + W * dd
    if args.tile is not None:
        g.set_tile(args.tile)
    lazy = not args.no_lazy_replicas and c.kind != "embedding" and algo != "local_sgd"    # Algorithm 2 has no collapsed state
    if lazy:
        g.set_lazy_replicas(True)
    if not args.no_lazy_replicas and c.kind == "embedding":
        gd.set_lazy_replicas(True)       # the dense blocks; the table's sparse sync never collapses

    handles = [g] + ([gd] if c.kind == "embedding" else [])

    def moved_bytes():
        m = [h.bytes_moved(literal=True) for h in handles]
        return sum(v[0] for v in m), sum(v[1] for v in m)

    # Warm-up (untimed), then on to the iteration right after an averaging one.  From there K timed iterations hold
    # floor(K / H) averaging iterations and as many that read the collapsed state, never more: a K that is not a whole
    # number of periods is not flattered by the cheaper iterations.  (Replayed periods start on a period boundary.)
    phase = 0 if args.graph else 1 % H
    t = 0

    def align():
        nonlocal t
        while t == 0 or t % H != phase:
            t += 1
            do_step(t)

    for _ in range(Wm):
        t += 1
        do_step(t)
    align()
    # Memory that the layout gave back to the driver (the unused part of the pool, the spacers of the spread layout)
    # is cleared by the driver in the background for some seconds, which takes a little bandwidth from everything
    # that runs meanwhile (measured: the step 0.7 % slower for up to 20 s after 240 GB were released).  Keep
    # stepping, untimed, until whole periods stop getting faster.
    settle = None
    if spread and not args.graph and not args.no_settle:
        # reference: what the tuner measured for the dominant kernel at the chosen placement (quadratic and explicit
        # workloads, whose first pool is the one the step runs on); otherwise wait for a plateau
        ref = tuning["pools"][0]["best_ms"] if tuning.get("pools") and c.kind != "embedding" else None
        t_settle, hist = time.perf_counter(), []
        n_it = max(H, (64 // H) * H)
        while time.perf_counter() - t_settle < 40.0:
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_it + 1)]
            ev[0].record()
            for i in range(n_it):
                t += 1
                do_step(t)
                ev[i + 1].record()
            torch.cuda.synchronize()
            ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(n_it)]
            tt0 = t - n_it + 1
            pl = sorted(m for i, m in enumerate(ms) if (tt0 + i) % H != 0 and not (lazy and (tt0 + i - 1) % H == 0)) or sorted(ms)
            hist.append(pl[len(pl) // 2])
            if ref is not None and len(hist) >= 2 and max(hist[-2:]) <= ref * 1.002:      # two windows in a row at the tuner's figure
                break
            if ref is None and len(hist) >= 4 and max(hist[-3:]) < min(hist[-3:]) * 1.0005:
                break
        settle = {"seconds": time.perf_counter() - t_settle, "untimed_iterations": len(hist) * n_it,
                  "plain_ms_first_window": hist[0], "plain_ms_at_end": hist[-1], "reference_ms": ref}
        align()
    if args.graph:
        K -= K % H
        g.run_periods_gen(3)                 # the first period of each kind runs as plain launches, the third records
        t += 3 * H
    torch.cuda.synchronize()

    reps = max(args.reps, 1)
    per_step_ms, kinds, walls = [], [], []   # over all repetitions; kind: "plain", "sync" (averages), "post" (reads the collapsed state)
    bytes_timed = [0, 0]                     # moved and literal bytes of the timed iterations (not of the realignment between repetitions)
    for _ in range(reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        if c.kind == "embedding":
            mid.clear()
            mid.update({t + i + 1: torch.cuda.Event(enable_timing=True) for i in range(K)})
        t_first = t + 1
        bytes_before = moved_bytes()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev[0].record()
        if args.graph:
            g.run_periods_gen(K // H)
            t += K
            ev[K].record()
        else:
            for i in range(K):
                t += 1
                do_step(t)
                ev[i + 1].record()
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t0)
        bytes_after = moved_bytes()
        bytes_timed = [bytes_timed[k] + bytes_after[k] - bytes_before[k] for k in (0, 1)]
        if args.graph:                       # no events inside a replayed period: the average over all iterations
            ms = [ev[0].elapsed_time(ev[K]) / K] * K
        elif c.kind == "embedding":          # the roofline line is the row-sparse step alone
            ms = [ev[i].elapsed_time(mid[t_first + i]) for i in range(K)]
        else:
            ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(K)]
        per_step_ms += ms
        # iteration tt averages when tt % H == 0 and, with lazy replicas, reads a collapsed state when the one before it averaged
        for i in range(K):
            tt = t_first + i
            if algo == "dist_adagrad":       # one kernel, every iteration
                kinds.append("plain")
            else:
                kinds.append("sync" if tt % H == 0 else "post" if lazy and tt > 1 and (tt - 1) % H == 0 else "plain")
        align()
    n_timed = reps * K
    if args.graph:
        assert g.replay_count() >= reps * (K // H), "the periods were not replayed from a graph"
        graph_inputs = step_bytes // d - (16 * W + 4)
        lazy_on = not args.no_lazy_replicas
        if H == 1:
            period_cols = (8 + graph_inputs + 8) if lazy_on else (16 * W + 8 + graph_inputs)
        elif lazy_on:    # H - 2 plain steps, the averaging one (writes the collapsed state), the one reading it
            period_cols = ((H - 2) * (16 * W + 4 + graph_inputs) + (8 * W + 4 + graph_inputs + 8)
                           + (8 + graph_inputs + 8 * W))
        else:
            period_cols = (H - 1) * (16 * W + 4 + graph_inputs) + (16 * W + 8 + graph_inputs)
        graph_step_bytes = period_cols * d // H

    # the dominant kernel is the plain step: neither the averaging one nor, with lazy replicas, the one right after it
    kernel_name = kernel_tag.rsplit("_", 1)[0]
    by_kind = {k: [m for m, kk in zip(per_step_ms, kinds) if kk == k] for k in ("plain", "sync", "post")}
    plain = by_kind["plain"]
    if not plain and c.kind != "embedding":
        # No plain step among the timed iterations (H = 1, H = 2 with lazy replicas, or very few iterations): the
        # dominant kernel is the averaging step if there is one, else the step that reads the collapsed state.
        inputs = step_bytes // d - (16 * W + 4)
        if by_kind["sync"]:     # reads the state (collapsed if the iteration before averaged too), writes the means
            state_in = 8 if (lazy and H == 1) else 8 * W + 4
            state_out = 8 if lazy else 8 * W + 4
            step_bytes = (state_in + inputs + state_out) * d
            kernel_tag += "_sync"
            kernel_name += " (averaging step)"
            plain = by_kind["sync"]
        else:                   # reads row 0 of x, snap and the inputs, writes every worker's rows
            step_bytes = (8 + inputs + 8 * W) * d
            kernel_tag += "_after_sync"
            kernel_name += " (step after an averaging)"
            plain = by_kind["post"]
    if not plain:
        plain = per_step_ms
    if args.graph:
        plain, step_bytes = per_step_ms, graph_step_bytes
        kernel_tag += "_graph"
        kernel_name += " (average over the iterations of a replayed period)"
    import statistics
    kern_ms = sum(plain) / len(plain)
    achieved = step_bytes / (kern_ms * 1e-3) / 1e9
    values = [updates_per_step * K / w for w in walls]
    value = statistics.median(values)
    mean_of = lambda v: (sum(v) / len(v)) if v else None
    ms_sync, ms_post = mean_of(by_kind["sync"]), mean_of(by_kind["post"])
    # one whole period in the steady state, from the per-kind iteration times: independent of how many iterations of
    # each kind the timed region happened to hold
    steady_ms = steady_value = None
    if algo == "dist_adagrad":
        steady_ms = mean_of(by_kind["plain"])
        steady_value = updates_per_step / (steady_ms * 1e-3)
    elif not args.graph and c.kind != "embedding":
        n_post = 1 if (lazy and H >= 2) else 0
        parts = [(H - 1 - n_post, mean_of(by_kind["plain"])), (1, ms_sync), (n_post, ms_post)]
        if all(n == 0 or m is not None for n, m in parts):
            steady_ms = sum(n * m for n, m in parts if n) / H
            steady_value = updates_per_step / (steady_ms * 1e-3)
    moved = bytes_timed[0] / (updates_per_step * n_timed)
    literal = bytes_timed[1] / (updates_per_step * n_timed)

    g.materialize()
    assert bool(torch.isfinite(g.x[W - 1, :4096]).all()), "non-finite parameters after the run"
    for _ in range(args.calibrate_copy):          # reads 4d bytes, writes 4d bytes
        B.debug_copy(g.acc[0], g.x[0])
    torch.cuda.synchronize()
    # The same machine's plain copy rate (one load and one store per thread, the library's copy kernel over one row
    # of the state), timed the same way: what a streaming kernel can reach here, next to the published peak.
    copy_gbs = None
    if d % 4 == 0 and d >= 1 << 22:
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.debug_copy(g.acc[0], g.x[0])
        c0.record()
        for _ in range(20):
            B.debug_copy(g.acc[0], g.x[0])
        c1.record()
        torch.cuda.synchronize()
        copy_gbs = 20 * 8 * d / (c0.elapsed_time(c1) * 1e-3) / 1e9

    # The same workload in ordinary packed tensors, a short run next to the spread one (the spread layout is this
    # benchmark's choice of placement; a caller with plain allocations gets this figure).
    packed = None
    if (c.kind == "quadratic" and spread and layouts and not layouts[0].startswith("packed") and not args.graph
            and not args.no_packed_compare and not args.unfused_sync and args.offsets != "array" and algo == "local_adaalter"):
        pa, pxs = a.clone(), xs.clone()
        gp = B.LocalAdaAlter(d, W, H, c.eta, c.eps)
        gp.init_state()
        gp.set_generator(B.GEN_QUADRATIC, c.seed, pa, pxs, None, om, c.noise_scale, c.off_scale)
        if args.tile is not None:
            gp.set_tile(args.tile)
        gp.set_lazy_replicas(lazy)
        Kp = max(H, min(K, 4 * H))
        for _ in range(H + 1):
            gp.step_gen()
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(Kp + 1)]
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        pe[0].record()
        for i in range(Kp):
            gp.step_gen()
            pe[i + 1].record()
        torch.cuda.synchronize()
        pwall = time.perf_counter() - p0
        pk = [pe[i].elapsed_time(pe[i + 1]) for i in range(Kp)
              if (H + 2 + i) % H != 0 and not (lazy and (H + 1 + i) % H == 0)]
        packed = {"value": updates_per_step * Kp / pwall, "steps": Kp,
                  "kernel_ms": (sum(pk) / len(pk)) if pk else None,
                  "frac": (step_bytes / (sum(pk) / len(pk) * 1e-3) / 1e9 / HBM_PEAK_GBS) if pk else None}
        del gp, pa, pxs

    traffic, traffic_source = traffic_from_profile(kernel_tag)
    valu_busy, valu_per_update, valu_source = valu_from_profile(kernel_tag)
    frac = achieved / HBM_PEAK_GBS
    out = {
        "metric": "element-updates/sec and achieved HBM GB/s (% of peak), step+sync, 1 GPU",
        "value": value, "unit": "element-updates/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": updates_per_step / value * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{c.name}: {'' if algo == 'local_adaalter' else 'algorithm=' + algo + ' '}d={d} W={W} H={H} eta={c.eta} eps={c.eps} kind={c.kind} "
                               f"offsets={args.offsets if c.kind == 'quadratic' else 'n/a'} "
                               f"sync={'separate kernel' if args.unfused_sync else 'fused into the H-th step'} "
                               f"lazy_replicas={'on' if lazy else 'off'} layout={'+'.join(layouts)}"
                               f"{' periods replayed from a HIP graph' if args.graph else ''}",
                   "repetitions": reps, "value_is": f"median over {reps} repetitions of {K} timed iterations",
                   "values": values,
                   "timed_iterations_by_kind": {k: len(v) for k, v in by_kind.items()},
                   "ms_sync_iteration": ms_sync, "ms_post_sync_iteration": ms_post,
                   "ms_per_step_steady_state": steady_ms, "value_steady_state": steady_value,
                   "bytes_per_element_update_moved": moved, "bytes_per_element_update_literal": literal,
                   "packed_layout": packed, "layout_tuning": tuning or None, "settling_after_release": settle,
                   "parity_bar": "1e-5 relative to max(|ref|, largest |x| on the trajectory, floor); floor 1 for x on "
                                 "generated gradients, 1e-3 otherwise"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": frac, "target_frac": 0.80, "meets_target": frac >= 0.80,
                     "traffic": traffic, "traffic_source": (f"stored: {traffic_source} (rocprofv3 counters of an earlier run "
                                                            "of this command, not measured in this run)") if traffic_source else None,
                     "valu_busy_pct": valu_busy, "valu_instructions_per_element_update": valu_per_update,
                     "valu_source": f"stored: {valu_source} (rocprofv3 counters of an earlier run)" if valu_source else None,
                     "kernel": kernel_name, "kernel_ms": kern_ms, "kernel_ms_min": min(plain),
                     "kernel_ms_median": statistics.median(plain), "kernel_ms_max": max(plain), "kernel_launches_timed": len(plain),
                     "algorithmic_bytes_per_launch": step_bytes, "copy_kernel_gbs_same_run": copy_gbs},
    }
    if not args.no_cpu_baseline and c.kind == "quadratic" and algo == "local_adaalter":
        out["cpu_baseline"] = cpu_baseline(c, min(args.cpu_sample_d, d), args.offsets, args.cpu_procs, args.cpu_reps)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
