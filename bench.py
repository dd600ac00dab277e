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
    p.add_argument("--layout", default="spread", choices=["spread", "packed"],
                   help="spread: all [W][d] rows and [d] vectors up to 10 GB apart over the HBM address range "
                        "(binding.spread_arrays); packed: ordinary dense tensors")
    p.add_argument("--no-lazy-replicas", action="store_true",
                   help="write the averaged state into all W rows at every sync (laa_set_lazy_replicas off)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--graph", action="store_true",
                   help="quadratic workloads: run whole periods through laa_run_periods_gen (one HIP graph per period, "
                        "replayed) on a side stream; for sizes where the launches dominate")
    p.add_argument("--side-stream", action="store_true", help="run on a non-default stream (as --graph does)")
    p.add_argument("--sparse-repeats", action="store_true",
                   help="workload c4: draw each worker's rows independently (with repeats) and use the coalescing sparse step")
    p.add_argument("--calibrate-copy", type=int, default=0,
                   help="after the run, launch the plain copy kernel this many times over one row of d floats "
                        "(a known volume for scaling profiler byte counters)")
    p.add_argument("--cpu-sample-d", type=int, default=524_288)
    p.add_argument("--cpu-procs", type=int, default=min(16, os.cpu_count() or 1),
                   help="processes of the all-cores CPU baseline (1 switches it off)")
    p.add_argument("--cpu-slice", type=int, nargs=2, metavar=("LO", "N"), default=None,
                   help="internal: run the oracle on columns [LO, LO+N) and print the seconds")
    return p.parse_args()


def traffic_from_profile(kernel_tag: str):
    """Last profiled HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated), if recorded."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{kernel_tag}.txt")
    try:
        for line in open(path):
            if line.startswith("bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


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


def cpu_baseline(c, sample_d, offsets, procs):
    """The oracle as it stands (single thread, fp64) on a column slice of the same workload, one sync period; then
    the same oracle as `procs` independent single-threaded processes on disjoint column slices (columns are
    independent, so this is the same computation)."""
    import subprocess
    dt = _oracle_period(c, 0, sample_d, offsets)
    out = {"value": c.W * sample_d * c.H / dt, "unit": "element-updates/s", "cores": 1, "kind": "oracle",
           "sample": f"first {sample_d} columns of {c.name}, W={c.W}, one sync period of H={c.H} steps, fp64, "
                     f"{dt:.1f} s"}
    if procs > 1:
        kids = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--workload", c.name, "--offsets", offsets,
                                  "--cpu-slice", str(i * sample_d), str(sample_d)], stdout=subprocess.PIPE, text=True)
                for i in range(procs)]
        times = [float(k.communicate()[0].strip().splitlines()[-1]) for k in kids]
        if all(k.returncode == 0 for k in kids):
            out["all_cores"] = {"value": procs * c.W * sample_d * c.H / max(times), "unit": "element-updates/s",
                                "cores": procs, "kind": "oracle",
                                "sample": f"{procs} processes x {sample_d} disjoint columns, slowest {max(times):.1f} s"}
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
    K, Wm = (args.steps if args.steps is not None else c.T), args.warmup
    d, W = c.d, c.W

    pitch = args.pitch or None
    spread = args.layout != "packed"
    keep, layouts = [], []

    def alloc(dd, n_mat, n_vec):
        """n_mat arrays [W][dd] and n_vec arrays [dd]: spread over the address range, else ordinary tensors."""
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
        mats, (bsnap, a, xs), rp = alloc(d, 3 if with_off else 2, 3)
        g = B.LocalAdaAlter(d, W, H, c.eta, c.eps, x=mats[0], acc=mats[1], snap=bsnap, pitch=rp)
        a.copy_(torch.from_numpy(wl.curvature(d, c.seed, c.a_dist)))
        xs.copy_(torch.from_numpy(wl.optimum(d, c.seed)))
        g.init_state()
        off = None
        if with_off:
            off = mats[2]
            for w in range(W):      # inputs only: N(0, off_scale^2) drawn on the device, one worker row at a time
                off[w].normal_(0.0, c.off_scale)
        om = {"philox": B.OFF_PHILOX, "array": B.OFF_ARRAY, "none": B.OFF_NONE}[args.offsets]
        g.set_generator(B.GEN_QUADRATIC, c.seed, a, xs, off, om, c.noise_scale, c.off_scale)
        step_bytes = (16 * W + 12 + (4 * W if off is not None else 0)) * d
        kernel_tag = f"step_kernel_{c.name}"
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
        mats, (bsnap, sig), rp = alloc(d, 2 + P, 2)
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
        mats, (bsnap,), rp = alloc(d, 2, 1)
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
        dmats, (dsnap, sigd), drp = alloc(dd, 2, 2)
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
    lazy = not args.no_lazy_replicas and c.kind != "embedding"
    if lazy:
        g.set_lazy_replicas(True)
    if not args.no_lazy_replicas and c.kind == "embedding":
        gd.set_lazy_replicas(True)       # the dense blocks; the table's sparse sync never collapses

    # warm-up (untimed), then realign to a period boundary so the timed region holds K/H syncs
    t = 0
    for _ in range(Wm):
        t += 1
        do_step(t)
    while t % H:
        t += 1
        do_step(t)
    torch.cuda.synchronize()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    if c.kind == "embedding":
        mid.update({t + i + 1: torch.cuda.Event(enable_timing=True) for i in range(K)})
    t_first = t + 1
    if args.graph:
        K -= K % H
        g.run_periods_gen(3)                 # the first period of each kind runs as plain launches, the third records
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    if args.graph:
        g.run_periods_gen(K // H)
        ev[K].record()
    else:
        for i in range(K):
            t += 1
            do_step(t)
            ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    if args.graph:                           # no events inside a replayed period: the average over all iterations
        assert g.replay_count() >= K // H, "the periods were not replayed from a graph"
        per_step_ms = [ev[0].elapsed_time(ev[K]) / K] * K
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
    else:
        per_step_ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(K)]
    if c.kind == "embedding":                 # the roofline line is the row-sparse step alone
        per_step_ms = [ev[i].elapsed_time(mid[t_first + i]) for i in range(K)]
    # the dominant kernel is the plain step: not the averaging one ((i+1) % H == 0) and, with lazy replicas, not the
    # one right after it (i % H == 0), which reads the collapsed state
    kernel_name = kernel_tag.rsplit("_", 1)[0]
    # timed iteration i is iteration t_first + i of the run; the warm-up ends on a period boundary, so iteration i
    # averages when (i + 1) % H == 0, and reads a collapsed state when the iteration before it averaged
    after_sync = [lazy and i % H == 0 and t_first + i > 1 for i in range(K)]
    plain = [per_step_ms[i] for i in range(K) if (i + 1) % H != 0 and not after_sync[i]]
    if not plain and c.kind != "embedding":
        # No plain step among the timed iterations (H = 1, H = 2 with lazy replicas, or very few iterations): the
        # dominant kernel is the averaging step if there is one, else the step that reads the collapsed state.
        inputs = step_bytes // d - (16 * W + 4)
        sync_idx = [i for i in range(K) if (i + 1) % H == 0]
        if sync_idx:            # reads the state (collapsed if the iteration before averaged too), writes the means
            state_in = 8 if after_sync[sync_idx[-1]] else 8 * W + 4
            state_out = 8 if lazy else 8 * W + 4
            step_bytes = (state_in + inputs + state_out) * d
            kernel_tag += "_sync"
            kernel_name += " (averaging step)"
            plain = [per_step_ms[i] for i in sync_idx if after_sync[i] == after_sync[sync_idx[-1]]]
        else:                   # reads row 0 of x, snap and the inputs, writes every worker's rows
            step_bytes = (8 + inputs + 8 * W) * d
            kernel_tag += "_after_sync"
            kernel_name += " (step after an averaging)"
            plain = per_step_ms
    if not plain:
        plain = per_step_ms
    if args.graph:
        plain, step_bytes = per_step_ms, graph_step_bytes
        kernel_tag += "_graph"
        kernel_name += " (average over the iterations of a replayed period)"
    post_sync = [per_step_ms[i] for i in range(K) if after_sync[i] and (i + 1) % H != 0]
    sync_it = [per_step_ms[i] for i in range(K) if (i + 1) % H == 0]
    kern_ms = sum(plain) / len(plain)
    achieved = step_bytes / (kern_ms * 1e-3) / 1e9
    value = updates_per_step * K / wall

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

    out = {
        "metric": "element-updates/sec and achieved HBM GB/s (% of peak), step+sync, 1 GPU",
        "value": value, "unit": "element-updates/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": wall * 1e3 / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{c.name}: d={d} W={W} H={H} eta={c.eta} eps={c.eps} kind={c.kind} "
                               f"offsets={args.offsets if c.kind == 'quadratic' else 'n/a'} "
                               f"sync={'separate kernel' if args.unfused_sync else 'fused into the H-th step'} "
                               f"lazy_replicas={'on' if lazy else 'off'} layout={'+'.join(layouts)}"
                               f"{' periods replayed from a HIP graph' if args.graph else ''}",
                   "syncs_in_timed_region": len(sync_it),
                   "ms_sync_iteration": (sum(sync_it) / len(sync_it)) if sync_it else None,
                   "ms_post_sync_iteration": (sum(post_sync) / len(post_sync)) if post_sync else None,
                   "method_bytes_per_element_update": 16 + 4 / W + (16 * W + 4) / (W * H)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic_from_profile(kernel_tag),
                     "kernel": kernel_name, "kernel_ms": kern_ms,
                     "algorithmic_bytes_per_launch": step_bytes, "copy_kernel_gbs_same_run": copy_gbs},
    }
    if not args.no_cpu_baseline and c.kind == "quadratic":
        out["cpu_baseline"] = cpu_baseline(c, min(args.cpu_sample_d, d), args.offsets, args.cpu_procs)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
