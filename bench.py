#!/usr/bin/env python3
"""Benchmark of the decentralized-SGD model-averaging hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input, with X and
G already resident in HBM:
    build the iteration's mixing table on the host (seeded random ring)   -> upload it
    fused mix + SGD kernel  X_out = mix(X) - lr * G                       (Sec. 2, Eq. 2)
    consensus distance of X_out                                            (Sec. 3)
    swap the X buffers (and rotate the gradient buffers)
Default workload: n = 64 learners, d = 100,000,000 parameters, bf16 gradients, randomized
ring (the configuration the 80 %-of-HBM target is quoted on).

After the timed region the default run also measures, in the same process and on the same box, what the
headline has to be read against (`legs` and `reference_streams` in the JSON): the same step in place, on plain
dense arrays through the entry points the baseline names, on the other workloads, and the traffic of the step
with the mixing taken out (read-only, write-only and x + a g streams in the step kernel's own access pattern),
plus the runtime's device-to-device copy.

Prints ONE JSON line on stdout; progress and per-kernel detail go to stderr.
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recorded_traffic(workload, variant):
    """HBM bytes per launch of the dominant kernel as read from hardware counters in an EARLIER rocprofv3 run
    (two --pmc runs, FETCH_SIZE then WRITE_SIZE, KiB per dispatch, each scaled by the same counter's reading
    for a plain device copy of known size).  The readings live in a small text file under profiles/ together
    with the commit they were taken at; a (workload, variant) that was not profiled reports null."""
    try:
        with open(TRAFFIC_FILE) as f:
            rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    except OSError:
        return None
    for r in rows:
        if len(r) >= 8 and r[0] == workload and r[1] == variant:
            fetch_kib, fetch_scale, write_kib, write_scale = float(r[2]), float(r[3]), float(r[4]), float(r[5])
            return {"bytes": (fetch_kib * fetch_scale + write_kib * write_scale) * 1024.0,
                    "commit": r[6], "date": r[7], "file": os.path.relpath(TRAFFIC_FILE, ROOT)}
    return None


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        return 1


def cpu_baseline(wl, seconds_budget=16.0):
    """The oracle as it stands, timed on the host: whole hot-path step (dense-matrix update
    in fp64 + two-pass consensus distance) on a column slice of the same workload."""
    import numpy as np
    from oracle import psgd_oracle as orc
    from paper_2002_01119_amd import inputs as inp
    threads = host_threads()
    cols = min(wl.d, 1_000_000)
    X = inp.host_normal_f32((wl.n, cols), wl.sigma_x, wl.seed_x)
    if wl.g_dtype == "bf16":
        G = inp.host_normal_bf16_bits((wl.n, cols), wl.sigma_g, wl.seed_g)
    else:
        G = inp.host_normal_f32((wl.n, cols), wl.sigma_g, wl.seed_g)
    steps, elapsed = 0, 0.0
    while steps < 2 or (elapsed < seconds_budget / 2 and steps < 8):
        t0 = time.perf_counter()
        T = orc.mixing_matrix(wl.topology, wl.n, wl.seed_perm, steps)
        Xn = orc.mix_step(X, G, T, wl.lr)
        orc.consensus_dist(Xn)
        elapsed += time.perf_counter() - t0
        X = Xn.astype(np.float32)
        steps += 1
    return {
        "value": wl.n * cols * steps / elapsed,
        "unit": "updates/s",
        "cores": threads,
        "kind": "oracle",
        "sample": "first %d of %d columns x all %d learners, %d steps (columns are independent; "
                  "dense fp64 mixing-matrix product + two-pass consensus distance, numpy)"
                  % (cols, wl.d, wl.n, steps),
    }


def cpu_baseline_sparse(wl, seconds_budget=8.0):
    """The oracle's sparse form (plain C gather-add over the 3-slot table + two-pass distance, fp64), one
    thread and all cores: the memory-bound CPU baseline of the same step."""
    import numpy as np
    from oracle import psgd_oracle as orc
    from paper_2002_01119_amd import inputs as inp
    cores = os.cpu_count() or 1
    try:
        cores = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        pass
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores) or cores))
    cols = min(wl.d, 1_000_000)
    X = inp.host_normal_f32((wl.n, cols), wl.sigma_x, wl.seed_x)
    if wl.g_dtype == "bf16":
        G = inp.host_normal_bf16_bits((wl.n, cols), wl.sigma_g, wl.seed_g)
    else:
        G = inp.host_normal_f32((wl.n, cols), wl.sigma_g, wl.seed_g)
    out = {"unit": "updates/s", "kind": "oracle (sparse C form)",
           "sample": "first %d of %d columns x all %d learners (columns are independent; gather-add over the 3-slot "
                     "table in fp64 + two-pass consensus distance, gcc -O2 -fopenmp)" % (cols, wl.d, wl.n)}
    for label, threads in (("single_thread", 1), ("all_cores", cores)):
        steps, elapsed = 0, 0.0
        while steps < 2 or (elapsed < seconds_budget / 2 and steps < 6):
            nbr, w = orc.neighbour_table(wl.topology, wl.n, wl.seed_perm, steps)
            t0 = time.perf_counter()
            Xn = orc.sparse_mix_step(X, G, nbr, w, wl.lr, threads=threads)
            orc.sparse_consensus_dist(Xn, threads=threads)
            elapsed += time.perf_counter() - t0
            steps += 1
        out[label] = {"value": wl.n * cols * steps / elapsed, "cores": threads, "steps": steps}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=5, help="1..5, the synthetic workload table")
    ap.add_argument("--no-consensus", action="store_true", help="leave the consensus distance out of the step")
    ap.add_argument("--unfused", action="store_true",
                    help="separate mix and consensus kernels instead of the fused psgd_mix_step_cd")
    ap.add_argument("--in-place", action="store_true", help="mix in place instead of ping-pong buffers")
    ap.add_argument("--overlap", action="store_true",
                    help="delay-by-one workloads: run the gradient producer of step k+1 on a second stream, "
                         "concurrently with the mix of step k (Sec. 4: gradient computation beside the averaging)")
    ap.add_argument("--global-average", action="store_true",
                    help="mix with T_u = (1/n) 1 1^T (psgd_mix_full: S-PSGD / the paper's own D1D-PSGD) instead of "
                         "the workload's ring table")
    ap.add_argument("--degree", type=int, default=3,
                    help="odd K > 3: mix with K neighbours on the workload's ring (self and (K-1)/2 learners on each "
                         "side, weight 1/K each) through psgd_mix_step_deg, the general sparse-table kernel")
    ap.add_argument("--two-rings", action="store_true",
                    help="3-slot table that is NOT one ring (two disjoint rings over the even and the odd learners): "
                         "takes the tiled fallback of the step kernel")
    ap.add_argument("--device-tables", action="store_true",
                    help="build each iteration's table on the device (psgd_build_mixing_device) instead of on the "
                         "host followed by an upload")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed region, capture the same K steps (tables built on the device from a device-side "
                         "iteration counter) in ONE HIP graph, replay it, and report its time per step beside the eager one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-legs", action="store_true",
                    help="skip the measurements that follow the timed region (in-place, dense layout, other workloads, "
                         "reference streams, device copy)")
    ap.add_argument("--layout", choices=["pitched", "spread", "interleaved", "probe", "dense"], default="pitched",
                    help="where the arrays live in HBM: 'pitched' interleaves the rows of all arrays across most of "
                         "the device (psgd_mix_step_ex), 'spread' is the same layout on psgd_spread_alloc memory "
                         "(rows physically as far apart, only the rows resident), 'interleaved' is plain dense arrays in one "
                         "psgd_interleaved_alloc block (1 GiB pieces from the three thirds of the device's memory in "
                         "turn), 'probe' keeps dense arrays but "
                         "places X / X_out on the windows of one pool where the step runs fastest, 'dense' is one "
                         "plain tensor per array")
    ap.add_argument("--span-fraction", type=float, default=0.65,
                    help="pitched layout: fraction of device memory the row slots are spread over")
    ap.add_argument("--g-apart", action="store_true",
                    help="pitched layout: keep the gradient buffers in a pitched pool of their own instead of in the "
                         "slots of X / X_out")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the warm-up, run a plain dense device copy of known size (printed); under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate the mix kernel's")
    args = ap.parse_args()
    if args.degree < 3 or args.degree % 2 == 0 or (args.degree > 3 and (args.global_average or args.device_tables)):
        log("bench.py: --degree takes an odd K >= 3 and excludes --global-average and --device-tables")
        sys.exit(2)
    if args.two_rings and (args.degree > 3 or args.global_average or args.device_tables or args.graph):
        log("bench.py: --two-rings excludes --degree, --global-average, --device-tables and --graph")
        sys.exit(2)
    if args.graph and (args.degree > 3 or args.overlap):
        log("bench.py: --graph excludes --degree and --overlap")
        sys.exit(2)
    if args.gpus != 1:
        log("bench.py: this build runs all learners on ONE GPU (no collectives); --gpus %d is not "
            "supported, run with --gpus 1" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2002_01119_amd import d1d
    from paper_2002_01119_amd import inputs as inp
    from paper_2002_01119_amd import placement as plc
    from paper_2002_01119_amd import psgd

    psgd.load()                      # no fallback: fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = inp.workload(args.workload)
    n, d = wl.n, wl.d
    K, W = args.steps, args.warmup
    total = K + W
    log("workload %s: n=%d d=%d G=%s steps=%d warmup=%d" % (wl.name, n, d, wl.g_dtype, K, W))
    stream = torch.cuda.Stream(device=dev)
    stream2 = torch.cuda.Stream(device=dev)

    def bytes_per_update(w_):
        return 10 if w_.g_dtype == "bf16" else 12        # X read + G read + X_out write

    def gdtype(w_):
        return torch.bfloat16 if w_.g_dtype == "bf16" else torch.float32

    def pitched_buffers(w_, in_place, with_delay_buffers, settle=True, spread=False):
        """Rows of every array interleaved across most of the HBM (placement.pitched_layout):
        slot i = [X_i | Y_i | (Xprev_i | noise_i) | G0_i | G1_i], slots `pitch` bytes apart.  With `spread` the
        slots come from psgd_spread_alloc: as far apart physically, but nothing between them stays allocated."""
        free, total_mem = torch.cuda.mem_get_info()
        specs = [("X", torch.float32)] + ([] if in_place else [("Y", torch.float32)])
        if with_delay_buffers:
            specs += [("Xprev", torch.float32), ("noise", torch.float32)]
        gspecs = [("G0", gdtype(w_)), ("G1", gdtype(w_))]
        span = min(int(args.span_fraction * total_mem), free - (8 << 30))
        pools = []
        if spread:
            views, owner, pitch = plc.spread_layout(w_.n, w_.d, specs + gspecs, span, dev)
            rep = {"layout": "spread", "pitch_GB": pitch / 1e9, "span_GB": w_.n * pitch / 1e9,
                   "pool_allocated_GB": owner.resident_bytes() / 1e9,
                   "data_resident_GB": sum(v.shape[0] * v.shape[1] * v.element_size() for v in views.values()) / 1e9,
                   "arrays": list(views.keys()), "gradients_in_own_pool": False}
            return views, [owner], rep
        if args.g_apart:
            gbytes = 2 * w_.n * w_.d * torch.empty((), dtype=gdtype(w_)).element_size()
            views, pool, pitch = plc.pitched_layout(w_.n, w_.d, specs, span - gbytes - (1 << 30), dev, settle=settle)
            gviews, gpool, _ = plc.pitched_layout(w_.n, w_.d, gspecs, 0, dev, settle=False)
            views.update(gviews)
            pools = [pool, gpool]
        else:
            views, pool, pitch = plc.pitched_layout(w_.n, w_.d, specs + gspecs, span, dev, settle=settle)
            pools = [pool]
        rep = {"layout": "pitched", "pitch_GB": pitch / 1e9, "span_GB": pool.numel() / 1e9,
               "pool_allocated_GB": sum(p.numel() for p in pools) / 1e9,
               "data_resident_GB": sum(v.shape[0] * v.shape[1] * v.element_size() for v in views.values()) / 1e9,
               "arrays": list(views.keys()), "gradients_in_own_pool": bool(args.g_apart)}
        return views, pools, rep

    # ---- resident inputs
    n_xbuf = 1 if args.in_place else (3 if wl.delay else 2)
    gdt = gdtype(wl)
    layout_report, pool, views = {"layout": args.layout}, None, None

    def draw_g(i):
        return (inp.device_normal_bf16 if wl.g_dtype == "bf16" else inp.device_normal_f32)(
            (n, d), wl.sigma_g, wl.seed_g + i, dev)

    if args.layout in ("pitched", "spread"):
        try:
            views, pool, layout_report = pitched_buffers(wl, args.in_place, wl.delay, spread=args.layout == "spread")
            log("%s layout: %d slots %.3f GB apart, %.1f GB allocated for %.1f GB of data"
                % (args.layout, n, layout_report["pitch_GB"], layout_report["pool_allocated_GB"],
                   layout_report["data_resident_GB"]))
        except torch.OutOfMemoryError:
            log("pitched layout does not fit; falling back to dense tensors")
            views, layout_report = None, {"layout": "dense (pitched did not fit)"}
        if views is not None:
            X = inp.fill_normal_rows_(views["X"], wl.sigma_x, wl.seed_x)
            Y = X if args.in_place else views["Y"]
            Gs = [inp.fill_normal_rows_(views["G%d" % i], wl.sigma_g, wl.seed_g + i) for i in range(2)]
    elif args.layout == "interleaved":
        specs = [("X", torch.float32)] + ([] if args.in_place else [("Y", torch.float32)])
        if wl.delay:
            specs += [("Xprev", torch.float32), ("noise", torch.float32)]
        specs += [("G0", gdt), ("G1", gdt)]
        views, pool = plc.interleaved_layout(n, d, specs, dev)
        data_gb = sum(v.numel() * v.element_size() for v in views.values()) / 1e9
        layout_report = {"layout": "interleaved", "pool_allocated_GB": (pool.nbytes + (1 << 30) - 1) // (1 << 30) * (1 << 30) / 1e9,
                         "data_resident_GB": data_gb, "arrays": list(views.keys()),
                         "note": "dense [n, d] arrays in one psgd_interleaved_alloc block"}
        log("interleaved layout: dense arrays, %.1f GB allocated for %.1f GB of data"
            % (layout_report["pool_allocated_GB"], data_gb))
        X = inp.fill_normal_rows_(views["X"], wl.sigma_x, wl.seed_x)
        Y = X if args.in_place else views["Y"]
        Gs = [inp.fill_normal_rows_(views["G%d" % i], wl.sigma_g, wl.seed_g + i) for i in range(2)]
    elif args.layout == "probe":
        # X and X_out are rewritten every step: put them where this chip writes fastest
        Gs = [draw_g(i) for i in range(2)]
        nbr0, w0 = psgd.build_mixing(wl.topology, n, wl.seed_perm, 0)
        extra = (n * d * 4 if wl.delay else 0) + (6 << 30)          # noise buffer + headroom
        try:
            wins, pool, rep = plc.place_replica_buffers(
                n, d, n_xbuf, Gs[0], torch.from_numpy(nbr0).to(dev), torch.from_numpy(w0).to(dev),
                reserve_bytes=extra, max_pool_bytes=12 * n * d * 4, log=log)
            layout_report.update(rep)
            views = {"X": wins[0]}
            if not args.in_place:
                views["Y"] = wins[1]
            if wl.delay:
                views["Xprev"] = wins[2]
            X = inp.fill_normal_rows_(views["X"], wl.sigma_x, wl.seed_x)
            Y = X if args.in_place else views["Y"]
        except (torch.OutOfMemoryError, RuntimeError) as e:
            log("placement probe skipped (%s); falling back to dense tensors" % (str(e).splitlines()[0],))
            views, layout_report = None, {"layout": "dense (probe did not fit)"}
            del Gs
    if views is None:
        X = inp.device_normal_f32((n, d), wl.sigma_x, wl.seed_x, dev)
        Y = X if args.in_place else torch.empty_like(X)
        Gs = [draw_g(i) for i in range(2)]
    noise = None
    if wl.delay:                      # delay-by-one: G_k = c * X_{k-1} + noise, three X buffers
        noise = views["noise"] if (views is not None and "noise" in views) else torch.empty((n, d), device=dev)
        inp.fill_normal_rows_(noise, wl.sigma_g, wl.seed_g + 7)
    X_prev = None
    if wl.delay:
        X_prev = views["Xprev"] if (views is not None and "Xprev" in views) else torch.empty((n, d), device=dev)
    deg = args.degree
    if deg > min(n, 32) or n * deg > 4096:
        log("bench.py: --degree %d does not fit n = %d" % (deg, n))
        sys.exit(2)
    nbr_host = torch.empty((total, n, deg), dtype=torch.int32, pin_memory=True)
    w_host = torch.empty((total, n, deg), dtype=torch.float32, pin_memory=True)
    nbr_dev = torch.empty((total, n, deg), dtype=torch.int32, device=dev)
    w_dev = torch.empty((total, n, deg), dtype=torch.float32, device=dev)
    cdist = torch.zeros(total, dtype=torch.float64, device=dev)
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    torch.cuda.synchronize()
    fused = not (args.unfused or args.no_consensus)

    def widen(nbr3, k=None):
        """K-slot table on the same ring: follow the right (left) pointers (K-1)/2 times."""
        k = deg if k is None else k
        left, right = nbr3[:, 1], nbr3[:, 2]
        cols, lo, hi = [nbr3[:, 0]], nbr3[:, 0], nbr3[:, 0]
        for _ in range((k - 1) // 2):
            lo, hi = left[lo], right[hi]
            cols += [lo, hi]
        return (np.ascontiguousarray(np.stack(cols, axis=1), dtype=np.int32),
                np.full((nbr3.shape[0], k), 1.0 / k, dtype=np.float32))

    def split_in_two(nbr3):
        """The same learners on two disjoint rings: every learner's neighbours become its neighbours' neighbours
        (for even n the ring falls apart into the even and the odd positions)."""
        left, right = nbr3[:, 1], nbr3[:, 2]
        return np.ascontiguousarray(np.stack([nbr3[:, 0], left[left], right[right]], axis=1), dtype=np.int32)

    def upload_table(k):
        if args.device_tables:
            psgd.build_mixing_device(wl.topology, n, wl.seed_perm, nbr_dev[k], w_dev[k], step_offset=k, stream=stream)
            return
        nbr, w = psgd.build_mixing(wl.topology, n, wl.seed_perm, k)
        if deg > 3:
            nbr, w = widen(nbr)
        if args.two_rings:
            nbr = split_in_two(nbr)
        nbr_host[k].copy_(torch.from_numpy(nbr))
        w_host[k].copy_(torch.from_numpy(w))
        nbr_dev[k].copy_(nbr_host[k], non_blocking=True)
        w_dev[k].copy_(w_host[k], non_blocking=True)

    # Delay-by-one workloads run through the two-stream schedule of d1d.DelayByOne (overlap or serial order);
    # its table callback uploads the iteration's table on the mix stream right before the mix.
    delayed = None
    if wl.delay:
        def table_of(k):
            return nbr_dev[k], w_dev[k]
        delayed = d1d.DelayByOne(X, Y, X_prev, Gs, noise, None if args.global_average else table_of, wl.lr,
                                 wl.grad_pull, overlap=args.overlap, mix_stream=stream, producer_stream=stream2)
        torch.cuda.synchronize()

    def one_step(k):
        nonlocal X, Y
        with torch.cuda.stream(stream):
            upload_table(k)
        cd = cdist[k:k + 1] if fused else None
        if delayed is not None:
            out = delayed.step(cdist_out=cd, before_mix=ev0[k].record, after_mix=ev1[k].record, more=k + 1 < total)
            if not (fused or args.no_consensus):
                psgd.consensus_dist_async(out, cdist[k:k + 1], stream=stream)
            ev2[k].record(stream)
            return
        G = Gs[k % 2]
        ev0[k].record(stream)
        if args.global_average:
            psgd.mix_full(X, Y, G, wl.lr, stream=stream, cdist_out=cd)
        else:
            psgd.mix_step(X, Y, G, nbr_dev[k], w_dev[k], wl.lr, stream=stream, cdist_out=cd)
        ev1[k].record(stream)
        if not (fused or args.no_consensus):
            psgd.consensus_dist_async(Y, cdist[k:k + 1], stream=stream)
        ev2[k].record(stream)
        if not args.in_place:
            X, Y = Y, X

    def device_copy_rate(nbytes):
        """The runtime's own device-to-device copy of two dense buffers (read nbytes, write nbytes)."""
        ca = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        cb = torch.empty_like(ca)
        with torch.cuda.stream(stream):
            cb.copy_(ca)
            t_c0, t_c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t_c0.record(stream)
            cb.copy_(ca)
            t_c1.record(stream)
        torch.cuda.synchronize()
        cms = t_c0.elapsed_time(t_c1)
        del ca, cb
        return cms, 2 * nbytes / cms / 1e6

    if args.calibrate_copy:
        cal_bytes = min(12_800_000_000, torch.cuda.mem_get_info()[0] // 3) // 4096 * 4096
        cms, cgbs = device_copy_rate(cal_bytes)
        log("calibration: plain dense device copy of %d bytes (= %d KiB read and as many written): %.3f ms -> "
            "%.1f GB/s (%.1f %% of peak)" % (cal_bytes, cal_bytes // 1024, cms, cgbs, cgbs / HBM_PEAK_GBS * 100))
    for k in range(W):
        one_step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(W, total):
        one_step(k)
    if delayed is not None:
        delayed.finish()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if delayed is not None:
        X, Y, X_prev = delayed.X, delayed.Y, delayed.X_prev
    graph_report = None
    if args.graph:
        # The same K steps as one graph: {table from the device-side counter, counter += 1, fused step} x K.
        step_dev = torch.full((1,), total, dtype=torch.int64, device=dev)
        tab_n = torch.empty((n, 3), dtype=torch.int32, device=dev)
        tab_w = torch.empty((n, 3), dtype=torch.float32, device=dev)

        def graph_step(k, cur):
            nonlocal X, Y, X_prev
            psgd.build_mixing_device(wl.topology, n, wl.seed_perm, tab_n, tab_w, step_dev=step_dev, advance=1, stream=cur)
            G = Gs[k % 2]
            if wl.delay:
                psgd.synth_grad(X_prev, noise, G, wl.grad_pull, stream=cur)
            cd = None if args.no_consensus else cdist[k:k + 1]
            if args.global_average:
                psgd.mix_full(X, Y, G, wl.lr, delay_mode=1 if wl.delay else 0, stream=cur,
                              cdist_out=None if args.unfused else cd)
            else:
                psgd.mix_step(X, Y, G, tab_n, tab_w, wl.lr, delay_mode=1 if wl.delay else 0, stream=cur,
                              cdist_out=None if args.unfused else cd)
            if args.unfused and cd is not None:
                psgd.consensus_dist_async(Y, cd, stream=cur)
            if wl.delay:
                X_prev, X, Y = X, Y, X_prev
            elif not args.in_place:
                X, Y = Y, X

        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=stream):
            for k in range(K):
                graph_step(k, torch.cuda.current_stream())
        gr.replay()                                  # warm-up replay
        torch.cuda.synchronize()
        reps = 3
        tg0 = time.perf_counter()
        for _ in range(reps):
            gr.replay()
        torch.cuda.synchronize()
        tg1 = time.perf_counter()
        gms = 1e3 * (tg1 - tg0) / (reps * K)
        graph_report = {"steps_per_graph": K, "replays": reps, "ms_per_step": gms, "value": n * d / (gms * 1e-3)}
        log("HIP graph of %d steps: %.4f ms per step over %d replays" % (K, gms, reps))
    if psgd.device_status() != 0:
        log("bench.py: a kernel flagged an invalid mixing table")
        sys.exit(4)

    wall = t1 - t0
    mix_ms = [ev0[k].elapsed_time(ev1[k]) for k in range(W, total)]
    con_ms = [ev1[k].elapsed_time(ev2[k]) for k in range(W, total)]
    mix_avg = sum(mix_ms) / len(mix_ms)
    con_avg = sum(con_ms) / len(con_ms)
    mix_bytes = bytes_per_update(wl) * n * d
    achieved = mix_bytes / (mix_avg * 1e-3) / 1e9
    cvals = cdist.cpu().numpy()
    log("mix kernel: avg %.3f ms (min %.3f, max %.3f) -> %.1f GB/s algorithmic, %.1f %% of %d GB/s"
        % (mix_avg, min(mix_ms), max(mix_ms), achieved, 100 * achieved / HBM_PEAK_GBS, HBM_PEAK_GBS))
    if fused:
        log("consensus distance is fused into the mix kernel; final reduce kernel avg %.4f ms" % con_avg)
        log("consensus distance after the timed steps: first %.6g last %.6g" % (cvals[W], cvals[-1]))
    elif not args.no_consensus:
        cgb = 4 * n * d / (con_avg * 1e-3) / 1e9
        log("consensus kernels: avg %.3f ms -> %.1f GB/s algorithmic (4 B/element), %.1f %% of peak"
            % (con_avg, cgb, 100 * cgb / HBM_PEAK_GBS))
        log("consensus distance after the timed steps: first %.6g last %.6g" % (cvals[W], cvals[-1]))
    log("whole step: %.3f ms wall per step over %d steps" % (1e3 * wall / K, K))

    variant = ("full" if args.global_average else "two_rings" if args.two_rings else "ring" if deg == 3
               else "degree%d" % deg)
    default_form = (args.layout == "pitched" and fused and not args.in_place and not args.g_apart
                    and not (wl.delay and args.overlap) and layout_report.get("layout") == "pitched")
    traffic = recorded_traffic(wl.name, variant) if default_form else None
    result = {
        "metric": "replica-param updates/s and achieved HBM GB/s (% of peak) for fused mix+SGD step",
        "metric_note": "value = replica-parameter updates per second of the whole hot-path step (table build, fused "
                       "mix+SGD kernel, consensus distance); achieved HBM GB/s and its fraction of the peak are in roofline",
        "value": n * d * K / wall,
        "unit": "updates/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": 1e3 * wall / K,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": wl.name, "n": n, "d": d, "g_dtype": wl.g_dtype,
            "topology": ("full (T_u)" if args.global_average else
                         "two disjoint rings (tiled fallback)" if args.two_rings else
                         {0: "ring", 1: "rand_ring"}[wl.topology]),
            "table_degree": deg, "tables_built_on": "device" if args.device_tables else "host",
            "lr": wl.lr,
            "delay_by_one": wl.delay, "consensus_every_step": not args.no_consensus,
            "consensus_fused_into_mix_kernel": fused,
            "in_place": bool(args.in_place), "producer_overlapped": bool(wl.delay and args.overlap),
            "hbm_layout": layout_report,
        },
        "roofline": {
            "kernel": ("mix_full_kernel" if args.global_average else "mix_deg_kernel" if deg > 3
                       else "mix_step_kernel (tiled path)" if args.two_rings else "mix_step_kernel")
                      + (" (with fused consensus statistics)" if fused else ""),
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            # counters are read in separate rocprofv3 --pmc runs of this same command, not in this run
            "traffic": traffic["bytes"] if traffic else None,
            "traffic_source": ({k_: traffic[k_] for k_ in ("file", "commit", "date")} if traffic else None),
            "algorithmic_bytes_per_launch": mix_bytes, "avg_launch_ms": mix_avg,
            "target_frac": 0.80, "target_met": bool(achieved / HBM_PEAK_GBS >= 0.80),
        },
        "mix_updates_per_s": n * d / (mix_avg * 1e-3),
    }
    if graph_report is not None:
        result["hip_graph"] = graph_report
    if not (args.no_consensus or fused):
        result["consensus"] = {"avg_ms": con_avg, "achieved_GBps": 4 * n * d / (con_avg * 1e-3) / 1e9,
                               "frac": 4 * n * d / (con_avg * 1e-3) / 1e9 / HBM_PEAK_GBS}

    # ------------------------------------------------------------------ what the headline is read against
    def timed(fn, warm=2, reps=5):
        """Average / min / max duration in ms of `reps` launches of fn(stream), HIP events on that stream."""
        for _ in range(warm):
            fn(stream)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record(stream)
            fn(stream)
            b.record(stream)
        torch.cuda.synchronize()
        ms = [a.elapsed_time(b) for a, b in evs]
        return sum(ms) / len(ms), min(ms), max(ms)

    def leg(label, w_, nbytes, ms, **extra):
        avg, lo, hi = ms
        gbs = nbytes / (avg * 1e-3) / 1e9
        r = {"workload": w_.name, "avg_launch_ms": avg, "min_launch_ms": lo, "max_launch_ms": hi,
             "value": w_.n * w_.d / (avg * 1e-3), "unit": "updates/s",
             "achieved_GBps": gbs, "frac": gbs / HBM_PEAK_GBS, "launches": 5}
        r.update(extra)
        log("  %-44s %8.3f ms  %7.1f GB/s  %5.1f %% of peak" % (label, avg, gbs, 100 * gbs / HBM_PEAK_GBS))
        return r

    def reference_streams(w_, Xr, Yr, Gr, layout):
        """Read-only, write-only and x + a g traffic of the step's own access pattern on these buffers."""
        nd = w_.n * w_.d
        gb = 2 if w_.g_dtype == "bf16" else 4
        out = {"layout": layout, "workload": w_.name,
               "note": "psgd_reference_stream: the step kernel's lane/column ownership, lockstep row batches and "
                       "persistent grid, without the mixing"}
        for name, kind, per in (("read_x_and_g", psgd.REF_READ, 4 + gb), ("write_x_out", psgd.REF_WRITE, 4),
                                ("axpy_x_plus_a_g", psgd.REF_AXPY, 8 + gb)):
            ms = timed(lambda s_: psgd.reference_stream(kind, Xr, Yr, Gr, 0.5, stream=s_))
            gbs = per * nd / (ms[0] * 1e-3) / 1e9
            out[name] = {"bytes_per_element": per, "avg_launch_ms": ms[0], "achieved_GBps": gbs,
                         "frac": gbs / HBM_PEAK_GBS}
            log("  reference %-24s %8.3f ms  %7.1f GB/s  %5.1f %% of peak" % (name, ms[0], gbs, 100 * gbs / HBM_PEAK_GBS))
        return out

    extra_ok = (not args.no_extra_legs and deg == 3 and not args.global_average and not args.two_rings
                and not args.graph and fused and args.layout == "pitched" and views is not None
                and not args.in_place and not args.device_tables)
    if extra_ok:
        log("legs beside the headline (5 launches each, same process):")
        legs = {}
        tab = (nbr_dev[total - 1], w_dev[total - 1])
        cd1 = torch.zeros(1, dtype=torch.float64, device=dev)
        Xa, Ya, Ga = X, Y, Gs[0]
        result["reference_streams"] = reference_streams(wl, Xa, Ya, Ga, "pitched (the headline's buffers)")
        # the headline's kernel again, so that the streams and the step stand side by side in one list
        ms = timed(lambda s_: psgd.mix_step(Xa, Ya, Ga, tab[0], tab[1], wl.lr, delay_mode=1 if wl.delay else 0,
                                            stream=s_, cdist_out=cd1))
        legs["pitched_out_of_place"] = leg("pitched, out of place (headline)", wl, mix_bytes, ms, layout="pitched",
                                           in_place=False, entry_point="psgd_mix_step_ex")
        if not wl.delay:
            ms = timed(lambda s_: psgd.mix_step(Xa, Xa, Ga, tab[0], tab[1], wl.lr, stream=s_, cdist_out=cd1))
            legs["pitched_in_place"] = leg("pitched, in place", wl, mix_bytes, ms, layout="pitched", in_place=True,
                                           entry_point="psgd_mix_step_ex")
        if not wl.delay and n % 2 == 0 and n >= 13:
            # ---- tables that are not one ring (the LDS-tiled kernel), and the distance as a pass of its own
            nb3, w3 = psgd.build_mixing(wl.topology, n, wl.seed_perm, total - 1)
            for key, label, (nb_, ww_) in (
                    ("tiled_two_rings_pitched", "two disjoint rings (tiled kernel)", (split_in_two(nb3), w3)),
                    ("tiled_degree13_pitched", "13 neighbours per learner (tiled kernel)", widen(nb3, 13))):
                nb_, ww_ = torch.from_numpy(nb_).to(dev), torch.from_numpy(ww_).to(dev)
                ms = timed(lambda s_: psgd.mix_step(Xa, Ya, Ga, nb_, ww_, wl.lr, stream=s_, cdist_out=cd1))
                legs[key] = leg(label, wl, mix_bytes, ms, layout="pitched", in_place=False,
                                entry_point="psgd_mix_step_ex" if nb_.shape[1] == 3 else "psgd_mix_step_deg",
                                table_degree=int(nb_.shape[1]))
            ms = timed(lambda s_: psgd.consensus_dist_async(Ya, cd1, stream=s_))
            legs["consensus_alone_pitched"] = leg("consensus distance alone (4 B per element)", wl, 4 * n * d, ms,
                                                  layout="pitched", entry_point="psgd_consensus_dist_async")
        del Xa, Ya, Ga
        # ---- the plain dense [n, d] arrays of the entry points the baseline names
        del X, Y, Gs, X_prev, views, pool, noise, delayed
        torch.cuda.empty_cache()
        try:
            Xd = inp.device_normal_f32((n, d), wl.sigma_x, wl.seed_x, dev)
            Yd = torch.empty_like(Xd)
            Gd = draw_g(0)
            ep = "psgd_mix_step_cd_bf16g" if wl.g_dtype == "bf16" else "psgd_mix_step_cd"
            ms = timed(lambda s_: psgd.mix_step(Xd, Yd, Gd, tab[0], tab[1], wl.lr, delay_mode=1 if wl.delay else 0,
                                                stream=s_, cdist_out=cd1))
            legs["dense_out_of_place"] = leg("dense arrays, out of place", wl, mix_bytes, ms, layout="dense",
                                             in_place=False, entry_point=ep)
            if not wl.delay:
                ms = timed(lambda s_: psgd.mix_step(Xd, Xd, Gd, tab[0], tab[1], wl.lr, stream=s_, cdist_out=cd1))
                legs["dense_in_place"] = leg("dense arrays, in place", wl, mix_bytes, ms, layout="dense",
                                             in_place=True, entry_point=ep)
            result["reference_streams_dense"] = reference_streams(wl, Xd, Yd, Gd, "dense")
            del Xd, Yd, Gd
        except torch.OutOfMemoryError:
            log("  dense leg skipped: out of memory")
        torch.cuda.empty_cache()
        cms, cgbs = device_copy_rate(min(12_800_000_000, torch.cuda.mem_get_info()[0] // 3) // 4096 * 4096)
        result["device_copy"] = {"what": "runtime device-to-device copy of two dense 12.8 GB buffers (torch copy_)",
                                 "avg_ms": cms, "achieved_GBps": cgbs, "frac": cgbs / HBM_PEAK_GBS}
        log("  runtime device-to-device copy       %8.3f ms  %7.1f GB/s  %5.1f %% of peak" % (cms, cgbs, 100 * cgbs / HBM_PEAK_GBS))
        # ---- the other HBM-sized workloads in the pitched layout (fused step + distance, their own shapes)
        if args.workload == 5:
            for idx in (2, 3, 4):
                w_ = inp.workload(idx)
                try:
                    v_, p_, _rep = pitched_buffers(w_, False, False)
                except torch.OutOfMemoryError:
                    log("  workload %d leg skipped: out of memory" % idx)
                    continue
                inp.fill_normal_rows_(v_["X"], w_.sigma_x, w_.seed_x)
                inp.fill_normal_rows_(v_["G0"], w_.sigma_g, w_.seed_g)
                nb_, ww_ = psgd.build_mixing(w_.topology, w_.n, w_.seed_perm, 0)
                nb_, ww_ = torch.from_numpy(nb_).to(dev), torch.from_numpy(ww_).to(dev)
                ms = timed(lambda s_: psgd.mix_step(v_["X"], v_["Y"], v_["G0"], nb_, ww_, w_.lr,
                                                    delay_mode=1 if w_.delay else 0, stream=s_, cdist_out=cd1))
                legs["workload%d_pitched" % idx] = leg("workload %d, pitched" % idx, w_, bytes_per_update(w_) * w_.n * w_.d,
                                                       ms, layout="pitched", in_place=False, entry_point="psgd_mix_step_ex")
                del v_, p_
                torch.cuda.empty_cache()
        # ---- the headline's workload with only its data resident, in processes of their own: (i) rows physically
        # spread by psgd_spread_alloc instead of living in a pool that spans the device, (ii) plain dense arrays in a
        # psgd_interleaved_alloc block.  Both rely on the order in which the driver hands out physical memory, which
        # is the address order only in a process that has not freed large allocations before (the spread rows
        # allocated in this process at this point: 64.8-66 %; fresh: 76-77.6 %).
        torch.cuda.empty_cache()
        for key, lay, label in (("spread_fresh_process", "spread", "spread rows, only the data resident"),
                                ("dense_interleaved_fresh_process", "interleaved", "dense arrays, interleaved block")):
            try:
                child = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", str(args.workload),
                                        "--layout", lay, "--no-extra-legs", "--no-cpu-baseline", "--steps", "5",
                                        "--warmup", "2", "--span-fraction", str(args.span_fraction)],
                                       capture_output=True, text=True, timeout=300)
                r_ = json.loads(child.stdout.strip().splitlines()[-1])
                roof_, lay_ = r_["roofline"], r_["config"]["hbm_layout"]
                legs[key] = {
                    "workload": wl.name, "avg_launch_ms": roof_["avg_launch_ms"], "value": r_["value"], "unit": "updates/s",
                    "achieved_GBps": roof_["achieved"], "frac": roof_["frac"], "launches": 5, "layout": lay,
                    "in_place": False,
                    "entry_point": "psgd_mix_step_ex" if lay == "spread" else
                                   ("psgd_mix_step_cd_bf16g" if wl.g_dtype == "bf16" else "psgd_mix_step_cd"),
                    "allocated_GB": lay_["pool_allocated_GB"],
                    "command": "bench.py --layout %s --no-extra-legs --steps 5 --warmup 2" % lay}
                log("  %-44s %8.3f ms  %7.1f GB/s  %5.1f %% of peak  (%.1f GB allocated)"
                    % (label, roof_["avg_launch_ms"], roof_["achieved"], 100 * roof_["frac"], lay_["pool_allocated_GB"]))
            except Exception as exc:                                  # a leg, not the measurement: report and go on
                log("  %s leg skipped: %r" % (lay, exc))
        result["legs"] = legs
        if psgd.device_status() != 0:
            log("bench.py: a kernel flagged an invalid mixing table")
            sys.exit(4)
    else:
        del X, Y, Gs, X_prev, views, pool
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl)
        log("cpu baseline (dense oracle): %.3g updates/s on %d threads" % (result["cpu_baseline"]["value"],
                                                                           result["cpu_baseline"]["cores"]))
        try:
            result["cpu_baseline_sparse"] = cpu_baseline_sparse(wl)
            sp = result["cpu_baseline_sparse"]
            log("cpu baseline (sparse C oracle): %.3g updates/s on 1 thread, %.3g on %d threads"
                % (sp["single_thread"]["value"], sp["all_cores"]["value"], sp["all_cores"]["cores"]))
        except Exception as e:                      # no host C compiler on the box: the dense oracle stands alone
            log("sparse CPU baseline skipped: %s" % (str(e).splitlines()[0] if str(e) else type(e).__name__))
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
