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

Prints ONE JSON line on stdout; progress and per-kernel detail go to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the (fused) mix kernel from two rocprofv3 --pmc runs (FETCH_SIZE,
# then WRITE_SIZE, in KiB per dispatch), each scaled by the same counter's reading for a plain
# device copy of known size (--calibrate-copy): FETCH_SIZE reads half the true bytes on this
# chip (factor 2.000), WRITE_SIZE reads them all (factor 1.000).  Workloads not yet measured
# report null.
MEASURED_TRAFFIC_BYTES = {
    ("cfg5_n64_d100M_bf16g_randring", "ring"): (18_750_609 * 2.000 + 25_000_166 * 1.000) * 1024,
    ("cfg5_n64_d100M_bf16g_randring", "degree5"): (18_751_856 * 2.000 + 25_000_067 * 1.000) * 1024,
    ("cfg5_n64_d100M_bf16g_randring", "degree9"): (18_750_863 * 2.000 + 25_000_033 * 1.000) * 1024,
    ("cfg5_n64_d100M_bf16g_randring", "full"): (18_750_535 * 2.000 + 25_000_558 * 1.000) * 1024,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(wl, seconds_budget=20.0):
    """The oracle as it stands, timed on the host: whole hot-path step (dense-matrix update
    in fp64 + two-pass consensus distance) on a column slice of the same workload."""
    import numpy as np
    from oracle import psgd_oracle as orc
    from paper_2002_01119_amd import inputs as inp
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
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
    ap.add_argument("--device-tables", action="store_true",
                    help="build each iteration's table on the device (psgd_build_mixing_device) instead of on the "
                         "host followed by an upload")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed region, capture the same K steps (tables built on the device from a device-side "
                         "iteration counter) in ONE HIP graph, replay it, and report its time per step beside the eager one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layout", choices=["pitched", "probe", "dense"], default="pitched",
                    help="where the arrays live in HBM: 'pitched' interleaves the rows of all arrays across most of "
                         "the device (psgd_mix_step_ex), 'probe' keeps dense arrays but places X / X_out on the "
                         "windows of one pool where the step runs fastest, 'dense' is one plain tensor per array")
    ap.add_argument("--span-fraction", type=float, default=0.65,
                    help="pitched layout: fraction of device memory the row slots are spread over")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the warm-up, run a plain dense device copy of known size (printed); under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate the mix kernel's")
    args = ap.parse_args()
    if args.degree < 3 or args.degree % 2 == 0 or (args.degree > 3 and (args.global_average or args.device_tables)):
        log("bench.py: --degree takes an odd K >= 3 and excludes --global-average and --device-tables")
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
    from paper_2002_01119_amd import inputs as inp
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

    # ---- resident inputs
    n_xbuf = 1 if args.in_place else (3 if wl.delay else 2)
    gdt = torch.bfloat16 if wl.g_dtype == "bf16" else torch.float32
    layout_report, pool, views = {"layout": args.layout}, None, None

    def draw_g(i):
        return (inp.device_normal_bf16 if wl.g_dtype == "bf16" else inp.device_normal_f32)(
            (n, d), wl.sigma_g, wl.seed_g + i, dev)

    if args.layout == "pitched":
        # Rows of every array interleaved across most of the HBM (see placement.pitched_layout):
        # slot i = [X_i | Y_i | (Xprev_i) | G0_i | G1_i | (noise_i)], slots `pitch` bytes apart.
        from paper_2002_01119_amd import placement as plc
        free, total_mem = torch.cuda.mem_get_info()
        specs = [("X", torch.float32)] + ([] if args.in_place else [("Y", torch.float32)])
        if wl.delay:
            specs += [("Xprev", torch.float32), ("noise", torch.float32)]
        specs += [("G0", gdt), ("G1", gdt)]
        span = min(int(args.span_fraction * total_mem), free - (8 << 30))
        try:
            views, pool, pitch = plc.pitched_layout(n, d, specs, span, dev)
            layout_report.update({"pitch_GB": pitch / 1e9, "span_GB": pool.numel() / 1e9,
                                  "arrays": [s_[0] for s_ in specs]})
            log("pitched layout: %d slots %.3f GB apart, pool %.1f GB" % (n, pitch / 1e9, pool.numel() / 1e9))
        except torch.OutOfMemoryError:
            log("pitched layout does not fit; falling back to dense tensors")
            views, layout_report = None, {"layout": "dense (pitched did not fit)"}
        if views is not None:
            X = inp.fill_normal_rows_(views["X"], wl.sigma_x, wl.seed_x)
            Y = X if args.in_place else views["Y"]
            Gs = [inp.fill_normal_rows_(views["G%d" % i], wl.sigma_g, wl.seed_g + i) for i in range(2)]
    elif args.layout == "probe":
        # X and X_out are rewritten every step: put them where this chip writes fastest
        from paper_2002_01119_amd import placement as plc
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
        X_prev.copy_(X)
    deg = args.degree
    if deg > min(n, 32) or n * deg > 4096:
        log("bench.py: --degree %d does not fit n = %d" % (deg, n))
        sys.exit(2)
    nbr_host = torch.empty((total, n, deg), dtype=torch.int32, pin_memory=True)
    w_host = torch.empty((total, n, deg), dtype=torch.float32, pin_memory=True)
    nbr_dev = torch.empty((total, n, deg), dtype=torch.int32, device=dev)
    w_dev = torch.empty((total, n, deg), dtype=torch.float32, device=dev)
    cdist = torch.zeros(total, dtype=torch.float64, device=dev)
    stream = torch.cuda.Stream(device=dev)
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(total)]
    stream2 = torch.cuda.Stream(device=dev)
    ev_prod = [torch.cuda.Event() for _ in range(total + 1)]
    if wl.delay and args.overlap:
        psgd.synth_grad(X_prev, noise, Gs[0], wl.grad_pull, stream=stream2)      # G_0 from X_{-1} = X_0
        ev_prod[0].record(stream2)
    torch.cuda.synchronize()

    def widen(nbr3):
        """K-slot table on the same ring: follow the right (left) pointers (K-1)/2 times."""
        left, right = nbr3[:, 1], nbr3[:, 2]
        cols, lo, hi = [nbr3[:, 0]], nbr3[:, 0], nbr3[:, 0]
        for _ in range((deg - 1) // 2):
            lo, hi = left[lo], right[hi]
            cols += [lo, hi]
        return (np.ascontiguousarray(np.stack(cols, axis=1), dtype=np.int32),
                np.full((n, deg), 1.0 / deg, dtype=np.float32))

    def one_step(k):
        nonlocal X, Y, X_prev
        if args.device_tables:
            psgd.build_mixing_device(wl.topology, n, wl.seed_perm, nbr_dev[k], w_dev[k], step_offset=k, stream=stream)
        else:
            nbr, w = psgd.build_mixing(wl.topology, n, wl.seed_perm, k)
            if deg > 3:
                nbr, w = widen(nbr)
            nbr_host[k].copy_(torch.from_numpy(nbr))
            w_host[k].copy_(torch.from_numpy(w))
            nbr_dev[k].copy_(nbr_host[k], non_blocking=True)
            w_dev[k].copy_(w_host[k], non_blocking=True)
        G = Gs[k % 2]
        overlap = wl.delay and args.overlap
        if overlap:
            stream.wait_event(ev_prod[k])                    # G_k was produced on the second stream
        elif wl.delay:
            psgd.synth_grad(X_prev, noise, G, wl.grad_pull, stream=stream)
        fused = not (args.unfused or args.no_consensus)
        ev0[k].record(stream)
        if args.global_average:
            psgd.mix_full(X, Y, G, wl.lr, delay_mode=1 if wl.delay else 0, stream=stream,
                          cdist_out=cdist[k:k + 1] if fused else None)
        else:
            psgd.mix_step(X, Y, G, nbr_dev[k], w_dev[k], wl.lr, delay_mode=1 if wl.delay else 0, stream=stream,
                          cdist_out=cdist[k:k + 1] if fused else None)
        ev1[k].record(stream)
        if not (fused or args.no_consensus):
            psgd.consensus_dist_async(Y, cdist[k:k + 1], stream=stream)
        ev2[k].record(stream)
        if overlap and k + 1 < total:
            # producer of G_{k+1} = c * X_k + noise: needs X_k (complete since step k-1) and the gradient
            # buffer that step k-1 read; runs beside the mix of step k, which only reads X_k
            if k > 0:
                stream2.wait_event(ev2[k - 1])
            psgd.synth_grad(X, noise, Gs[(k + 1) % 2], wl.grad_pull, stream=stream2)
            ev_prod[k + 1].record(stream2)
        if wl.delay:
            X_prev, X, Y = X, Y, X_prev
        elif not args.in_place:
            X, Y = Y, X

    with torch.cuda.stream(stream):
        if args.calibrate_copy:
            cal_bytes = min(12_800_000_000, torch.cuda.mem_get_info()[0] // 3) // 4096 * 4096
            ca = torch.zeros(cal_bytes, dtype=torch.uint8, device=dev)
            cb = torch.empty_like(ca)
            cb.copy_(ca)
            t_c0, t_c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t_c0.record(stream)
            cb.copy_(ca)
            t_c1.record(stream)
            torch.cuda.synchronize()
            cms = t_c0.elapsed_time(t_c1)
            log("calibration: plain dense device copy of %d bytes (= %d KiB read and as many written): %.3f ms -> "
                "%.1f GB/s (%.1f %% of peak)" % (cal_bytes, cal_bytes // 1024, cms, 2 * cal_bytes / cms / 1e6,
                                                 2 * cal_bytes / cms / 1e6 / HBM_PEAK_GBS * 100))
            del ca, cb
        for k in range(W):
            one_step(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(W, total):
            one_step(k)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
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
    bytes_per_update = 10 if wl.g_dtype == "bf16" else 12       # X read + G read + X_out write
    mix_bytes = bytes_per_update * n * d
    achieved = mix_bytes / (mix_avg * 1e-3) / 1e9
    cvals = cdist.cpu().numpy()
    log("mix kernel: avg %.3f ms (min %.3f, max %.3f) -> %.1f GB/s algorithmic, %.1f %% of %d GB/s"
        % (mix_avg, min(mix_ms), max(mix_ms), achieved, 100 * achieved / HBM_PEAK_GBS, HBM_PEAK_GBS))
    fused = not (args.unfused or args.no_consensus)
    if fused:
        log("consensus distance is fused into the mix kernel; final reduce kernel avg %.4f ms" % con_avg)
        log("consensus distance after the timed steps: first %.6g last %.6g" % (cvals[W], cvals[-1]))
    elif not args.no_consensus:
        cgb = 4 * n * d / (con_avg * 1e-3) / 1e9
        log("consensus kernels: avg %.3f ms -> %.1f GB/s algorithmic (4 B/element), %.1f %% of peak"
            % (con_avg, cgb, 100 * cgb / HBM_PEAK_GBS))
        log("consensus distance after the timed steps: first %.6g last %.6g" % (cvals[W], cvals[-1]))
    log("whole step: %.3f ms wall per step over %d steps" % (1e3 * wall / K, K))

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
            "topology": "full (T_u)" if args.global_average else {0: "ring", 1: "rand_ring"}[wl.topology],
            "table_degree": deg, "tables_built_on": "device" if args.device_tables else "host",
            "lr": wl.lr,
            "delay_by_one": wl.delay, "consensus_every_step": not args.no_consensus,
            "consensus_fused_into_mix_kernel": fused,
            "in_place": bool(args.in_place), "producer_overlapped": bool(wl.delay and args.overlap),
            "hbm_layout": layout_report,
        },
        "roofline": {
            "kernel": ("mix_full_kernel" if args.global_average else "mix_deg_kernel" if deg > 3
                       else "mix_step_kernel")
                      + (" (with fused consensus statistics)" if fused else ""),
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(
                (wl.name, "full" if args.global_average else "ring" if deg == 3 else "degree%d" % deg)),
            "algorithmic_bytes_per_launch": mix_bytes, "avg_launch_ms": mix_avg,
        },
        "mix_updates_per_s": n * d / (mix_avg * 1e-3),
    }
    if graph_report is not None:
        result["hip_graph"] = graph_report
    if not (args.no_consensus or fused):
        result["consensus"] = {"avg_ms": con_avg, "achieved_GBps": 4 * n * d / (con_avg * 1e-3) / 1e9,
                               "frac": 4 * n * d / (con_avg * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del X, Y, Gs, X_prev, views, pool
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl)
        log("cpu baseline: %.3g updates/s on %d threads" % (result["cpu_baseline"]["value"],
                                                            result["cpu_baseline"]["cores"]))
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
