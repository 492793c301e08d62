"""Benchmark of the Global-QSGD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]

A step is one pass of the whole path over one batch of K resident synthetic gradients:
global_norm -> fused quantize+aggregate (quantisation of all workers and the integer sum, in
registers) -> dequantize.  HIP events on the launch stream bracket the timed steps and each call
inside them.  One JSON line is printed:

  value      the headline metric: algorithmic GB/s of the fused quantize+aggregate call
             (4K bytes read + 4 bytes written per output coordinate, divided by the call's mean
             duration inside the timed steps), inputs resident in HBM
  roofline   the same kernel against MI355X's 8 TB/s HBM peak; `traffic` is the HBM byte count per
             launch from rocprofv3 FETCH_SIZE/WRITE_SIZE counters (read from profiles/, null if absent)
  step_*     the whole step: ms, algorithmic bytes, GB/s
  cpu_baseline  the CPU oracle (as it stands) on a bounded sample of the same buffers
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X: 8 TB/s HBM3E (published peak)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "fused_quantize_aggregate_c3_traffic_figures.txt")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--rows", action="store_true",
                    help="also time every entry point on its own (quantize per worker, int_aggregate, "
                         "dequantize, fused variants) and report them under \"rows\"")
    ap.add_argument("--cpu-sample", type=int, default=1 << 26, help="coordinates per worker timed on the CPU oracle")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, run three plain 1 GiB device copies (a kernel of known "
                         "traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-bucket-norm", action="store_true",
                    help="bucketed workloads (c5): every bucket under its OWN norm (gq_bucketed_quantize_aggregate), "
                         "timed with the serial schedule and with the next bucket's norm on a second stream; "
                         "both step times are reported under \"per_bucket_norm\"")
    ap.add_argument("--two-streams", action="store_true",
                    help="with --per-bucket-norm: the headline ms_per_step is the two-stream schedule (default: serial)")
    ap.add_argument("--no-window-ab", action="store_true",
                    help="skip the interleaved timing of the fused call with its write windows forced off and on")
    ap.add_argument("--norm", default=None, choices=["linf", "l2"],
                    help="override the workload's norm (c3 under the L2 norm is the low-density case of the sparse branch)")
    ap.add_argument("--windows", default="default", choices=["default", "on", "off"],
                    help="write windows of the fused call in the timed steps: the library's policy, forced on, or forced off "
                         "(gq_params.flags); for profiling one variant at a time")
    ap.add_argument("--ab-rounds", type=int, default=15, help="rounds of the write-window A/B (each times off, then on)")
    ap.add_argument("--workers", type=int, default=None,
                    help="override the workload's worker count K (1..64): the same value distribution at another shape, for sweeps")
    ap.add_argument("--coords", type=int, default=None,
                    help="override the workload's coordinates per worker d (not for the bucketed workload)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture the step in a HIP graph and time its replays (reported as graph_replay_ms_per_step)")
    return ap.parse_args()


def cpu_baseline(xs, nf, scheme, s, seed, sample, bytes_per_coord):
    """The oracle's quantize+sum on the first `sample` coordinates of every worker, split over
    host threads (the C routine runs without the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import gq_oracle as O
    d = xs[0].numel()
    sample = min(sample, d)
    host = [x[:sample].cpu().numpy() for x in xs]
    # every host core this job may use: a GPU machine gives a one-GPU job a share of 16 cores whatever
    # os.cpu_count() shows there (OMP_NUM_THREADS carries that share)
    share = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    threads = max(1, min(os.cpu_count() or 1, share if share > 0 else 16))
    per = (sample + threads - 1) // threads
    per = (per + 3) & ~3
    cuts = [(lo, min(sample, lo + per)) for lo in range(0, sample, per)]

    def work(c):
        lo, hi = c
        return O.quantize_aggregate([h[lo:hi] for h in host], nf, scheme, s, seed, lo)

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(work, cuts))
    dt = time.perf_counter() - t0
    # and on one thread, on a sixteenth of the sample
    one = max(4, (sample // 16) & ~3)
    t1 = time.perf_counter()
    O.quantize_aggregate([h[:one] for h in host], nf, scheme, s, seed, 0)
    dt1 = time.perf_counter() - t1
    return {
        "value": sample * bytes_per_coord / dt * 1e-9, "unit": "GB/s", "cores": min(threads, len(cuts)),
        "kind": "oracle", "seconds": dt, "coords_per_s": sample / dt,
        "sample": "first %d of %d coordinates of all %d workers (same buffers, same accounting)" % (sample, d, len(xs)),
        "single_thread": {"value": one * bytes_per_coord / dt1 * 1e-9, "unit": "GB/s", "coords_per_s": one / dt1,
                          "seconds": dt1, "sample": "first %d coordinates of all %d workers" % (one, len(xs))},
    }, parts, cuts


def time_rows(gq, torch, xs, norm, params, cfg, args):
    """Every entry point on its own, in the workload's own formats: algorithmic GB/s from HIP events."""
    K, d = len(xs), xs[0].numel()
    dev = xs[0].device
    pack = {"i8": gq.GQ_PACK_I8, "i4": gq.GQ_PACK_I4, "u8s": gq.GQ_PACK_U8_SIGNPLANE, "u4s": gq.GQ_PACK_U4_SIGNPLANE}[cfg["pack"]]
    aggf = gq.GQ_AGG_I16 if cfg["agg"] == "i16" else gq.GQ_AGG_I32
    p = gq.make_params(params.scheme, params.s, pack, aggf, seed=params.seed)
    bits = 4 if pack in (gq.GQ_PACK_I4, gq.GQ_PACK_U4_SIGNPLANE) else 8
    plane = pack >= gq.GQ_PACK_U8_SIGNPLANE
    abytes = 2 if aggf == gq.GQ_AGG_I16 else 4
    lvs = [torch.empty(gq.levels_nbytes(d, pack), dtype=torch.uint8, device=dev) for _ in range(K)]
    sps = [torch.empty(gq.signplane_nwords(d), dtype=torch.int32, device=dev) for _ in range(K)] if plane else None
    agg = torch.empty(d, dtype=torch.int16 if abytes == 2 else torch.int32, device=dev)
    out = torch.empty(d, dtype=torch.float32, device=dev)
    lvb = bits / 8.0 + (1.0 / 8.0 if plane else 0.0)

    def timed(fn, nbytes):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(max(5, args.steps // 2)):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record(); b.synchronize()
            ts.append(a.elapsed_time(b))
        ms = sum(ts) / len(ts)
        return {"ms": ms, "min_ms": min(ts), "GBps": nbytes / ms * 1e-6, "bytes": nbytes}

    def quantize_all():
        for i in range(K):
            gq.quantize(xs[i], norm, p, i, 0, lvs[i], sps[i] if plane else None)

    rows = {}
    rows["quantize_xK"] = timed(quantize_all, K * d * (4.0 + lvb))
    rows["int_aggregate"] = timed(lambda: gq.int_aggregate(lvs, sps, d, p, agg), d * (K * lvb + abytes))
    rows["dequantize"] = timed(lambda: gq.dequantize(agg, d, norm, p, K, out), d * (abytes + 4.0))
    rows["fused_agg"] = timed(lambda: gq.fused_quantize_aggregate(xs, norm, p, 0, agg, None), d * (4.0 * K + abytes))
    rows["fused_dequant"] = timed(lambda: gq.fused_quantize_aggregate(xs, norm, p, 0, None, out), d * (4.0 * K + 4.0))
    rows["fused_agg_levels"] = timed(lambda: gq.fused_quantize_aggregate(xs, norm, p, 0, agg, None, lvs, sps),
                                     d * (4.0 * K + K * lvb + abytes))
    # short draws: 16 random bits per coordinate, one Philox call per eight coordinates
    p16 = gq.make_params(params.scheme, params.s, pack, aggf, seed=params.seed, rng_bits=16)

    def quantize_all_16():
        for i in range(K):
            gq.quantize(xs[i], norm, p16, i, 0, lvs[i], sps[i] if plane else None)

    rows["fused_agg_rng16"] = timed(lambda: gq.fused_quantize_aggregate(xs, norm, p16, 0, agg, None), d * (4.0 * K + abytes))
    rows["quantize_xK_rng16"] = timed(quantize_all_16, K * d * (4.0 + lvb))
    if params.scheme == gq.GQ_EXP:
        # Algorithm 2 on int8 codes: reduced (sign, e) bytes and the fp32 mean; ALU-bound (K-1 Philox calls and
        # branch-free pair reductions per four coordinates), so GB/s here is far below the HBM roof by design
        p8 = gq.make_params(params.scheme, params.s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=params.seed)
        lv8 = lvs if pack == gq.GQ_PACK_I8 else [torch.empty(d, dtype=torch.uint8, device=dev) for _ in range(K)]
        if lv8 is not lvs:
            for i in range(K):
                gq.quantize(xs[i], norm, p8, i, 0, lv8[i])
        red = torch.empty(d, dtype=torch.int8, device=dev)
        rows["exp_reduce_alg2"] = timed(lambda: gq.exp_reduce(lv8, d, p8, 0, norm, red, out), d * (K + 1.0 + 4.0))
        npad = 1
        while npad < K:
            npad *= 2
        rows["exp_reduce_alg2"]["coords_per_s"] = d / rows["exp_reduce_alg2"]["ms"] * 1e3
        rows["exp_reduce_alg2"]["tree_nodes_per_coordinate"] = npad - 1
    if params.scheme == gq.GQ_LINEAR and pack in (gq.GQ_PACK_I8, gq.GQ_PACK_I4):
        # Implementation section: averaging inside every reduce step; codes in, one code vector and the fp32 mean out
        red = torch.empty(gq.levels_nbytes(d, pack), dtype=torch.uint8, device=dev)
        rows["avg_reduce_in_step"] = timed(lambda: gq.avg_reduce(lvs, d, p, 0, norm, red, out), d * (K * lvb + lvb + 4.0))
    if pack == gq.GQ_PACK_I8 and d < (1 << 32):
        # Algorithm 1's sparse branch: compaction of every worker's non-zero codes, then the sum of the K lists
        cnts = [torch.zeros(1, dtype=torch.int64, device=dev) for _ in range(K)]
        ws = torch.empty(gq.compact_workspace_bytes(d), dtype=torch.uint8, device=dev)
        probe_i = torch.empty(1, dtype=torch.int32, device=dev)
        probe_v = torch.empty(1, dtype=torch.int8, device=dev)
        for i in range(K):
            gq.compact(lvs[i], d, p, probe_i, probe_v, cnts[i], ws)
        torch.cuda.synchronize()
        nnz = [int(c.item()) for c in cnts]
        idxs = [torch.empty(max(n, 1), dtype=torch.int32, device=dev) for n in nnz]
        vals = [torch.empty(max(n, 1), dtype=torch.int8, device=dev) for n in nnz]
        tabs = [torch.empty(gq.tile_starts_len(d), dtype=torch.int32, device=dev) for _ in range(K)]

        def compact_all():
            for i in range(K):
                gq.compact(lvs[i], d, p, idxs[i], vals[i], cnts[i], ws, tile_starts_out=tabs[i])

        tot = float(sum(nnz))
        # the method's bytes: every code read once, every pair (4-byte index + 1-byte code) written once
        rows["compact_xK"] = timed(compact_all, 1.0 * K * d + 5.0 * tot)

        # the sender in one call, straight from the gradients: 4 bytes read per coordinate, 5 written per non-zero
        def quantize_compact_all():
            for i in range(K):
                gq.quantize_compact(xs[i], norm, p, i, 0, idxs[i], vals[i], cnts[i], ws, tile_starts_out=tabs[i])

        rows["quantize_compact_xK"] = timed(quantize_compact_all, 4.0 * K * d + 5.0 * tot)
        rows["quantize_compact_xK"]["two_calls_ms"] = rows["quantize_xK"]["ms"] + rows["compact_xK"]["ms"]
        if aggf == gq.GQ_AGG_I32:
            # with the senders' tables of tile starts, and without them (the receiver then searches the lists)
            rows["sparse_aggregate"] = timed(lambda: gq.sparse_aggregate(idxs, vals, cnts, d, p, agg, tile_starts=tabs), 4.0 * d + 5.0 * tot)
            rows["sparse_aggregate_searching"] = timed(lambda: gq.sparse_aggregate(idxs, vals, cnts, d, p, agg), 4.0 * d + 5.0 * tot)
        rows["nonzero_fraction"] = tot / (float(K) * d)
        if cfg["norm"] == "l2":
            # Theorem 1's regime: the bound on the expected count that the lists can be sized by
            rows["nonzero_fraction_bound"] = gq.sparse_nnz_bound(p, K, d) / (float(K) * d)
    rows["formats"] = {"pack": cfg["pack"], "agg": cfg["agg"]}
    return rows


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the K workers are K resident buffers); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2305_18627_amd as gq
    import synth_inputs as SI

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = SI.CONFIGS[args.workload]
    K, d, s = cfg["K"], cfg["d"], cfg["s"]
    own_shape = args.workers is None and args.coords is None
    if not own_shape:
        if cfg.get("bucket") and args.coords is not None:
            print("bench.py: --coords is not offered for the bucketed workload", file=sys.stderr)
            sys.exit(2)
        K = args.workers if args.workers is not None else K
        d = args.coords if args.coords is not None else d
        if not (1 <= K <= 64) or d < 1:
            print("bench.py: --workers must lie in 1..64 and --coords be positive", file=sys.stderr)
            sys.exit(2)
    scheme = gq.GQ_LINEAR if cfg["scheme"] == "linear" else gq.GQ_EXP
    if args.norm:
        cfg = dict(cfg, norm=args.norm)
    kind = {"linf": gq.GQ_NORM_LINF, "l2": gq.GQ_NORM_L2}[cfg["norm"]]
    win_flags = {"default": 0, "on": gq.GQ_FLAG_WRITE_WINDOWS_ON, "off": gq.GQ_FLAG_WRITE_WINDOWS_OFF}[args.windows]
    params = gq.make_params(scheme, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED, flags=win_flags)

    xs = SI.make_workers(args.workload, d=d, K=K, device=dev)
    norm = torch.zeros(1, device=dev)
    flags = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(gq.norm_workspace_bytes(K, d), dtype=torch.uint8, device=dev)
    agg = torch.empty(0 if cfg.get("bucket") else d, dtype=torch.int32, device=dev)
    out = torch.empty(d, dtype=torch.float32, device=dev)

    bucket = cfg.get("bucket")
    views = None
    if bucket:      # bucketed workload: per bucket one fused quantize+aggregate+dequantize call, offsets passed on
        views = [(lo, [x[lo:min(d, lo + bucket)] for x in xs], out[lo:min(d, lo + bucket)]) for lo in range(0, d, bucket)]

    per_bucket = bool(bucket) and args.per_bucket_norm
    if args.per_bucket_norm and not bucket:
        print("bench.py: --per-bucket-norm needs a bucketed workload (c5)", file=sys.stderr)
        sys.exit(2)
    side = torch.cuda.Stream() if per_bucket else None          # default priority, like the main stream
    if per_bucket:
        nbk = SI.num_buckets(d, bucket)
        norms_b = torch.zeros(nbk, device=dev)
        flags_b = torch.zeros(nbk, dtype=torch.int32, device=dev)
        ws_b = torch.empty(gq.bucketed_workspace_bytes(K, d, bucket), dtype=torch.uint8, device=dev)

    def bucketed_step(two_streams):
        gq.bucketed_quantize_aggregate(xs, bucket, kind, params, norms_b, flags_b, None, out, ws_b,
                                       side_stream=side if two_streams else None)

    def step(ev=None):
        if per_bucket:
            # norm and fused calls alternate bucket by bucket inside one library call: only the whole step is timed
            if ev: ev[0].record(); ev[1].record()
            bucketed_step(args.two_streams)
            if ev: ev[2].record(); ev[3].record()
            return
        if ev: ev[0].record()
        gq.global_norm(xs, kind, norm, flags, ws)
        if ev: ev[1].record()
        if bucket:
            for lo, xv, ov in views:
                gq.fused_quantize_aggregate(xv, norm, params, lo, None, ov)
            if ev: ev[2].record()
        else:
            gq.fused_quantize_aggregate(xs, norm, params, 0, agg, None)
            if ev: ev[2].record()
            gq.dequantize(agg, d, norm, params, K, out)
        if ev: ev[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    total_ms = evs[0][0].elapsed_time(evs[-1][3])
    t_norm = [e[0].elapsed_time(e[1]) for e in evs]
    t_fused = [e[1].elapsed_time(e[2]) for e in evs]
    t_deq = [e[2].elapsed_time(e[3]) for e in evs]
    ms_per_step = total_ms / args.steps

    # algorithmic bytes: what the method must move (every gradient coordinate read once per pass)
    b_norm = 4.0 * K * d
    b_fused = (4.0 * K + 4.0) * d
    b_deq = 0.0 if bucket else 8.0 * d
    fused_ms = float(np.mean(t_fused)) if not per_bucket else ms_per_step
    fused_gbps = b_fused / fused_ms * 1e-6
    step_gbps = (b_norm + b_fused + b_deq) / ms_per_step * 1e-6

    def time_calls(fn, n):
        ts = []
        for _ in range(n):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record(); b.synchronize()
            ts.append(a.elapsed_time(b))
        return ts

    schedules = None
    if per_bucket:
        # both schedules of the per-bucket-norm step, interleaved in this warmed-up process
        ser, two = [], []
        for _ in range(max(3, args.steps // 2)):
            ser += time_calls(lambda: bucketed_step(False), 1)
            two += time_calls(lambda: bucketed_step(True), 1)
        schedules = {"serial_ms": float(np.mean(ser)), "two_streams_ms": float(np.mean(two)),
                     "serial_min_ms": float(np.min(ser)), "two_streams_min_ms": float(np.min(two)),
                     "headline": "two_streams" if args.two_streams else "serial", "buckets": nbk,
                     "algorithmic_bytes": (8.0 * K + 4.0) * d,
                     "note": "norm of bucket b+1 on a second stream beside the fused call of bucket b; identical outputs"}

    windows_ab = None
    if not bucket and not args.no_window_ab:
        # the fused call with its write windows forced off and forced on, interleaved, same buffers, same process
        p_off = gq.make_params(scheme, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED, flags=gq.GQ_FLAG_WRITE_WINDOWS_OFF)
        p_on = gq.make_params(scheme, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED, flags=gq.GQ_FLAG_WRITE_WINDOWS_ON)
        t_off, t_on = [], []
        for _ in range(args.ab_rounds):
            t_off += time_calls(lambda: gq.fused_quantize_aggregate(xs, norm, p_off, 0, agg, None), 1)
            t_on += time_calls(lambda: gq.fused_quantize_aggregate(xs, norm, p_on, 0, agg, None), 1)
        by_policy = K >= 8 and float(K) * d >= 2.5e8
        windows_ab = {"windows_off_ms": float(np.mean(t_off)), "windows_on_ms": float(np.mean(t_on)),
                      "windows_off_median_ms": float(np.median(t_off)), "windows_on_median_ms": float(np.median(t_on)),
                      "rounds": args.ab_rounds,
                      "headline_used": ("windows_" + args.windows) if args.windows != "default" else ("windows_on" if by_policy else "windows_off"),
                      "note": "interleaved off/on calls after the timed steps; the headline is the library's default policy"}

    traffic = valu_busy = traffic_note = None
    if args.workload == "c3" and own_shape and os.path.exists(TRAFFIC_FILE):
        # rocprofv3 cannot run inside this process: the HBM byte counts were profiled offline, and the file says on
        # which library version; figures of another version are not reported
        try:
            prof = json.load(open(TRAFFIC_FILE))
            if prof.get("library_version") == gq.version():
                traffic = prof.get("hbm_bytes_per_launch")
                valu_busy = prof.get("valu_busy_frac")          # from the SQ counters of the same command
                traffic_note = "profiled offline with rocprofv3 on library version %d (%s)" % (gq.version(), prof.get("source"))
            else:
                traffic_note = ("profiles/ holds counters of library version %s, this is %d: not reported"
                                % (prof.get("library_version"), gq.version()))
        except Exception as e:
            traffic = valu_busy = None
            traffic_note = "traffic figures unreadable: %r" % (e,)

    line = {
        "metric": ("fused quantize+aggregate GB/s and % of HBM peak, d=110M K=16 fp32" if args.workload == "c3" and own_shape else
                   "fused quantize+aggregate GB/s and %% of HBM peak, workload %s (d=%d K=%d fp32)" % (args.workload, d, K)),
        "value": fused_gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: d=%d fp32 per worker, K=%d resident workers, %s, %s norm, %s dithering s=%d, "
                               "int32 integer sum" % (args.workload, d, K, cfg["dist"], cfg["norm"], cfg["scheme"], s),
                   "step": ("global_norm -> per bucket fused quantize+aggregate+dequantize" if bucket
                            else "global_norm -> fused quantize+aggregate -> dequantize"), "seed": SI.QUANT_SEED},
        "pct_of_hbm_peak": 100.0 * fused_gbps / HBM_PEAK_GBPS,
        "output_coords_per_s": d / fused_ms * 1e3,
        "roofline": {"bound": "hbm", "achieved": fused_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": fused_gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "quantize_aggregate_kernel", "algorithmic_bytes_per_launch": b_fused,
                     "avg_ms": fused_ms, "median_ms": float(np.median(t_fused)), "min_ms": float(np.min(t_fused)),
                     "valu_busy_frac_profiled": valu_busy, "traffic_note": traffic_note},
        "step_GBps": step_gbps, "step_algorithmic_bytes": b_norm + b_fused + b_deq, "wall_ms_per_step": wall_ms / args.steps,
        "calls_ms": {"global_norm": float(np.mean(t_norm)), "fused_quantize_aggregate": fused_ms,
                     "dequantize": float(np.mean(t_deq))},
        "buckets": len(views) if views else None,
        "calls_GBps": {"global_norm": b_norm / max(float(np.mean(t_norm)), 1e-9) * 1e-6, "fused_quantize_aggregate": fused_gbps,
                       "dequantize": (b_deq / max(float(np.mean(t_deq)), 1e-9) * 1e-6) if b_deq else None},
        "norm_flags": int(flags.item()),
    }
    if windows_ab:
        line["roofline"].update(windows_ab)
    if schedules:
        line["per_bucket_norm"] = schedules
        line["config"]["step"] = "per bucket: global_norm of the bucket -> fused quantize+aggregate+dequantize (%s schedule)" % schedules["headline"]
        line["calls_ms"] = {"bucketed_quantize_aggregate": ms_per_step}
        line["calls_GBps"] = {"bucketed_quantize_aggregate": schedules["algorithmic_bytes"] / ms_per_step * 1e-6}
        line["value"] = line["calls_GBps"]["bucketed_quantize_aggregate"]
        line["metric"] = "per-bucket norm + fused quantize+aggregate+dequantize GB/s, workload %s (d=%d K=%d fp32)" % (args.workload, d, K)
        line["pct_of_hbm_peak"] = 100.0 * line["value"] / HBM_PEAK_GBPS
        line["roofline"] = {"bound": "hbm", "achieved": line["value"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": line["value"] / HBM_PEAK_GBPS, "traffic": None,
                            "kernel": "norm_tile_kernel + quantize_aggregate_kernel per bucket",
                            "algorithmic_bytes_per_launch": schedules["algorithmic_bytes"]}
        line["norm_flags"] = int(flags_b.max().item())
    if 4.0 * K * d <= 256e6:
        line["config"]["note"] = ("the inputs (%.0f MB) fit the 256 MB last-level cache and every call is launch-bound: "
                                  "not an HBM figure" % (4.0 * K * d / 1e6))
    if args.graph:
        # the calls only enqueue (no allocation, no synchronisation), so the step can be captured once and replayed:
        # what a launch-bound caller (small d) gains from that
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            g.replay()
        b.record(); b.synchronize()
        line["graph_replay_ms_per_step"] = a.elapsed_time(b) / args.steps
    if args.rows:
        line["rows"] = time_rows(gq, torch, xs, norm, params, cfg, args)
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        line["calibration_copy_bytes_each_way"] = src.numel() * 4
    if not args.no_cpu_baseline:
        # the oracle is given a norm that does not come from the library: torch's reduction of the same buffers
        if kind == gq.GQ_NORM_LINF:
            nf = np.float32(max(float(x.abs().max()) for x in xs))
        else:
            nf = np.float32(np.sqrt(sum(float((x.double() * x.double()).sum()) for x in xs)))
        base, parts, cuts = cpu_baseline(xs, nf, scheme, s, SI.QUANT_SEED, args.cpu_sample, 4.0 * K + 4.0)
        # the sample doubles as a parity check of the timed launch
        if bucket:
            base["matches_gpu"] = None          # the bucketed step stores the mean only
        else:
            # (the max norm is exact, so the timed launch used the same norm; under an L2 norm the launch is
            #  repeated with the oracle's norm before comparing)
            if np.float32(norm.item()) != nf:
                norm.fill_(float(nf))
                gq.fused_quantize_aggregate(xs, norm, params, 0, agg, None)
                torch.cuda.synchronize()
            got = agg[:cuts[-1][1]].cpu().numpy().astype(np.int64)
            base["matches_gpu"] = bool(all(np.array_equal(got[lo:hi], p) for (lo, hi), p in zip(cuts, parts)))
        base["gpu_over_cpu"] = fused_gbps / base["value"]
        line["cpu_baseline"] = base
    print(json.dumps(line))


if __name__ == "__main__":
    main()
