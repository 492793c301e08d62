"""Benchmark of the Global-QSGD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]

A step is one pass of the whole path over one batch of K resident synthetic gradients:
global_norm -> fused quantize+aggregate (quantisation of all workers and the integer sum, in
registers) -> dequantize.  HIP events on the launch stream bracket the timed steps and each call
inside them.  One JSON line is printed:

  value      the metric the benchmark spec names: algorithmic GB/s of the fused quantize+aggregate call
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "fused_quantize_aggregate_c3_traffic.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3"])
    ap.add_argument("--cpu-sample", type=int, default=1 << 26, help="coordinates per worker timed on the CPU oracle")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, run three plain 1 GiB device copies (a kernel of known "
                         "traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def cpu_baseline(xs, nf, scheme, s, seed, sample, bytes_per_coord):
    """The oracle's quantize+sum on the first `sample` coordinates of every worker, split over
    host threads (the C routine runs without the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import gq_oracle as O
    d = xs[0].numel()
    sample = min(sample, d)
    host = [x[:sample].cpu().numpy() for x in xs]
    threads = max(1, min(16, os.cpu_count() or 1))
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
    return {
        "value": sample * bytes_per_coord / dt * 1e-9, "unit": "GB/s", "cores": min(threads, len(cuts)),
        "kind": "oracle", "seconds": dt, "coords_per_s": sample / dt,
        "sample": "first %d of %d coordinates of all %d workers (same buffers, same accounting)" % (sample, d, len(xs)),
    }, parts, cuts


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
    scheme = gq.GQ_LINEAR if cfg["scheme"] == "linear" else gq.GQ_EXP
    kind = {"linf": gq.GQ_NORM_LINF, "l2": gq.GQ_NORM_L2}[cfg["norm"]]
    params = gq.make_params(scheme, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)

    xs = SI.make_workers(args.workload, device=dev)
    norm = torch.zeros(1, device=dev)
    flags = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(gq.norm_workspace_bytes(K, d), dtype=torch.uint8, device=dev)
    agg = torch.empty(d, dtype=torch.int32, device=dev)
    out = torch.empty(d, dtype=torch.float32, device=dev)

    def step(ev=None):
        if ev: ev[0].record()
        gq.global_norm(xs, kind, norm, flags, ws)
        if ev: ev[1].record()
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
    b_deq = 8.0 * d
    fused_ms = float(np.mean(t_fused))
    fused_gbps = b_fused / fused_ms * 1e-6
    step_gbps = (b_norm + b_fused + b_deq) / ms_per_step * 1e-6

    traffic = None
    if args.workload == "c3" and os.path.exists(TRAFFIC_FILE):
        try:
            traffic = json.load(open(TRAFFIC_FILE)).get("hbm_bytes_per_launch")
        except Exception:
            traffic = None

    line = {
        "metric": "fused quantize+aggregate GB/s and % of HBM peak, d=110M K=16 fp32",
        "value": fused_gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: d=%d fp32 per worker, K=%d resident workers, %s, %s norm, %s dithering s=%d, "
                               "int32 integer sum" % (args.workload, d, K, cfg["dist"], cfg["norm"], cfg["scheme"], s),
                   "step": "global_norm -> fused quantize+aggregate -> dequantize", "seed": SI.QUANT_SEED},
        "pct_of_hbm_peak": 100.0 * fused_gbps / HBM_PEAK_GBPS,
        "output_coords_per_s": d / fused_ms * 1e3,
        "roofline": {"bound": "hbm", "achieved": fused_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": fused_gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "quantize_aggregate_kernel", "algorithmic_bytes_per_launch": b_fused,
                     "avg_ms": fused_ms, "min_ms": float(np.min(t_fused))},
        "step_GBps": step_gbps, "step_algorithmic_bytes": b_norm + b_fused + b_deq, "wall_ms_per_step": wall_ms / args.steps,
        "calls_ms": {"global_norm": float(np.mean(t_norm)), "fused_quantize_aggregate": fused_ms,
                     "dequantize": float(np.mean(t_deq))},
        "calls_GBps": {"global_norm": b_norm / float(np.mean(t_norm)) * 1e-6, "fused_quantize_aggregate": fused_gbps,
                       "dequantize": b_deq / float(np.mean(t_deq)) * 1e-6},
        "norm_flags": int(flags.item()),
    }
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        line["calibration_copy_bytes_each_way"] = src.numel() * 4
    if not args.no_cpu_baseline:
        nf = np.float32(norm.item())
        base, parts, cuts = cpu_baseline(xs, nf, scheme, s, SI.QUANT_SEED, args.cpu_sample, 4.0 * K + 4.0)
        # the sample doubles as a parity check of the timed launch
        got = agg[:cuts[-1][1]].cpu().numpy().astype(np.int64)
        base["matches_gpu"] = bool(all(np.array_equal(got[lo:hi], p) for (lo, hi), p in zip(cuts, parts)))
        line["cpu_baseline"] = base
    print(json.dumps(line))


if __name__ == "__main__":
    main()
