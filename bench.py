#!/usr/bin/env python3
"""Benchmark of the whole hot path (pard_estimate_drop + pard_compact) on one MI355X.

One step = one pass of the path over one batch of synthetic snapshots that is already
resident in HBM.  Prints ONE JSON line: requests evaluated per second, the roofline
figures of the dominant kernel (measured live with HIP events on the launch stream) and
the CPU oracle timed on the host cores beside it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth

# Algorithmic bytes per request of the estimate+drop call:
#   read deadline 4 + stage 4 (+ arrival 4 under FCFS); write est 4 + drop 1 + order 4.
# On-chip path (snapshots <= 8192 requests): that is all, 17 B/request.
# Radix-sort path: + count pass 8, histogram pass 8, (passes-1) * 16 for the key/index
# ping-pong, + 8 for the epilogue's read of the sorted pairs.
def estimate_drop_bytes_per_request(fused: bool, passes: int, fcfs: bool) -> float:
    io = 8 + 9 + (4 if fcfs else 0)
    if fused:
        return float(io)
    return float(io + 8 + 8 + 16 * (passes - 1) + 8 + 8)   # last +8: final pass writes pairs


def recorded_traffic(workload_cfg: int, kernel: str, source: str):
    """HBM bytes per launch of `kernel` taken from the committed rocprofv3 counter summary,
    or None when there is none for this workload or the kernel source changed since."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_cfg{workload_cfg}.txt")
    try:
        sha = hashlib.sha256(open(os.path.join(ROOT, "paper_2602_08747_amd", "csrc", source), "rb").read()).hexdigest()[:16]
        for line in open(path):
            f = line.split()
            if len(f) == 5 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel and f[3] == "source_sha256":
                return int(f[2]) if f[4] == sha else None
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (default: the largest)")
    ap.add_argument("--permute", action="store_true", help="shuffle request order inside every snapshot")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (snapshots would shard across GPUs with no "
              "communication, see DESIGN.md); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_08747_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load_library()

    t0 = time.time()
    w = workloads.make_workload(args.config, permute=args.permute)
    gen_s = time.time() - t0
    s = binding.Session(w)
    fused = s.max_snap <= binding.PARD_FUSED_SNAPSHOT_CAPACITY
    n = w.n

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # one dispatch that reads and writes exactly this many bytes
        torch.cuda.synchronize()
        del src, dst

    for _ in range(max(args.warmup, 1)):
        s.run()
    torch.cuda.synchronize()

    # timed region: exactly --steps passes of the whole path
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b, c in ev:
        a.record()
        s.estimate_drop()
        b.record()
        s.compact()
        c.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    est_ms = float(np.mean([a.elapsed_time(b) for a, b, _ in ev]))
    cmp_ms = float(np.mean([b.elapsed_time(c) for _, b, c in ev]))

    res = s.results()
    drop_frac = float(res["drop"].mean()) if n else 0.0
    status = s.status_word()

    # roofline of the dominant kernel
    fcfs = bool((w.order_mode == workloads.MODE_FCFS).any())
    if fused:
        kernel = "fused_snapshot_kernel (whole pard_estimate_drop call: one launch)"
        passes = 0
    else:
        kernel = "pard_estimate_drop call (count, setup, histogram, radix passes, epilogue)"
        span = int(w.deadline.max()) - int(w.deadline.min()) if n else 0
        passes = max(1, -(-(max(span, 0).bit_length() + max(w.K * w.S - 1, 0).bit_length()) // 8))
    bpr = estimate_drop_bytes_per_request(fused, passes, fcfs)
    alg_bytes = bpr * n
    achieved = alg_bytes / (est_ms * 1e-3) / 1e9 if est_ms > 0 else 0.0
    traffic = recorded_traffic(args.config, "fused_snapshot_kernel", "pard_fused.hip") if fused and not args.permute else None
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "kernel": kernel, "bytes_per_request": bpr, "launch_ms": round(est_ms, 4)}

    out = {
        "metric": "requests evaluated/sec (estimate+drop+compact)",
        "value": round(n / (ms_per_step * 1e-3), 1),
        "unit": "requests/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name, "requests": n, "snapshots": w.K, "stages": w.S,
                   "path": "on-chip" if fused else "radix-sort", "radix_passes": passes,
                   "drop_fraction": round(drop_frac, 4), "status_word": status,
                   "estimate_drop_ms": round(est_ms, 4), "compact_ms": round(cmp_ms, 4),
                   "generate_s": round(gen_s, 2)},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        import oracle
        threads = min(os.cpu_count() or 1, 16)
        # the oracle finishes the whole workload in seconds, so the sample is the whole workload
        sub = w
        sample = f"whole workload ({n} requests), 1 run"
        oracle.build_oracle()
        t0 = time.perf_counter()
        oracle.run(sub, threads=threads)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(sub.n / cpu_s, 1), "unit": "requests/s", "cores": threads,
                               "kind": "oracle", "sample": sample, "seconds": round(cpu_s, 3)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
