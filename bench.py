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

INT_ALU_PEAK_TOPS = 39.3     # 256 CUs x 64 integer lanes per clock x 2.4 GHz (fp32 FMA peak 157.3 = this x 2 x 2)

# Algorithmic bytes per request of the estimate+drop call (what the method must move, not
# what this implementation moves):
#   read deadline 4 + stage 4 (+ arrival 4 under FCFS); write est 4 + drop 1 + order 4.
# On-chip path (snapshots <= 8192 requests): that is all, 17 B/request.
# Out-of-core sort with p digit passes: every pass but the last moves key + index in and
# out (16 B), the last one is read once more (8 B) and leaves the outputs:
#   8 + 16 (p - 1) + 8 + 9  B/request.
def estimate_drop_bytes_per_request(fused: bool, passes: int, fcfs: bool) -> float:
    io = 8 + 9 + (4 if fcfs else 0)
    if fused:
        return float(io)
    return float(io + 16 * (passes - 1) + 8)


def arrives_in_deadline_order(w) -> bool:
    """Whether the large-snapshot path finds the requests in deadline order and orders the queues with a stable split by
    stage instead of sorting (the library decides this on the device; this is the same rule on the host, for the label
    and the byte count of the roofline only): every stage orders by deadline the same way, at most 64 queues, no
    deadline below its predecessor inside a snapshot, and under high budget first no long run of equal deadlines.
    Under sequentially consistent dropping the split only orders the queues and the consistent kernels follow."""
    import numpy as np
    from paper_2602_08747_amd import workloads
    n = w.n
    if n == 0 or w.K * w.S > 64:
        return False
    modes = np.unique(w.order_mode)
    if len(modes) != 1 or int(modes[0]) == workloads.MODE_FCFS:
        return False
    d = w.deadline.astype(np.int64)
    falls = np.diff(d) < 0
    inner = np.asarray(w.snap_ptr[1:-1], dtype=np.int64)
    inner = inner[(inner > 0) & (inner < n)]
    falls[inner - 1] = False                       # the order may restart where a snapshot starts
    if falls.any():
        return False
    if int(modes[0]) == workloads.MODE_HBF:
        r = np.arange(32, n, 4)
        if (d[r] == d[r - 32]).any():
            return False
    return True


def usable_cores() -> int:
    """Host cores this process may use: its affinity mask, and no more than the share the machine's
    own thread-count setting (OMP_NUM_THREADS) grants a one-GPU job."""
    try:
        cores = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        cores = os.cpu_count() or 1
    share = os.environ.get("OMP_NUM_THREADS", "")
    if share.isdigit() and int(share) > 0:
        cores = min(cores, int(share))
    return max(1, cores)


def copy_calibration(torch, nbytes: int, reps: int = 5) -> float:
    """GB/s (bytes read + bytes written) of a plain device-to-device copy that moves `nbytes` in total."""
    half = max(int(nbytes) // 2, 1 << 20)
    src = torch.ones(half, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    del src, dst
    return 2.0 * half / (ms * 1e-3) / 1e9 if ms > 0 else 0.0


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


def suffix_lengths(S, row_ptr, col):
    """For one DAG: the number of later stages of every (source-to-sink path, position) pair."""
    succ = [[int(col[e]) for e in range(int(row_ptr[v]), int(row_ptr[v + 1]))] for v in range(S)]
    indeg = [0] * S
    for v in range(S):
        for t in succ[v]:
            indeg[t] += 1
    lens = []

    def walk(v, depth):
        if not succ[v]:
            lens.extend(range(depth, -1, -1))         # a path of depth+1 stages: suffixes of depth, ..., 0 stages
        for t in succ[v]:
            walk(t, depth + 1)

    for v in range(S):
        if indeg[v] == 0:
            walk(v, 0)
    return lens


def bench_planner(args, w, s, gen_s):
    """Queue lengths + L_sub (sampled variant, M = 10,000, lambda = 0.1) per step."""
    import numpy as np
    import torch
    from paper_2602_08747_amd import binding
    M, lam = 10_000, (1, 10)
    rng = np.random.default_rng([20260208, 99])
    samples = np.cumsum(np.floor(rng.exponential(20.0, M))).astype(np.int32)          # a 50k/s arrival process
    picks = rng.integers(0, 2**32, M * w.S, dtype=np.uint64).astype(np.uint32)
    d_samples = torch.from_numpy(samples).to(s.dev)
    d_picks = torch.from_numpy(picks.view(np.int32)).to(s.dev)
    for _ in range(max(args.warmup, 1)):
        s.planner(binding.SUB_FULL, lam, d_samples, d_picks)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b, c in ev:
        a.record()
        binding.pard_queue_lengths(s.plan, s.n, s.stage, s.snap_ptr, s.qlen)
        b.record()
        binding.pard_sub_latency(s.plan, s.qlen, binding.SUB_FULL, lam[0], lam[1], M, d_samples, d_picks, s.sub)
        c.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    q_ms = float(np.mean([a.elapsed_time(b) for a, b, _ in ev]))
    sub_ms = float(np.mean([b.elapsed_time(c) for _, b, c in ev]))
    # integer operations the sampling itself needs: per (path entry, sample) one draw reduced mod M,
    # one arrival reduced mod d, one complement and one add per later stage, plus three counting rounds
    D = 1 if w.dag_shared else w.K
    ops_per_sample = 0
    entries = 0
    col_base = 0
    for d in range(D):
        rp = w.dag_row_ptr[d * (w.S + 1):(d + 1) * (w.S + 1)]
        lens = suffix_lengths(w.S, rp, w.dag_col[col_base:col_base + int(rp[w.S])])
        col_base += int(rp[w.S])
        mult = w.K if w.dag_shared else 1
        entries += mult * sum(1 for x in lens if x > 0)
        ops_per_sample += mult * sum(4 * x + 3 for x in lens if x > 0)
    ops = float(ops_per_sample) * M
    achieved = ops / (sub_ms * 1e-3) / 1e12 if sub_ms > 0 else 0.0
    out = {
        "metric": "downstream-latency evaluations/sec (queue lengths + L_sub with sampled batch-wait quantile)",
        "value": round(w.K * w.S / (ms_per_step * 1e-3), 1), "unit": "snapshot-stages/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name + "+planner", "requests": w.n, "snapshots": w.K, "stages": w.S,
                   "samples": M, "lambda": "1/10", "path_entries_with_later_stages": entries,
                   "queue_lengths_ms": round(q_ms, 4), "sub_latency_ms": round(sub_ms, 4), "generate_s": round(gen_s, 2)},
        "roofline": {"bound": "alu", "achieved": round(achieved, 3), "peak": INT_ALU_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(achieved / INT_ALU_PEAK_TOPS, 4), "traffic": None,
                     "kernel": "sub_quantile_kernel (the pard_sub_latency call: fill + one launch)",
                     "ops_per_launch": ops, "launch_ms": round(sub_ms, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle
        threads = usable_cores()
        oracle.build_oracle()
        Ks = w.K if w.dag_shared else min(w.K, 64)      # bounded sample: the first snapshots
        qlen = s.qlen.cpu().numpy()
        if w.dag_shared:
            rp, cl, B, W, L = w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us
        else:
            rp = w.dag_row_ptr[:Ks * (w.S + 1)]
            ncol = int(sum(int(rp[d * (w.S + 1) + w.S]) for d in range(Ks)))
            cl, B, W, L = w.dag_col[:ncol], w.batch[:Ks * w.S], w.workers[:Ks * w.S], w.lat_us[:Ks * w.S * 64]
        t0 = time.perf_counter()
        oracle.sub_latency(Ks, w.S, w.dag_shared, rp, cl, B, W, L, qlen[:Ks * w.S], oracle.VARIANT_FULL, lam, samples, picks,
                           threads=threads)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(Ks * w.S / cpu_s, 1), "unit": "snapshot-stages/s", "cores": threads,
                               "kind": "oracle", "sample": f"first {Ks} of {w.K} snapshots, 1 run",
                               "seconds": round(cpu_s, 3)}
    return out


def bench_priority(args, w, s, gen_s):
    """Adaptive priority: 1024 rate samples per (snapshot, stage), window 50."""
    import numpy as np
    import torch
    from paper_2602_08747_amd import binding
    T, window = 1024, 50
    rng = np.random.default_rng([20260208, 98])
    latB = w.lat_us.reshape(-1, 64)[np.arange(w.batch.size), w.batch - 1].astype(np.int64)
    cap = w.workers.astype(np.int64) * w.batch * 1_000_000 // np.maximum(1, latB)
    idx = np.arange(w.K * w.S) % w.S if w.dag_shared else np.arange(w.K * w.S)
    rate = np.clip(cap[idx][:, None] * rng.uniform(0.6, 1.5, (w.K * w.S, T)), 0, 2**31 - 1).astype(np.int32)
    d_rate = torch.from_numpy(rate).to(s.dev)
    d_mode = torch.empty(w.K * w.S, dtype=torch.int32, device=s.dev)
    for _ in range(max(args.warmup, 1)):
        binding.pard_priority_modes(s.plan, T, window, d_rate, None, d_mode)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        binding.pard_priority_modes(s.plan, T, window, d_rate, None, d_mode)
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    k_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    alg_bytes = 4.0 * rate.size                       # every sample is needed once
    achieved = alg_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    out = {
        "metric": "priority decisions/sec (adaptive priority from a 1024-sample rate series per stage)",
        "value": round(w.K * w.S / (ms_per_step * 1e-3), 1), "unit": "snapshot-stages/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name + "+priority", "snapshots": w.K, "stages": w.S, "series_len": T, "window": window,
                   "hbf_fraction": round(float(d_mode.float().mean().item()), 4), "generate_s": round(gen_s, 2)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "priority_modes_kernel",
                     "bytes_per_sample": 4.0, "launch_ms": round(k_ms, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_oracle()
        Ks = w.K if w.dag_shared else min(w.K, 512)
        nrec = w.S if w.dag_shared else Ks * w.S
        t0 = time.perf_counter()
        oracle.priority_modes(Ks, w.S, w.dag_shared, w.batch[:nrec], w.workers[:nrec], w.lat_us[:nrec * 64], rate[:Ks * w.S], window)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(Ks * w.S / cpu_s, 1), "unit": "snapshot-stages/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {Ks} of {w.K} snapshots, 1 run", "seconds": round(cpu_s, 3)}
    return out


def bench_queue_delay(args, w, s, gen_s):
    """Monitored queueing delay: 1024 time-stamped delay samples per (snapshot, stage), 5 s window."""
    import numpy as np
    import torch
    from paper_2602_08747_amd import binding
    L, window = 1024, 5_000_000
    rng = np.random.default_rng([20260208, 97])
    G = w.K * w.S
    now = w.now.astype(np.int64).repeat(w.S)[:, None]
    tm = (now - rng.integers(0, 2 * window, size=(G, L))).clip(-2**31, 2**31 - 1).astype(np.int32)   # half inside the window
    dl = rng.integers(0, 400_000, size=(G, L)).astype(np.int32)
    d_time, d_delay = torch.from_numpy(tm).to(s.dev), torch.from_numpy(dl).to(s.dev)
    d_q = torch.empty(G, dtype=torch.int32, device=s.dev)
    for _ in range(max(args.warmup, 1)):
        binding.pard_queue_delay(s.plan, L, window, d_time, d_delay, s.now, d_q)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        binding.pard_queue_delay(s.plan, L, window, d_time, d_delay, s.now, d_q)
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    k_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    alg_bytes = 8.0 * tm.size                         # time and delay of every sample, once
    achieved = alg_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    out = {
        "metric": "queueing-delay estimates/sec (linearly weighted 5 s window over 1024 delay samples per stage)",
        "value": round(G / (ms_per_step * 1e-3), 1), "unit": "snapshot-stages/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name + "+queue-delay", "snapshots": w.K, "stages": w.S, "series_len": L, "window_us": window,
                   "mean_q_us": round(float(d_q.float().mean().item()), 1), "generate_s": round(gen_s, 2)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "queue_delay_kernel",
                     "bytes_per_sample": 8.0, "launch_ms": round(k_ms, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_oracle()
        Ks = min(w.K, 1024)
        t0 = time.perf_counter()
        oracle.queue_delay(Ks, w.S, tm[:Ks * w.S], dl[:Ks * w.S], w.now[:Ks], window)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(Ks * w.S / cpu_s, 1), "unit": "snapshot-stages/s", "cores": 1, "kind": "oracle",
                               "sample": f"first {Ks} of {w.K} snapshots, 1 run", "seconds": round(cpu_s, 3)}
    return out


def bench_reactive(args, w, gen_s):
    """The reactive policies of Section 5.1 on the same snapshots: window scan over the queues in arrival order
    and per-module SLO split, timed per call, and how their drop sets differ from the proactive estimate's."""
    import dataclasses
    import numpy as np
    import torch
    from paper_2602_08747_amd import binding, workloads
    s = binding.Session(w)                                      # the plan's own queue order: the proactive estimate
    s.estimate_drop()
    proactive = s.drop[:w.n].clone()
    wf = dataclasses.replace(w, order_mode=np.full_like(w.order_mode, workloads.MODE_FCFS))
    f = binding.Session(wf)                                     # the same snapshots, queues in arrival order
    f.estimate_drop()
    scan = torch.empty(max(w.n, 1), dtype=torch.uint8, device=f.dev)
    split = torch.empty_like(scan)
    first = torch.empty(w.K * w.S, dtype=torch.int32, device=f.dev)

    def window_scan():
        binding.pard_reactive_drop(f.plan, binding.REACTIVE_WINDOW_SCAN, w.n, None, f.deadline, None, None, f.now, f.order, f.seg_ptr,
                                   scan, first)

    def slo_split():
        binding.pard_reactive_drop(f.plan, binding.REACTIVE_SLO_SPLIT, w.n, f.arrival, f.deadline, f.stage, f.snap_ptr, f.now, None, None,
                                   split, None)

    for _ in range(max(args.warmup, 1)):
        window_scan()
        slo_split()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b, c in ev:
        a.record()
        window_scan()
        b.record()
        slo_split()
        c.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    scan_ms = float(np.mean([a.elapsed_time(b) for a, b, _ in ev]))
    split_ms = float(np.mean([b.elapsed_time(c) for _, b, c in ev]))
    n = max(w.n, 1)
    frac = lambda t: round(float(t.float().sum().item()) / n, 4)          # noqa: E731
    p, a, b = proactive[:w.n].bool(), scan[:w.n].bool(), split[:w.n].bool()
    alg_bytes = 9.0 * w.n                                         # order 4 + the deadline it points at 4 + the drop byte 1
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    out = {
        "metric": "requests decided/sec by the reactive policies (window scan + per-module SLO split)",
        "value": round(w.n / (ms_per_step * 1e-3), 1), "unit": "requests/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name + "+reactive", "requests": w.n, "snapshots": w.K, "stages": w.S,
                   "window_scan_ms": round(scan_ms, 4), "slo_split_ms": round(split_ms, 4),
                   "drop_fraction": {"proactive": frac(p), "window_scan": frac(a), "slo_split": frac(b)},
                   # how the drop sets differ: requests only the one or only the other policy drops, as fractions of all
                   "dropped_only_by_proactive_vs_window_scan": frac(p & ~a), "dropped_only_by_window_scan": frac(a & ~p),
                   "dropped_only_by_proactive_vs_slo_split": frac(p & ~b), "dropped_only_by_slo_split": frac(b & ~p),
                   "generate_s": round(gen_s, 2)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "the window-scan call (window_scan_kernel, window_tail_kernel, window_mask_kernel)",
                     "bytes_per_request": 9.0, "launch_ms": round(scan_ms, 4)},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_oracle()
        order, seg_ptr = f.order[:w.n].cpu().numpy(), f.seg_ptr.cpu().numpy()
        t0 = time.perf_counter()
        oracle.nexus_drop(w.K, w.S, w.dag_shared, w.batch, w.lat_us, w.deadline, order, seg_ptr, w.now)
        oracle.clipper_drop(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.lat_us, w.arrival, w.deadline, w.stage,
                            w.snap_ptr, w.now)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(w.n / cpu_s, 1), "unit": "requests/s", "cores": 1, "kind": "oracle",
                               "sample": f"whole workload ({w.n} requests), both policies, 1 run", "seconds": round(cpu_s, 3)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5 (default: the largest)")
    ap.add_argument("--permute", action="store_true", help="shuffle request order inside every snapshot")
    ap.add_argument("--snapshots", type=int, default=None,
                    help="configuration 5 only: this many snapshots instead of 4,096 (other shapes of the same sweep)")
    ap.add_argument("--per-snapshot", type=int, default=None,
                    help="configuration 5 only: this many requests per snapshot instead of 8,192")
    ap.add_argument("--half-survivors", action="store_true",
                    help="configurations 2-4 only: a labelled variant that is NOT one of the five configurations "
                         "(SLO = half the arrival span, latencies scaled down) so that about half of every queue "
                         "survives")
    ap.add_argument("--one-call", action="store_true",
                    help="time pard_estimate_drop_compact, the one call that does both steps (same outputs; the estimate "
                         "kernels then also stage the survivors), instead of pard_estimate_drop followed by pard_compact")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-side-leg", action="store_true",
                    help="do not time the other form of the call (one call / two calls) beside the timed region, so that a "
                         "kernel trace of the run holds the timed configuration only")
    ap.add_argument("--consistent", action="store_true",
                    help="sequentially consistent dropping (positions count kept requests only)")
    ap.add_argument("--ranked", action="store_true",
                    help="ranked positions in the later queues (a request takes the place its budget gives it there)")
    ap.add_argument("--workload", choices=["hot-path", "planner", "priority", "queue-delay", "reactive"], default="hot-path",
                    help="hot-path: estimate+drop+compact (default); planner: queue lengths + downstream latency "
                         "with the sampled batch-wait quantile on the same snapshots; priority: adaptive priority "
                         "from a rate series per (snapshot, stage); queue-delay: the sliding-window queueing delay "
                         "from delay samples per (snapshot, stage); reactive: the window-scan and SLO-split policies the "
                         "paper compares with, and how their drop sets differ from the proactive estimate's")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.ranked and args.consistent:
        print("bench.py: --ranked and --consistent are separate variants", file=sys.stderr)
        sys.exit(2)
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (snapshots would shard across GPUs with no "
              "communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_08747_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load_library()

    t0 = time.time()
    reshaped = args.snapshots is not None or args.per_snapshot is not None
    if reshaped and args.config != 5:
        print("bench.py: --snapshots/--per-snapshot reshape configuration 5 only", file=sys.stderr)
        sys.exit(2)
    shape = {}
    if args.snapshots is not None:
        shape["n_snapshots"] = args.snapshots
    if args.per_snapshot is not None:
        shape["per_snapshot"] = args.per_snapshot
    w = workloads.make_workload(args.config, permute=args.permute, **shape)
    if args.half_survivors:
        if args.config not in (2, 3, 4):
            print("bench.py: --half-survivors is a variant of configurations 2-4", file=sys.stderr)
            sys.exit(2)
        w = workloads.half_survivors(w)
    gen_s = time.time() - t0
    if args.workload == "reactive":
        print(json.dumps(bench_reactive(args, w, gen_s)))
        return
    s = binding.Session(w)
    # host-to-device time of the request arrays (outside every timed region; the boundary takes device buffers)
    torch.cuda.synchronize()
    t_up = time.perf_counter()
    for host in (w.arrival, w.deadline, w.stage):
        torch.from_numpy(host).to(s.dev)
    torch.cuda.synchronize()
    h2d_ms = (time.perf_counter() - t_up) * 1e3
    fused = s.max_snap <= binding.PARD_FUSED_SNAPSHOT_CAPACITY
    n = w.n

    if args.workload == "planner":
        print(json.dumps(bench_planner(args, w, s, gen_s)))
        return
    if args.workload == "priority":
        print(json.dumps(bench_priority(args, w, s, gen_s)))
        return
    if args.workload == "queue-delay":
        print(json.dumps(bench_queue_delay(args, w, s, gen_s)))
        return

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # one dispatch that reads and writes exactly this many bytes
        torch.cuda.synchronize()
        del src, dst

    one_call = args.one_call and not (args.consistent or args.ranked)     # the variants have no one-call form
    for _ in range(max(args.warmup, 1)):
        if one_call:
            s.run_one_call()
        else:
            s.run(consistent=args.consistent, ranked=args.ranked)
    torch.cuda.synchronize()

    # timed region: exactly --steps passes of the whole path
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    if one_call:
        for _, b, _ in ev:
            b.record()                      # creates the event; the library records it again between its two steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b, c in ev:
        a.record()
        if one_call:
            s.run_one_call(between_event=b.cuda_event)
        else:
            s.estimate_drop(consistent=args.consistent, ranked=args.ranked)
            b.record()
            s.compact()
        c.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    est_ms = float(np.mean([a.elapsed_time(b) for a, b, _ in ev]))
    cmp_ms = float(np.mean([b.elapsed_time(c) for _, b, c in ev]))

    # the same path through the one call that does both steps, timed beside it (outside the timed region above)
    other_ms = None
    if not (args.consistent or args.ranked or args.no_side_leg):
        run_other = s.run if one_call else s.run_one_call
        run_other()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            run_other()
        torch.cuda.synchronize()
        other_ms = (time.perf_counter() - t1) * 1e3 / args.steps

    res = s.results()
    drop_frac = float(res["drop"].mean()) if n else 0.0
    status = s.status_word()

    # roofline of the dominant kernel
    fcfs = bool((w.order_mode == workloads.MODE_FCFS).any())
    in_order = not fused and not args.ranked and arrives_in_deadline_order(w)
    if fused:
        small = s.max_snap <= 128
        kernel = ("wave_snapshot_kernel (the estimate step: one launch)" if small else
                  "the estimate step: presorted_snapshot_kernel for snapshots in queue order, then fused_snapshot_kernel "
                  "for the others (both launches are inside the timed interval)")
        passes = 0
    else:
        kernel = ("pard_estimate_drop call: count_kernel (which finds the requests in deadline order), setup_kernel, "
                  "split_kernel; the radix launches that follow find nothing to do" if in_order else
                  "pard_estimate_drop call (count, setup, histograms and radix passes, the last of which forms the results, "
                  "and their way back to request order)")
        # The denominator for snapshots beyond the chip's LDS is the out-of-core sort model with p passes of 8 bits
        # over the key range, also when the call exploits input that is already in order and moves less: that
        # lowers the bytes moved, not the model (the 17 B/request I/O floor is reported beside it).
        span = int(w.deadline.max()) - int(w.deadline.min()) if n else 0
        passes = max(1, -(-(max(span, 0).bit_length() + max(w.K * w.S - 1, 0).bit_length()) // 8))
    bpr = estimate_drop_bytes_per_request(fused, passes, fcfs)
    io_bpr = estimate_drop_bytes_per_request(True, 0, fcfs)
    alg_bytes = bpr * n
    achieved = alg_bytes / (est_ms * 1e-3) / 1e9 if est_ms > 0 else 0.0
    traffic = (recorded_traffic(args.config, "presorted_snapshot_kernel", "pard_presorted.hip")
               if fused and not args.permute and not args.consistent and not args.ranked and not reshaped else None)
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": (f"profiles/hbm_traffic_cfg{args.config}.txt (rocprofv3 counters, valid for the "
                                   "kernel source it names)") if traffic is not None else None,
                "kernel": kernel, "bytes_per_request": bpr, "launch_ms": round(est_ms, 4),
                # the same duration against the bare inputs and outputs (8 B in, 9 B out, + 4 under arrival order)
                "io_floor_bytes_per_request": io_bpr,
                "io_floor_frac": round(io_bpr * n / (est_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if est_ms > 0 else 0.0,
                # a plain device copy moving the same number of bytes, timed in this run
                "copy_calibration_gbs": round(copy_calibration(torch, int(alg_bytes)), 1)}

    out = {
        "metric": "requests evaluated/sec (estimate+drop+compact)",
        "value": round(n / (ms_per_step * 1e-3), 1),
        "unit": "requests/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": w.name + ("+consistent" if args.consistent else "") + ("+ranked" if args.ranked else ""), "requests": n, "snapshots": w.K,
                   "stages": w.S, "path": "on-chip" if fused else ("deadline-order split" if in_order else "radix-sort"), "radix_passes": passes,
                   "radix_passes_run": 0 if (fused or in_order) else passes,
                   "calls": "pard_estimate_drop_compact" if one_call else "pard_estimate_drop + pard_compact",
                   ("two_calls_ms_per_step" if one_call else "one_call_ms_per_step"): None if other_ms is None else round(other_ms, 4),
                   "drop_fraction": round(drop_frac, 4), "status_word": status,
                   "estimate_drop_ms": round(est_ms, 4), "compact_ms": round(cmp_ms, 4),
                   "h2d_ms": round(h2d_ms, 2), "generate_s": round(gen_s, 2)},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        import oracle
        threads = usable_cores()
        # the oracle finishes the whole workload in seconds, so the sample is the whole workload
        sub = w
        sample = f"whole workload ({n} requests), 1 run"
        if args.ranked:
            # the oracle counts the requests ahead in every later queue one by one (quadratic in the snapshot size)
            if w.K > 1:
                sub = workloads.make_workload(args.config, n_snapshots=min(w.K, 64), permute=args.permute)
                sample = f"first {sub.K} of {w.K} snapshots ({sub.n} requests), 1 run"
            else:
                sub = workloads.make_workload(args.config, n_requests=min(n, 200_000), permute=args.permute)
                sample = f"the same workload at {sub.n} requests, 1 run"
        oracle.build_oracle()
        t0 = time.perf_counter()
        oracle.run(sub, threads=threads, consistent=args.consistent, ranked=args.ranked)
        cpu_s = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.run(sub, threads=1, consistent=args.consistent, ranked=args.ranked)
        cpu1_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(sub.n / cpu_s, 1), "unit": "requests/s", "cores": threads,
                               "kind": "oracle", "sample": sample, "seconds": round(cpu_s, 3),
                               "single_thread": {"value": round(sub.n / cpu1_s, 1), "unit": "requests/s", "cores": 1,
                                                 "seconds": round(cpu1_s, 3)},
                               "host_cores": os.cpu_count(),
                               "cores_note": "cores = every host core this job may use (affinity mask, capped by the "
                                             "machine's OMP_NUM_THREADS share)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
