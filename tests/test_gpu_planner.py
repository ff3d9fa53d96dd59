"""GPU parity of the State Planner side: queue lengths, downstream latency with the sampled
batch-wait quantile and its variants, and the estimate that takes it (C-ABI vs the CPU oracle,
bit for bit)."""
import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

pytestmark = pytest.mark.gpu

FORCE_SORT = 1 << 20
KEYS = ("est", "drop", "order", "seg_ptr", "surv_idx", "surv_ptr")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libpard.so")
    from paper_2602_08747_amd import binding
    binding.load_library()
    return binding


def draws(seed, M, S, span, negatives=False):
    rng = np.random.default_rng(seed)
    samples = rng.integers(-1000 if negatives else 0, span, M).astype(np.int32)
    picks = rng.integers(0, 2**32, M * S, dtype=np.uint64).astype(np.uint32)
    return samples, picks


def workloads():
    yield wl.make_workload(5, n_snapshots=40, per_snapshot=3000, permute=True)          # own DAG per snapshot
    yield wl.random_workload(11, K=7, S=9, n_per_snapshot=400, dag_shared=1)           # one DAG, several snapshots
    yield wl.make_workload(4, n_requests=200001, permute=True)                          # 12 stages, 16 paths
    yield wl.make_workload(1)
    w = wl.random_workload(12, K=5, S=6, n_per_snapshot=9000, dag_shared=0)             # ragged, some large
    yield w


def oracle_qlen(w):
    out = np.zeros(w.K * w.S, np.int32)
    for u in range(w.K):
        lo, hi = int(w.snap_ptr[u]), int(w.snap_ptr[u + 1])
        out[u * w.S:(u + 1) * w.S] = np.bincount(np.clip(w.stage[lo:hi], 0, w.S - 1), minlength=w.S)
    return out


def test_queue_lengths(gpu):
    import torch
    cases = list(workloads())
    cases.append(wl.make_workload(5, n_snapshots=3000, per_snapshot=1))                 # more queues per chunk than LDS counters
    cases.append(wl.make_workload(3, n_requests=0))
    w = wl.make_workload(1, n_requests=5000)
    w.stage[::7] = -3
    w.stage[3::11] = 99
    cases.append(w)
    for w in cases:
        print("case", w.name, w.n, w.K, w.S, flush=True)
        s = gpu.Session(w)
        qlen = torch.full((w.K * w.S,), -1, dtype=torch.int32, device=s.dev)
        gpu.pard_queue_lengths(s.plan, w.n, s.stage, s.snap_ptr, qlen)
        torch.cuda.synchronize()
        assert np.array_equal(qlen.cpu().numpy(), oracle_qlen(w))


@pytest.mark.parametrize("which", range(5))
def test_sub_latency_variants(gpu, oracle_mod, which):
    import torch
    w = list(workloads())[which]
    s = gpu.Session(w)
    qlen = oracle_qlen(w)
    plan_args = (w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, qlen)
    d_qlen = torch.from_numpy(qlen).to(s.dev)
    d_sub = torch.empty(w.K * w.S, dtype=torch.int64, device=s.dev)
    for variant in (gpu.SUB_LOWER, gpu.SUB_UPPER, gpu.SUB_SF, gpu.SUB_BACK):
        d_sub.fill_(-5)
        gpu.pard_sub_latency(s.plan, d_qlen, variant, 0, 1, 0, None, None, d_sub)
        torch.cuda.synchronize()
        assert np.array_equal(d_sub.cpu().numpy(), oracle_mod.sub_latency(*plan_args, variant)), variant
    for M, lam, neg in ((10_000, (1, 10), False), (1, (1, 2), False), (37, (36, 37), True), (1000, (999, 1000), False),
                        (16384, (1, 3), True), (513, (0, 1), False), (513, (5, 5), False), (4097, (1, 4097), False)):
        samples, picks = draws(77 + M, M, w.S, 80_000_000, neg)
        want = oracle_mod.sub_latency(*plan_args, gpu.SUB_FULL, lam, samples, picks, threads=8)
        d_sub.fill_(-5)
        gpu.pard_sub_latency(s.plan, d_qlen, gpu.SUB_FULL, lam[0], lam[1], M, torch.from_numpy(samples).to(s.dev),
                             torch.from_numpy(picks.view(np.int32)).to(s.dev), d_sub)
        torch.cuda.synchronize()
        got = d_sub.cpu().numpy()
        assert np.array_equal(got, want), (M, lam, np.flatnonzero(got != want)[:5], got[got != want][:5], want[got != want][:5])


def test_sub_latency_zero_and_equal_durations(gpu, oracle_mod):
    """Zero durations are skipped; equal durations give many tied totals (rank inside a run of equal values)."""
    import torch
    w = wl.make_workload(3, n_requests=3000)
    w.lat_us[:] = 4096
    w.lat_us[64:128] = 0
    s = gpu.Session(w)
    qlen = oracle_qlen(w)
    M = 2000
    samples = (np.arange(M, dtype=np.int32) % 7) * 1024        # only 7 distinct arrivals: waits in {0, 1024, ...}
    picks = np.random.default_rng(5).integers(0, 2**32, M * w.S, dtype=np.uint64).astype(np.uint32)
    d_sub = torch.empty(w.K * w.S, dtype=torch.int64, device=s.dev)
    for lam in ((1, 10), (1, 2), (9, 10)):
        want = oracle_mod.sub_latency(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, qlen,
                                      gpu.SUB_FULL, lam, samples, picks)
        gpu.pard_sub_latency(s.plan, torch.from_numpy(qlen).to(s.dev), gpu.SUB_FULL, lam[0], lam[1], M,
                             torch.from_numpy(samples).to(s.dev), torch.from_numpy(picks.view(np.int32)).to(s.dev), d_sub)
        torch.cuda.synchronize()
        assert np.array_equal(d_sub.cpu().numpy(), want)


@pytest.mark.parametrize("max_snap", [None, FORCE_SORT])
def test_estimate_with_planner_output(gpu, oracle_mod, max_snap):
    """Queue lengths -> L_sub -> estimate, drop, compaction, all on the GPU, against the oracle chain."""
    import torch
    for w in (wl.make_workload(5, n_snapshots=23, per_snapshot=5000, permute=True),
              wl.random_workload(21, K=3, S=7, n_per_snapshot=2500, dag_shared=1)):
        w.now[:] = np.maximum(0, w.now.astype(np.int64) - 250000).astype(np.int32)
        M = 10_000
        samples, picks = draws(9, M, w.S, 60_000_000)
        s = gpu.Session(w, max_snapshot_requests=max_snap)
        d_samples = torch.from_numpy(samples).to(s.dev)
        d_picks = torch.from_numpy(picks.view(np.int32)).to(s.dev)
        qlen = oracle_qlen(w)
        for variant, lam in ((gpu.SUB_FULL, (1, 10)), (gpu.SUB_UPPER, (0, 1)), (gpu.SUB_BACK, (0, 1)), (gpu.SUB_LOWER, (0, 1))):
            sub = s.planner(variant, lam, d_samples, d_picks)
            s.run(sub=sub)
            got = s.results()
            want_sub = oracle_mod.sub_latency(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us,
                                              qlen, variant, lam, samples, picks, threads=8)
            assert np.array_equal(s.sub.cpu().numpy(), want_sub)
            est, drop, order, seg_ptr = oracle_mod.estimate_drop(
                w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, w.order_mode,
                w.arrival, w.deadline, w.stage, w.snap_ptr, w.now, threads=8, sub=want_sub)
            surv_idx, surv_ptr = oracle_mod.compact(w.K, w.S, order, seg_ptr, drop)
            ref = dict(est=est, drop=drop, order=order, seg_ptr=seg_ptr, surv_idx=surv_idx, surv_ptr=surv_ptr)
            for k in KEYS:
                assert np.array_equal(got[k], ref[k]), (w.name, variant, k)
            if variant == gpu.SUB_LOWER:                       # the plain call computes the same thing on its own
                s.run()
                plain = s.results()
                for k in KEYS:
                    assert np.array_equal(plain[k], ref[k]), (w.name, "plain", k)
            assert s.status_word() == 0


def test_planner_error_codes(gpu):
    import torch
    w = wl.make_workload(1)
    s = gpu.Session(w)
    q = torch.zeros(w.K * w.S, dtype=torch.int32, device=s.dev)
    sub = torch.zeros(w.K * w.S, dtype=torch.int64, device=s.dev)
    smp = torch.zeros(16, dtype=torch.int32, device=s.dev)
    pk = torch.zeros(16 * w.S, dtype=torch.int32, device=s.dev)
    assert gpu.pard_sub_latency(s.plan, q, 9, 1, 10, 16, smp, pk, sub, check=False) == -2
    assert gpu.pard_sub_latency(s.plan, q, gpu.SUB_FULL, 11, 10, 16, smp, pk, sub, check=False) == -2
    assert gpu.pard_sub_latency(s.plan, q, gpu.SUB_FULL, 1, 10, 0, smp, pk, sub, check=False) == -2
    assert gpu.pard_sub_latency(s.plan, q, gpu.SUB_FULL, 1, 10, 1 << 20, smp, pk, sub, check=False) == -2
    assert gpu.pard_sub_latency(s.plan, q, gpu.SUB_FULL, 1, 10, 16, None, pk, sub, check=False) == -1
    assert gpu.pard_sub_latency(s.plan, None, gpu.SUB_LOWER, 0, 1, 0, None, None, sub, check=False) == -1
    assert gpu.pard_queue_lengths(s.plan, -1, s.stage, s.snap_ptr, q, check=False) == -2
    w2 = wl.make_workload(1)
    w2.lat_us[5] = (1 << 25) + 1
    s2 = gpu.Session(w2)
    assert gpu.pard_sub_latency(s2.plan, q, gpu.SUB_FULL, 1, 10, 16, smp, pk, sub, check=False) == -11
    assert gpu.pard_sub_latency(s2.plan, q, gpu.SUB_UPPER, 1, 10, 16, smp, pk, sub, check=False) == 0
    torch.cuda.synchronize()


# ---- sequentially consistent dropping ------------------------------------------------------------

def consistent_cases():
    w = wl.make_workload(5, n_snapshots=31, per_snapshot=8192, permute=True)
    w.now[:] = np.maximum(0, w.now.astype(np.int64) - 250000).astype(np.int32)
    yield w
    w = wl.make_workload(5, n_snapshots=9, per_snapshot=5000, permute=True, order_mode=None)
    w.order_mode[:] = np.arange(w.order_mode.size) % 3
    w.deadline[::5] = w.deadline[1::5][: w.deadline[::5].size]
    yield w
    yield wl.make_workload(1)
    for seed in range(6):
        yield wl.random_workload(300 + seed, K=1 + seed, S=1 + (seed * 5) % 9, n_per_snapshot=200 + 311 * seed,
                                 monotone=(seed % 2 == 0), tie_heavy=(seed % 3 == 1), dag_shared=seed % 2)
    for m in (0, 1, 63, 64, 65, 8191):
        yield wl.make_workload(5, n_snapshots=3, per_snapshot=m, permute=True)
    w = wl.make_workload(2, n_requests=6000, permute=True)          # slow-path stage constants, huge latencies
    w.batch[:] = [1, 64, 5, 33, 2]
    w.workers[:] = [1 << 20, 1, 3, 1, 999]
    w.lat_us[:] = (w.lat_us.astype(np.int64) * 5000).clip(0, 2**31 - 1).astype(np.int32)
    yield w
    w = wl.make_workload(3, n_requests=5000, permute=True)          # clustered keys: the wide-key bucket path
    w.deadline[::2] = 77
    w.deadline[1::4] = 2**31 - 1
    w.deadline[3::8] = 0
    yield w


@pytest.mark.parametrize("max_snap", [None, FORCE_SORT])
def test_consistent_dropping(gpu, oracle_mod, max_snap):
    mixed = 0
    for w in consistent_cases():
        print("case", w.name, w.n, w.K, w.S, flush=True)
        ref = oracle_mod.run(w, threads=8, consistent=True)
        s = gpu.Session(w, max_snapshot_requests=max_snap)
        s.run(consistent=True)
        got = s.results()
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (w.name, k)
        assert s.status_word() == 0
        one = oracle_mod.run(w, threads=8)
        mixed += int(not np.array_equal(one["drop"], ref["drop"]))
    assert mixed >= 3                       # the variant really decides differently on several of them


def test_consistent_with_planner_output(gpu, oracle_mod):
    import torch
    w = wl.make_workload(5, n_snapshots=12, per_snapshot=6000, permute=True)
    w.now[:] = np.maximum(0, w.now.astype(np.int64) - 200000).astype(np.int32)
    M = 3000
    samples, picks = draws(4, M, w.S, 60_000_000)
    s = gpu.Session(w)
    sub = s.planner(gpu.SUB_FULL, (1, 10), torch.from_numpy(samples).to(s.dev), torch.from_numpy(picks.view(np.int32)).to(s.dev))
    s.run(sub=sub, consistent=True)
    got = s.results()
    want_sub = oracle_mod.sub_latency(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us,
                                      oracle_qlen(w), gpu.SUB_FULL, (1, 10), samples, picks, threads=8)
    ref = oracle_mod.run(w, threads=8, sub=want_sub, consistent=True)
    for k in KEYS:
        assert np.array_equal(got[k], ref[k]), k
    assert 0 < ref["drop"].mean() < 1


def large_consistent_cases():
    """(workload, downstream latency or None).  With the downstream term taken from the snapshot the later
    stages' full queues swamp every budget in these overloaded snapshots; a given, modest L_sub lets the
    position in the own queue decide."""
    yield wl.make_workload(3, n_requests=200_003), None                    # deep overload: few candidates, at the queues' ends
    w = wl.make_workload(4, n_requests=300_000, permute=True)              # skewed queues, high budget first
    yield w, np.full(w.K * w.S, 30_000, np.int64)
    w = wl.make_workload(2, n_requests=250_000)                            # nothing has expired: every request is a candidate
    w.now[:] = 0
    yield w, None
    w = wl.make_workload(3, n_requests=180_000, permute=True)              # in between, mixed orders, FCFS among them
    w.now[:] = int(np.median(w.arrival))
    w.order_mode[:] = np.arange(w.order_mode.size) % 3
    yield w, (np.arange(w.K * w.S, dtype=np.int64) * 7000)
    w = wl.make_workload(4, n_requests=150_001)                            # candidates scattered: random deadlines
    rng = np.random.default_rng(8)
    w.now[:] = 2**30
    w.deadline[:] = (2**30 + rng.integers(-10_000_000, 60_000_000, w.n)).astype(np.int32)
    w.deadline[::9] = 2**31 - 1
    yield w, np.zeros(w.K * w.S, np.int64)
    w = wl.make_workload(2, n_requests=60_000, permute=True)               # degenerate stage constants on the closed-form side
    w.now[:] = int(np.quantile(w.arrival, 0.9))
    w.batch[:] = [1, 2, 64, 7, 64]
    w.workers[:] = [1, 3, 1 << 20, 5, 1]
    lat = w.lat_us.reshape(w.S, 64)
    lat[0] = 0                                                             # free stage: nobody is ever late there
    lat[1] = 5000                                                          # flat table
    lat[2] = np.minimum(lat[2].astype(np.int64) * 3000, 2**31 - 1)         # huge latencies, huge worker count
    lat[4, :63] = 100                                                      # a queue shorter than one batch sees only these
    w.order_mode[:] = [0, 1, 0, 1, 0]
    w.deadline[::13] = 2**31 - 1
    yield w, np.array([0, 1_000_000, 0, 250_000, 0], np.int64)
    w = wl.random_workload(77, K=5, S=6, n_per_snapshot=9000, dag_shared=0)  # ragged snapshots, queues that start inside a mask word
    yield w, None
    w = wl.random_workload(78, K=40, S=3, n_per_snapshot=700, dag_shared=1, tie_heavy=True)   # more queues than the LDS table holds
    yield w, np.full(w.K * w.S, 1000, np.int64)


def test_consistent_large_snapshots(gpu, oracle_mod):
    import torch
    mixed = 0
    for w, sub in large_consistent_cases():
        print("case", w.name, w.n, w.K, w.S, flush=True)
        ref = oracle_mod.run(w, threads=8, sub=sub, consistent=True)
        s = gpu.Session(w, max_snapshot_requests=max(FORCE_SORT, w.max_snapshot_requests))
        s.run(sub=None if sub is None else torch.from_numpy(sub).to(s.dev), consistent=True)
        got = s.results()
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (w.name, k, np.flatnonzero(got[k] != ref[k])[:5])
        assert s.status_word() == 0
        one = oracle_mod.run(w, threads=8, sub=sub)
        mixed += int(not np.array_equal(one["drop"], ref["drop"]))
        print("   drop fraction", ref["drop"].mean(), "plain", one["drop"].mean(), flush=True)
    assert mixed >= 6


# ---- adaptive priority -----------------------------------------------------------------------

def rate_series(w, T, seed, lat=None):
    """Per (snapshot, stage) a series around the stage's throughput, some far off, some zero."""
    rng = np.random.default_rng(seed)
    lat = w.lat_us if lat is None else lat
    latB = lat.reshape(-1, 64)[np.arange(w.batch.size), w.batch - 1].astype(np.int64)
    cap = w.workers.astype(np.int64) * w.batch * 1_000_000 // np.maximum(1, latB)
    idx = np.arange(w.K * w.S) % w.S if w.dag_shared else np.arange(w.K * w.S)
    base = np.repeat(cap[idx], T).reshape(w.K * w.S, T)
    rate = np.clip(base * rng.uniform(0.6, 1.5, (w.K * w.S, T)), 0, 2**31 - 1).astype(np.int32)
    rate[rng.random((w.K * w.S, T)) < 0.05] = 0
    return rate


@pytest.mark.parametrize("T,window", [(1, 1), (7, 3), (64, 5), (65, 64), (200, 250), (1000, 50), (4097, 129)])
def test_priority_modes(gpu, oracle_mod, T, window):
    import torch
    for w in (wl.make_workload(5, n_snapshots=37, per_snapshot=10), wl.random_workload(55, K=6, S=9, n_per_snapshot=10, dag_shared=1),
              wl.make_workload(4, n_requests=10)):
        s = gpu.Session(w)
        rate = rate_series(w, T, 5 * T + window)
        for prev in (None, (np.arange(w.K * w.S) % 2).astype(np.int32)):
            want = oracle_mod.priority_modes(w.K, w.S, w.dag_shared, w.batch, w.workers, w.lat_us, rate, window, prev)
            d_mode = torch.full((w.K * w.S,), -1, dtype=torch.int32, device=s.dev)
            gpu.pard_priority_modes(s.plan, T, window, torch.from_numpy(rate).to(s.dev),
                                    None if prev is None else torch.from_numpy(prev).to(s.dev), d_mode)
            torch.cuda.synchronize()
            got = d_mode.cpu().numpy()
            assert np.array_equal(got, want), (w.name, T, window, np.flatnonzero(got != want)[:5])
        assert 0 < want.mean() < 1 or T == 1


def test_priority_extremes(gpu, oracle_mod):
    import torch
    w = wl.make_workload(1)
    w.batch[:] = 64
    w.workers[:] = 1 << 20
    lat = w.lat_us.copy()
    lat[:] = 2**31 - 1
    lat[64:128] = 0                                    # unbounded throughput: the load factor is 0
    w.lat_us = lat
    s = gpu.Session(w)
    T = 3000
    rate = np.full((w.K * w.S, T), 2**31 - 1, np.int32)
    rate[2, ::2] = 0
    want = oracle_mod.priority_modes(w.K, w.S, w.dag_shared, w.batch, w.workers, lat, rate, 7)
    d_mode = torch.empty(w.K * w.S, dtype=torch.int32, device=s.dev)
    gpu.pard_priority_modes(s.plan, T, 7, torch.from_numpy(rate).to(s.dev), None, d_mode)
    torch.cuda.synchronize()
    assert np.array_equal(d_mode.cpu().numpy(), want)
    assert gpu.pard_priority_modes(s.plan, 0, 7, torch.from_numpy(rate).to(s.dev), None, d_mode, check=False) == -2
    assert gpu.pard_priority_modes(s.plan, T, 0, torch.from_numpy(rate).to(s.dev), None, d_mode, check=False) == -2
    assert gpu.pard_priority_modes(s.plan, T, 7, None, None, d_mode, check=False) == -1


@pytest.mark.parametrize("max_snap", [None, FORCE_SORT])
def test_priority_feeds_the_queue_order(gpu, oracle_mod, max_snap):
    """Rates -> priorities -> plan -> estimate: the same as the oracle run with those order modes."""
    import torch
    for w in (wl.make_workload(5, n_snapshots=14, per_snapshot=3000, permute=True),
              wl.random_workload(56, K=1, S=7, n_per_snapshot=6000, dag_shared=1)):
        s = gpu.Session(w, max_snapshot_requests=max_snap)
        T, window = 300, 20
        rate = rate_series(w, T, 11)
        modes = oracle_mod.priority_modes(w.K, w.S, w.dag_shared, w.batch, w.workers, w.lat_us, rate, window)
        d_mode = torch.empty(w.K * w.S, dtype=torch.int32, device=s.dev)
        gpu.pard_priority_modes(s.plan, T, window, torch.from_numpy(rate).to(s.dev), None, d_mode)
        gpu.pard_plan_set_modes(s.plan, d_mode)
        s.run()
        got = s.results()
        assert np.array_equal(d_mode.cpu().numpy(), modes) and 0 < modes.mean() < 1
        w.order_mode = modes[: w.order_mode.size].astype(np.int32)
        ref = oracle_mod.run(w, threads=8)
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (w.name, k)


# ---- monitored queueing delay (sliding window) -------------------------------------------------------

def delay_series(w, L, window, seed, wide=False):
    """Time-stamped delay samples per (snapshot, stage): ages spread over about two windows, some later
    than now."""
    rng = np.random.default_rng(seed)
    G = w.K * w.S
    now = w.now.astype(np.int64).repeat(w.S)[:, None]
    span = min(2 * window, 2**31 - 1)
    time = (now - rng.integers(-span // 16 - 1, span, size=(G, L))).clip(-2**31, 2**31 - 1).astype(np.int32)
    delay = rng.integers(-1000, 2**31 - 1 if wide else 400_000, size=(G, L)).astype(np.int32)
    return time, delay


@pytest.mark.parametrize("L,window", [(0, 5_000_000), (1, 5_000_000), (63, 1000), (64, 5_000_000), (65, 7),
                                      (257, 2**31 - 1), (1000, 5_000_000), (4099, 1_000_000)])
def test_queue_delay(gpu, oracle_mod, L, window):
    import torch
    for w in (wl.make_workload(5, n_snapshots=50, per_snapshot=10), wl.random_workload(31, K=3, S=5, n_per_snapshot=4, dag_shared=1)):
        for wide in (False, True):
            print("case", w.name, L, window, wide, flush=True)
            s = gpu.Session(w)
            time, delay = delay_series(w, L, window, 7 + L, wide)
            want = oracle_mod.queue_delay(w.K, w.S, time, delay, w.now, window)
            q = torch.full((w.K * w.S,), -9, dtype=torch.int32, device=s.dev)
            d_time = torch.from_numpy(time.ravel().copy()).to(s.dev) if L else None
            d_delay = torch.from_numpy(delay.ravel().copy()).to(s.dev) if L else None
            gpu.pard_queue_delay(s.plan, L, window, d_time, d_delay, s.now, q)
            torch.cuda.synchronize()
            got = q.cpu().numpy()
            assert np.array_equal(got, want), (np.flatnonzero(got != want)[:5], got[got != want][:5], want[got != want][:5])


def test_queue_delay_extremes_and_errors(gpu, oracle_mod):
    import torch
    w = wl.make_workload(1)
    w.now[:] = 2**31 - 1
    s = gpu.Session(w)
    L = 5000
    big = 2**31 - 1
    time = np.full((w.S, L), big, np.int32)
    delay = np.full((w.S, L), big, np.int32)
    time[1, ::2] = 0                                     # half the samples at the far edge: weight 0 at age = window
    delay[2, :] = np.arange(L)
    q = torch.empty(w.S, dtype=torch.int32, device=s.dev)
    d_time, d_delay = torch.from_numpy(time.ravel()).to(s.dev), torch.from_numpy(delay.ravel()).to(s.dev)
    gpu.pard_queue_delay(s.plan, L, big, d_time, d_delay, s.now, q)
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), oracle_mod.queue_delay(w.K, w.S, time, delay, w.now, big))
    assert q.cpu().numpy()[0] == big
    # the same series from buffers that do not start on a 16-byte boundary
    pad = torch.zeros(1, dtype=torch.int32, device=s.dev)
    o_time, o_delay = torch.cat([pad, d_time])[1:], torch.cat([pad, d_delay])[1:]
    assert o_time.data_ptr() % 16 == 4
    q2 = torch.empty_like(q)
    gpu.pard_queue_delay(s.plan, L, big, o_time, o_delay, s.now, q2)
    torch.cuda.synchronize()
    assert torch.equal(q, q2)
    assert gpu.pard_queue_delay(s.plan, L, 0, d_time, d_delay, s.now, q, check=False) == -2
    assert gpu.pard_queue_delay(s.plan, L, 2**31, d_time, d_delay, s.now, q, check=False) == -2
    assert gpu.pard_queue_delay(s.plan, -1, 10, d_time, d_delay, s.now, q, check=False) == -2
    assert gpu.pard_queue_delay(s.plan, L, 10, None, d_delay, s.now, q, check=False) == -1
    assert gpu.pard_queue_delay(s.plan, L, 10, d_time, d_delay, s.now, None, check=False) == -1
    sub = torch.zeros(w.K * w.S, dtype=torch.int64, device=s.dev)
    assert gpu.pard_sub_latency_q(s.plan, q, None, gpu.SUB_LOWER, 0, 1, 0, None, None, sub, check=False) == -1
    torch.cuda.synchronize()


@pytest.mark.parametrize("max_snap", [None, FORCE_SORT])
def test_monitored_delay_feeds_the_estimate(gpu, oracle_mod, max_snap):
    """Delay samples -> q_i -> L_sub with the sampled batch wait -> estimate, drop, compaction on the GPU,
    against the same chain of oracle calls."""
    import torch
    for w in (wl.make_workload(5, n_snapshots=19, per_snapshot=4000, permute=True),
              wl.random_workload(41, K=4, S=6, n_per_snapshot=1500, dag_shared=1)):
        w.now[:] = np.maximum(0, w.now.astype(np.int64) - 200000).astype(np.int32)
        window = 5_000_000
        time, delay = delay_series(w, 300, window, 99)
        M = 2000
        samples, picks = draws(19, M, w.S, 60_000_000)
        s = gpu.Session(w, max_snapshot_requests=max_snap)
        d_q = torch.empty(w.K * w.S, dtype=torch.int32, device=s.dev)
        gpu.pard_queue_delay(s.plan, 300, window, torch.from_numpy(time.ravel().copy()).to(s.dev),
                             torch.from_numpy(delay.ravel().copy()).to(s.dev), s.now, d_q)
        want_q = oracle_mod.queue_delay(w.K, w.S, time, delay, w.now, window)
        qlen = oracle_qlen(w)
        d_samples = torch.from_numpy(samples).to(s.dev)
        d_picks = torch.from_numpy(picks.view(np.int32)).to(s.dev)
        for variant, lam in ((gpu.SUB_FULL, (1, 10)), (gpu.SUB_LOWER, (0, 1)), (gpu.SUB_UPPER, (0, 1)), (gpu.SUB_SF, (0, 1))):
            sub = s.planner(variant, lam, d_samples, d_picks, qdelay=d_q)
            s.run(sub=sub)
            got = s.results()
            assert np.array_equal(d_q.cpu().numpy(), want_q)
            want_sub = oracle_mod.sub_latency(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us,
                                              qlen, variant, lam, samples, picks, threads=8, qdelay=want_q)
            assert np.array_equal(s.sub.cpu().numpy(), want_sub), variant
            est, drop, order, seg_ptr = oracle_mod.estimate_drop(
                w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, w.order_mode,
                w.arrival, w.deadline, w.stage, w.snap_ptr, w.now, threads=8, sub=want_sub)
            surv_idx, surv_ptr = oracle_mod.compact(w.K, w.S, order, seg_ptr, drop)
            ref = dict(est=est, drop=drop, order=order, seg_ptr=seg_ptr, surv_idx=surv_idx, surv_ptr=surv_ptr)
            for k in KEYS:
                assert np.array_equal(got[k], ref[k]), (w.name, variant, k)
            assert 0 < drop.mean() < 1, drop.mean()


# ---- ranked positions in the later queues --------------------------------------------------------------

def ranked_cases():
    w = wl.make_workload(5, n_snapshots=6, per_snapshot=8192, permute=True)
    w.now[:] = np.maximum(0, w.now.astype(np.int64) - 250000).astype(np.int32)
    yield w
    w = wl.make_workload(5, n_snapshots=7, per_snapshot=3000, permute=True, order_mode=None)
    w.order_mode[:] = np.arange(w.order_mode.size) % 3
    w.deadline[::5] = w.deadline[1::5][: w.deadline[::5].size]                     # ties across queues
    yield w
    yield wl.make_workload(1)
    for seed in range(6):
        yield wl.random_workload(900 + seed, K=1 + seed, S=1 + (seed * 5) % 9, n_per_snapshot=150 + 211 * seed,
                                 monotone=(seed % 2 == 0), tie_heavy=(seed % 3 == 1), dag_shared=seed % 2)
    yield wl.make_workload(4, n_requests=20_001, permute=True)                      # 12 stages, 16 paths, high budget first
    w = wl.make_workload(3, n_requests=15_000)                                      # arrival order, three SLOs
    w.now[:] = int(np.median(w.arrival))
    yield w
    w = wl.make_workload(2, n_requests=9000, permute=True)                          # extreme values
    w.deadline[::7] = 2**31 - 1
    w.deadline[3::11] = -2**31
    w.workers[:] = [1 << 20, 1, 3, 1, 999]
    yield w


def test_ranked_positions(gpu, oracle_mod):
    differs = 0
    for w in ranked_cases():
        print("case", w.name, w.n, w.K, w.S, flush=True)
        ref = oracle_mod.run(w, threads=8, ranked=True)
        for max_snap in (None, FORCE_SORT):
            s = gpu.Session(w, max_snapshot_requests=None if max_snap is None else max(max_snap, w.max_snapshot_requests))
            s.run(ranked=True)
            got = s.results()
            for k in KEYS:
                assert np.array_equal(got[k], ref[k]), (w.name, max_snap, k, np.flatnonzero(got[k] != ref[k])[:5])
            assert s.status_word() == 0
        differs += int(not np.array_equal(oracle_mod.run(w, threads=8)["drop"], ref["drop"]))
    assert differs >= 6                      # the variant really decides differently on most of them


def test_ranked_many_stages_and_errors(gpu, oracle_mod):
    S, K = 64, 3
    rng = np.random.default_rng(77)
    rp, col = wl.csr_from_edges(S, wl.chain_edges(S) + [(5, 30), (12, 63)])
    sizes = rng.integers(500, 2500, size=K)
    snap_ptr = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    n = int(snap_ptr[-1])
    arrival = rng.integers(0, 200_000, n).astype(np.int32)
    w = wl.Workload(name="chain64-ranked", K=K, S=S, dag_shared=1, dag_row_ptr=rp, dag_col=col,
                    batch=rng.integers(1, 65, S).astype(np.int32), workers=rng.integers(1, 9, S).astype(np.int32),
                    lat_us=np.ascontiguousarray(wl.monotone_tables(rng, S).reshape(-1) // 20, np.int32),
                    order_mode=rng.integers(0, 3, S).astype(np.int32), arrival=arrival,
                    deadline=(arrival + rng.choice([100_000, 900_000, 4_000_000], n)).astype(np.int32),
                    stage=rng.integers(0, S, n).astype(np.int32), snap_ptr=snap_ptr, now=np.full(K, 150_000, np.int32))
    ref = oracle_mod.run(w, threads=8, ranked=True)
    for max_snap in (None, FORCE_SORT):
        s = gpu.Session(w, max_snapshot_requests=max_snap)
        s.run(ranked=True)
        got = s.results()
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (max_snap, k)
    assert gpu.pard_estimate_drop_ranked(s.plan, -1, s.max_snap, s.arrival, s.deadline, s.stage, s.snap_ptr, s.now, s.est, s.drop,
                                         s.order, s.seg_ptr, s.workspace, check=False) == -2
    assert gpu.pard_estimate_drop_ranked(s.plan, s.n, s.max_snap, s.arrival, None, s.stage, s.snap_ptr, s.now, s.est, s.drop,
                                         s.order, s.seg_ptr, s.workspace, check=False) == -1
