"""GPU parity of the reactive dropping policies (Section 5.1 "Baselines": window scan, per-module SLO split)
against the CPU oracle, bit for bit, through the C-ABI, on both kernel paths of the estimate call."""
import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

pytestmark = pytest.mark.gpu

FORCE_SORT = 1 << 20


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libpard.so")
    from paper_2602_08747_amd import binding
    binding.load_library()
    return binding


def run_both(gpu, oracle_mod, w, max_snap=None, threads=8):
    """Queues from the estimate call, then both policies; returns the drop fractions."""
    import torch
    print(f"case {w.name} n={w.n} K={w.K} S={w.S} max_snap={max_snap}", flush=True)
    ref = oracle_mod.run(w, threads=threads)
    s = gpu.Session(w, max_snapshot_requests=max_snap)
    s.estimate_drop()
    torch.cuda.synchronize()
    assert np.array_equal(s.order[:w.n].cpu().numpy(), ref["order"])
    drop = torch.full((max(w.n, 1),), 7, dtype=torch.uint8, device=s.dev)
    first = torch.full((w.K * w.S,), -5, dtype=torch.int32, device=s.dev)
    gpu.pard_reactive_drop(s.plan, gpu.REACTIVE_WINDOW_SCAN, w.n, None, s.deadline, None, None, s.now, s.order, s.seg_ptr, drop, first)
    torch.cuda.synchronize()
    want_drop, want_first = oracle_mod.nexus_drop(w.K, w.S, w.dag_shared, w.batch, w.lat_us, w.deadline, ref["order"], ref["seg_ptr"], w.now)
    got_first = first.cpu().numpy()
    assert np.array_equal(got_first, want_first), (np.flatnonzero(got_first != want_first)[:8], got_first[got_first != want_first][:8],
                                                   want_first[got_first != want_first][:8])
    assert np.array_equal(drop[:w.n].cpu().numpy(), want_drop)
    frac_scan = float(want_drop.mean()) if w.n else 0.0
    drop.fill_(7)
    gpu.pard_reactive_drop(s.plan, gpu.REACTIVE_SLO_SPLIT, w.n, s.arrival, s.deadline, s.stage, s.snap_ptr, s.now, None, None, drop, None)
    torch.cuda.synchronize()
    want = oracle_mod.clipper_drop(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.lat_us, w.arrival, w.deadline,
                                   w.stage, w.snap_ptr, w.now)
    assert np.array_equal(drop[:w.n].cpu().numpy(), want)
    return frac_scan, float(want.mean()) if w.n else 0.0


@pytest.mark.parametrize("cfg,kw", [(1, {}), (2, dict(n_requests=300_001)), (3, dict(n_requests=250_007)), (4, dict(n_requests=700_003)),
                                     (5, dict(n_snapshots=97, per_snapshot=8192))])
@pytest.mark.parametrize("fcfs", [True, False])
def test_config_shapes(gpu, oracle_mod, cfg, kw, fcfs):
    """The five configurations' shapes, shuffled; queues in arrival order (the paper's baseline) and in the plan's
    own order; time set so that both policies drop part of the queue."""
    w = wl.make_workload(cfg, permute=True, order_mode=wl.MODE_FCFS if fcfs else None, **kw)
    w.now[:] = np.maximum(0, w.now.astype(np.int64) - (150_000 if cfg != 1 else 0)).astype(np.int32)
    a, b = run_both(gpu, oracle_mod, w)
    if cfg != 1:
        assert 0 < b < 1, b
        if fcfs:                                 # (under high-budget-first the very first window fits)
            assert 0 < a < 1, a


@pytest.mark.parametrize("order", ["arrival", "plan"])
def test_mixed_snapshot_sizes(gpu, oracle_mod, order):
    """Snapshots of a few thousand requests on average, whose drop mask one workgroup each collects in request order,
    next to ones too large for that (they keep the walk over the queue slots), empty ones, sizes that leave the next
    snapshot on an odd address, and a single-request one."""
    sizes = [20000, 3001, 0, 17, 16384, 16385, 1, 8192, 5003, 0, 12289, 4099]
    base = wl.make_workload(5, n_snapshots=len(sizes), per_snapshot=max(sizes), permute=True,
                            order_mode=wl.MODE_FCFS if order == "arrival" else None)
    w = wl.with_snapshot_sizes(base, np.array(sizes))
    assert 1024 <= w.n // w.K <= 16384
    w.now[:] = np.maximum(0, w.now.astype(np.int64) - 150_000).astype(np.int32)
    a, b = run_both(gpu, oracle_mod, w, max_snap=FORCE_SORT)
    assert 0 < b < 1


def test_full_config5_and_4(gpu, oracle_mod):
    for cfg in (5, 4):
        w = wl.make_workload(cfg, order_mode=wl.MODE_FCFS)
        run_both(gpu, oracle_mod, w, threads=16)


@pytest.mark.parametrize("seed", range(10))
def test_random_plans_both_paths(gpu, oracle_mod, seed):
    """Random DAGs, every batch size, empty queues, queues shorter than a batch, ties; both estimate paths."""
    w = wl.random_workload(8100 + seed, K=1 + (seed * 5) % 9, S=1 + (seed * 3) % 9, n_per_snapshot=30 + 170 * (seed % 4),
                           monotone=(seed % 3 != 0), tie_heavy=(seed % 4 == 1), slo_choices=(20000, 60000, 200000))
    run_both(gpu, oracle_mod, w)
    run_both(gpu, oracle_mod, w, max_snap=FORCE_SORT)


def test_window_positions(gpu, oracle_mod):
    """One late request at every kind of place (start and end of a chunk of 64 slots, of a wave's tile, of the
    queue), batch sizes 1, 2, 63 and 64, queues whose only fitting window is one of the cut-off ones."""
    rp, cl = wl.csr_from_edges(1, [])
    for B in (1, 2, 7, 63, 64):
        n = 5000
        lat = (1000 + 10 * np.arange(1, 65)).astype(np.int32)
        places = [0, 1, B - 1, B, 62, 63, 64, 65, 127, 128, 1023, 1024, 1025, 4095, 4096, n - B - 1, n - B, n - 2, n - 1]
        K = len(places) + 2
        deadline = np.full((K, n), 60_000, np.int32)
        for u, i in enumerate(places):
            if 0 <= i < n:
                deadline[u, :i + 1] = 0                  # everything up to and including place i is late
        deadline[K - 2, :] = 0                           # nobody fits
        deadline[K - 2, n - 1] = 1000 + 10               # ... except a batch of one at the very end
        deadline[K - 1, :] = 0                           # nobody at all
        w = wl.Workload(name=f"late-B{B}", K=K, S=1, dag_shared=1, dag_row_ptr=rp, dag_col=cl, batch=np.array([B], np.int32),
                        workers=np.ones(1, np.int32), lat_us=lat, order_mode=np.full(1, wl.MODE_FCFS, np.int32),
                        arrival=np.tile(np.arange(n, dtype=np.int32), K), deadline=deadline.reshape(-1),
                        stage=np.zeros(K * n, np.int32), snap_ptr=(np.arange(K + 1) * n).astype(np.int32), now=np.zeros(K, np.int32))
        run_both(gpu, oracle_mod, w)
        run_both(gpu, oracle_mod, w, max_snap=FORCE_SORT)


def test_error_codes(gpu):
    import torch
    w = wl.make_workload(1)
    s = gpu.Session(w)
    s.estimate_drop()
    drop = torch.zeros(w.n, dtype=torch.uint8, device=s.dev)
    first = torch.zeros(w.K * w.S, dtype=torch.int32, device=s.dev)
    args = (None, s.deadline, None, None, s.now, s.order, s.seg_ptr, drop, first)
    assert gpu.pard_reactive_drop(s.plan, 2, w.n, *args, check=False) == -2
    assert gpu.pard_reactive_drop(s.plan, gpu.REACTIVE_WINDOW_SCAN, -1, *args, check=False) == -2
    assert gpu.pard_reactive_drop(s.plan, gpu.REACTIVE_WINDOW_SCAN, w.n, None, s.deadline, None, None, s.now, None, s.seg_ptr, drop, first,
                                  check=False) == -1
    assert gpu.pard_reactive_drop(s.plan, gpu.REACTIVE_SLO_SPLIT, w.n, None, s.deadline, s.stage, s.snap_ptr, s.now, None, None, drop, None,
                                  check=False) == -1
    # durations that add up beyond 2^30 along a path: the split's 64-bit products are not guaranteed any more
    w.lat_us[:] = 2**30
    big = gpu.Session(w)
    assert gpu.pard_reactive_drop(big.plan, gpu.REACTIVE_SLO_SPLIT, w.n, big.arrival, big.deadline, big.stage, big.snap_ptr, big.now,
                                  None, None, drop, None, check=False) == -11
