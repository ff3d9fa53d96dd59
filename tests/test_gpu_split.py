"""GPU parity of the large-snapshot path when the requests come in deadline order (no sort: the queues are a
stable split by stage; under high budget first the reverse with equal deadlines kept in request order), against
the oracle, bit for bit, through the C-ABI."""
import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

pytestmark = pytest.mark.gpu

INT32_MAX = 2**31 - 1
KEYS = ("est", "drop", "order", "seg_ptr", "surv_idx", "surv_ptr")
FORCE_SORT = 1 << 20


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libpard.so")
    from paper_2602_08747_amd import binding
    binding.load_library()
    return binding


def check(gpu, oracle_mod, w, max_snap=FORCE_SORT, sub=None, threads=8, consistent=False):
    import torch
    print(f"case {w.name} n={w.n} K={w.K} S={w.S} max_snap={max_snap} consistent={consistent}", flush=True)
    ref = oracle_mod.run(w, threads=threads, sub=sub, consistent=consistent)
    s = gpu.Session(w, max_snapshot_requests=max(max_snap, w.max_snapshot_requests))
    s.run(sub=None if sub is None else torch.from_numpy(sub).to(s.dev), consistent=consistent)
    got = s.results()
    for k in KEYS:
        if not np.array_equal(got[k], ref[k]):
            bad = np.flatnonzero(got[k] != ref[k]) if got[k].shape == ref[k].shape else None
            raise AssertionError(f"{w.name}: {k} differs; first bad {None if bad is None else bad[:8]}; "
                                 f"got {None if bad is None else got[k][bad[:8]]} want {None if bad is None else ref[k][bad[:8]]}")
    assert s.status_word() == 0
    return s, ref


@pytest.mark.parametrize("cfg,n", [(2, 300_001), (2, None), (3, 250_007), (4, 700_003), (4, None)])
@pytest.mark.parametrize("mode", [wl.MODE_LBF, wl.MODE_HBF])
def test_configurations_in_arrival_order(gpu, oracle_mod, cfg, n, mode):
    """Configurations 2 and 4 as generated come in deadline order (one SLO); configuration 3 mixes three SLOs and
    takes the radix passes.  Both deadline orders, deep overload and mixed masks."""
    w = wl.make_workload(cfg, n_requests=n, order_mode=mode)
    check(gpu, oracle_mod, w, threads=16)
    if n is not None:
        w.now[:] = np.maximum(0, w.now.astype(np.int64) - 280000).astype(np.int32)
        w.lat_us[:] = np.maximum(1, w.lat_us // 400)
        _, ref = check(gpu, oracle_mod, w)
        assert 0 < ref["drop"].mean() < 1
        # sequentially consistent dropping on the same queues: the split then only orders them
        _, cons = check(gpu, oracle_mod, w, consistent=True)
        assert 0 < cons["drop"].mean() < 1


@pytest.mark.parametrize("seed", range(10))
def test_random_plans_in_deadline_order(gpu, oracle_mod, seed):
    """Random DAGs and tables, one and several large snapshots (own DAG each), up to 64 queues, heavy ties (runs of
    equal deadlines: short ones are resolved in place, long ones send the call to the radix passes), odd sizes."""
    K = 1 + seed % 3
    S = 1 + (seed * 5) % 12
    mode = wl.MODE_HBF if seed % 2 else wl.MODE_LBF
    w = wl.in_deadline_order(wl.random_workload(9100 + seed, K=K, S=S, n_per_snapshot=9000 + 1777 * seed, dag_shared=seed % 2,
                                                modes=(mode,), tie_heavy=(seed % 5 == 4), time_span=40_000 if seed % 3 else 400_000,
                                                monotone=(seed % 4 != 0), vary_sizes=False))
    check(gpu, oracle_mod, w)
    sub = np.random.default_rng(seed).integers(0, 60_000, size=w.K * w.S).astype(np.int64)
    check(gpu, oracle_mod, w, sub=sub)
    check(gpu, oracle_mod, w, consistent=True)
    check(gpu, oracle_mod, w, sub=sub // 8, consistent=True)


def test_runs_of_equal_deadlines(gpu, oracle_mod):
    """High budget first: runs of 1..45 equal deadlines (up to 40 are resolved by looking left and right, longer ones
    are noticed by the count and the call takes the radix passes), runs across chunk and workgroup boundaries."""
    rng = np.random.default_rng(11)
    for longest in (1, 2, 7, 31, 35, 36, 45):
        n = 100_000
        runs = rng.integers(1, longest + 1, size=n)
        runs[::97] = longest
        d = np.repeat(np.cumsum(rng.integers(1, 50, size=n)), runs)[:n].astype(np.int32)
        w = wl.make_workload(4, n_requests=n, order_mode=wl.MODE_HBF)
        w.deadline[:] = d
        w.arrival[:] = d - 1000
        w.now[:] = int(d[n // 2])
        w.lat_us[:] = np.maximum(1, w.lat_us // 2000)
        _, ref = check(gpu, oracle_mod, w)
        assert 0 < ref["drop"].mean() < 1
        check(gpu, oracle_mod, w, consistent=True)


def test_one_falling_pair_takes_the_radix_passes(gpu, oracle_mod):
    for place in (1, 4095, 4096, 8191, 8192, 50_000, 99_999):
        w = wl.make_workload(2, n_requests=100_000)
        w.deadline[place - 1] = w.deadline[place] + 1
        w.stage[place - 1] = w.stage[place]
        check(gpu, oracle_mod, w)


def test_extremes_in_deadline_order(gpu, oracle_mod):
    w = wl.make_workload(2, n_requests=60_000)
    w.deadline[:500] = np.sort(np.random.default_rng(0).integers(-2**31, 0, 500)).astype(np.int32)
    w.deadline[-700:] = INT32_MAX
    w.stage[::11] = -7
    w.stage[5::13] = 1000
    check(gpu, oracle_mod, w)
    check(gpu, oracle_mod, w, consistent=True)
    w.now[:] = INT32_MAX
    check(gpu, oracle_mod, w)
    w.now[:] = -(2**31)
    w.lat_us[:] = INT32_MAX
    check(gpu, oracle_mod, w)
    for n in (0, 1, 2, 5, 4097, 8192, 8193):
        check(gpu, oracle_mod, wl.make_workload(2, n_requests=n))
        if n:
            check(gpu, oracle_mod, wl.make_workload(4, n_requests=n))


@pytest.mark.parametrize("mode", [wl.MODE_LBF, wl.MODE_HBF])
def test_many_small_and_empty_snapshots(gpu, oracle_mod, mode):
    """Up to 64 snapshots of one stage each, most of them far smaller than the 512 requests a wave takes at a time and
    some empty, so that several snapshot boundaries (also coinciding ones) fall inside one wave's chunk."""
    rng = np.random.default_rng(5)
    for K, S in ((64, 1), (21, 3), (7, 9)):
        sizes = rng.integers(0, 300, size=K)
        sizes[rng.integers(0, K, size=K // 4)] = 0
        sizes[K // 2] = 20_000
        w = wl.with_snapshot_sizes(wl.random_workload(777 + K, K=K, S=S, n_per_snapshot=20_000, dag_shared=1, modes=(mode,),
                                                      time_span=300_000, vary_sizes=False), sizes)
        check(gpu, oracle_mod, wl.in_deadline_order(w))


@pytest.mark.parametrize("mode", [wl.MODE_LBF, wl.MODE_HBF])
def test_deadline_order_unaligned_buffers(gpu, oracle_mod, mode):
    """Request arrays and outputs that start at odd offsets (views into larger allocations): the 16-byte accesses fall
    back to single ones, the results stay the same and nothing is written outside the views."""
    import torch
    w = wl.make_workload(4, n_requests=70_001, order_mode=mode)
    w.now[:] = int(w.deadline[w.n // 2])
    w.lat_us[:] = np.maximum(1, w.lat_us // 3000)
    s, ref = check(gpu, oracle_mod, w)
    n = w.n
    for o32, o8 in ((1, 1), (2, 6), (3, 3)):
        def view32(src):
            big = torch.full((n + 32,), -7, dtype=torch.int32, device=s.dev)
            v = big[o32:o32 + n]
            if src is not None:
                v.copy_(src)
            return big, v
        _, arrival = view32(s.arrival)
        _, deadline = view32(s.deadline)
        _, stage = view32(s.stage)
        est_big, est = view32(None)
        order_big, order = view32(None)
        drop_big = torch.full((n + 64,), 9, dtype=torch.uint8, device=s.dev)
        drop = drop_big[o8:o8 + n]
        gpu.pard_estimate_drop(s.plan, n, s.max_snap, arrival, deadline, stage, s.snap_ptr, s.now,
                               est, drop, order, s.seg_ptr, s.workspace)
        torch.cuda.synchronize()
        assert np.array_equal(est.cpu().numpy(), ref["est"]), (o32,)
        assert np.array_equal(drop.cpu().numpy(), ref["drop"]), (o8,)
        assert np.array_equal(order.cpu().numpy(), ref["order"]), (o32,)
        for big, off in ((est_big, o32), (order_big, o32)):
            h = big.cpu().numpy()
            assert (h[:off] == -7).all() and (h[off + n:] == -7).all()
        h = drop_big.cpu().numpy()
        assert (h[:o8] == 9).all() and (h[o8 + n:] == 9).all()


@pytest.mark.parametrize("mode", [wl.MODE_LBF, wl.MODE_HBF])
def test_graph_replays_choose_the_path_again(gpu, oracle_mod, mode):
    """A recorded call decides on the device, at every replay, whether the requests come in deadline order: the same
    graph is replayed on inputs in order (split), shuffled (radix passes), in order with another `now`, with one
    falling pair, and in order again, with eager work in between; every replay must match the oracle."""
    import torch
    w = wl.make_workload(4, n_requests=150_001, order_mode=mode)
    w.lat_us[:] = np.maximum(1, w.lat_us // 3000)
    w.now[:] = int(w.deadline[w.n // 3])
    s = gpu.Session(w, max_snapshot_requests=FORCE_SORT)
    s.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s.run()
    rng = np.random.default_rng(3)
    ordered = (w.arrival.copy(), w.deadline.copy(), w.stage.copy())
    perm = rng.permutation(w.n)
    for step in ("in order", "shuffled", "later now", "one falling pair", "in order again"):
        a, d, st = (x.copy() for x in ordered)
        if step == "shuffled":
            a, d, st = a[perm], d[perm], st[perm]
        if step == "one falling pair":
            d[70_000] = d[70_001] + 5
        if step == "later now":
            w.now[:] = int(ordered[1][2 * w.n // 3])
        w.arrival[:], w.deadline[:], w.stage[:] = a, d, st
        s.arrival.copy_(torch.from_numpy(w.arrival).to(s.dev))
        s.deadline.copy_(torch.from_numpy(w.deadline).to(s.dev))
        s.stage.copy_(torch.from_numpy(w.stage).to(s.dev))
        s.now.copy_(torch.from_numpy(w.now).to(s.dev))
        s.est.zero_(); s.drop.zero_(); s.order.zero_(); s.surv_idx.zero_()      # eager work between the replays
        torch.cuda.synchronize()
        print(f"replay: {step}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        got = s.results()
        ref = oracle_mod.run(w, threads=8)
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (step, k)
        assert s.status_word() == 0
        assert 0 < ref["drop"].mean() < 1
