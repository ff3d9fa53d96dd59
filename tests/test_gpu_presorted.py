"""GPU parity of the on-chip kernel for snapshots that already come in queue order (rising deadlines under
low-budget-first): such snapshots are finished by a stable split by stage, every other snapshot of the same
batch is marked and taken by the general kernel.  Bit for bit against the oracle, through the C-ABI."""
import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

pytestmark = pytest.mark.gpu

INT32_MAX = 2**31 - 1
KEYS = ("est", "drop", "order", "seg_ptr", "surv_idx", "surv_ptr")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libpard.so")
    from paper_2602_08747_amd import binding
    binding.load_library()
    return binding


def check(gpu, oracle_mod, w, max_snap=None, sub=None):
    import torch
    print(f"case {w.name} n={w.n} K={w.K} S={w.S} max_snap={max_snap}", flush=True)
    ref = oracle_mod.run(w, threads=8, sub=sub)
    s = gpu.Session(w, max_snapshot_requests=max_snap)
    s.run(sub=None if sub is None else torch.from_numpy(sub).to(s.dev))
    got = s.results()
    for k in KEYS:
        if not np.array_equal(got[k], ref[k]):
            bad = np.flatnonzero(got[k] != ref[k]) if got[k].shape == ref[k].shape else None
            raise AssertionError(f"{w.name}: {k} differs; first bad {None if bad is None else bad[:8]}; "
                                 f"got {None if bad is None else got[k][bad[:8]]} want {None if bad is None else ref[k][bad[:8]]}")
    assert s.status_word() == 0
    if sub is None:
        # the whole path in one call must leave the same outputs (survivors staged by the estimate kernels)
        for t in (s.est, s.drop, s.order, s.seg_ptr, s.surv_idx, s.surv_ptr):
            t.fill_(0x55)
        s.run_one_call()
        got = s.results()
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (w.name, "one call", k)
        assert s.status_word() == 0
    return s, ref


def marks(s):
    """The workspace's word per snapshot behind its 256-byte header, as the in-order kernel left it:
    0 = finished there, 1 = left to the general kernel."""
    return s.workspace[64:64 + s.w.K].cpu().numpy()


@pytest.mark.parametrize("cap", [1024, 2048, 4096, 8192])
def test_in_order_every_capacity(gpu, oracle_mod, cap):
    """Snapshots in arrival order that fill the workgroup's capacity exactly, fall short of it, and ragged mixes
    whose snapshots start at any offset of the request arrays."""
    for per in (cap, cap - 1, cap // 2 + 3, 300):
        w = wl.make_workload(5, n_snapshots=6, per_snapshot=per)
        s, ref = check(gpu, oracle_mod, w, max_snap=cap)
        assert (marks(s) == 0).all()                 # every snapshot was finished by the in-order kernel
        if per == 8192:
            assert 0 < ref["drop"].mean() < 1
    base = wl.make_workload(5, n_snapshots=60, per_snapshot=cap)
    sizes = np.random.default_rng(cap).integers(0, cap + 1, 60)
    check(gpu, oracle_mod, wl.with_snapshot_sizes(base, sizes), max_snap=cap)
    check(gpu, oracle_mod, wl.with_snapshot_sizes(base, np.minimum(sizes, 700)), max_snap=cap)


def test_batch_mixing_ordered_and_shuffled_snapshots(gpu, oracle_mod):
    """One batch in which some snapshots come in queue order, some are shuffled, some are in order except for
    one swapped pair (which passes the first look at 64 deadlines and fails the full check), some are empty."""
    K, per = 64, 8192
    w = wl.make_workload(5, n_snapshots=K, per_snapshot=per)
    sh = wl.make_workload(5, n_snapshots=K, per_snapshot=per, permute=True)
    rng = np.random.default_rng(17)
    for u in range(K):
        lo, hi = u * per, (u + 1) * per
        kind = u % 4
        if kind == 1:
            w.arrival[lo:hi], w.deadline[lo:hi], w.stage[lo:hi] = sh.arrival[lo:hi], sh.deadline[lo:hi], sh.stage[lo:hi]
        elif kind == 2:
            i = int(rng.integers(1, per - 1))
            j = lo + i
            while w.deadline[j] == w.deadline[j - 1] and j + 1 < hi:
                j += 1
            for a in (w.arrival, w.deadline, w.stage):
                a[j - 1], a[j] = a[j], a[j - 1]
            w.stage[j - 1] = w.stage[j]            # one queue: treating the snapshot as ordered would misplace the pair
    s, _ = check(gpu, oracle_mod, w)
    assert np.array_equal(marks(s), np.isin(np.arange(K) % 4, (1, 2)).astype(np.int32))
    sizes = np.where(np.arange(K) % 5 == 3, 0, rng.integers(1, per + 1, K))
    check(gpu, oracle_mod, wl.with_snapshot_sizes(w, sizes))


def test_one_falling_pair_anywhere(gpu, oracle_mod):
    """A single pair out of order, of one stage, at every kind of place the order check treats differently: inside
    a lane's group of four, between neighbouring lanes, between the sub-blocks of a wave, between waves, at both
    ends.  Every such snapshot must be marked and come out right."""
    places = [1, 2, 3, 4, 5, 8, 255, 256, 257, 259, 260, 511, 512, 1023, 1024, 1025, 2047, 2048, 4095, 4096, 6143, 6144,
              7167, 7168, 8188, 8189, 8190, 8191]
    K, per = len(places), 8192
    w = wl.make_workload(5, n_snapshots=K, per_snapshot=per)
    for u, p in enumerate(places):
        j = u * per + p
        w.deadline[j - 1] = w.deadline[j] + 1          # still between its neighbours' neighbours or not: either way a fall
        w.stage[j - 1] = w.stage[j]
    s, _ = check(gpu, oracle_mod, w)
    assert (marks(s) == 1).all(), marks(s)
    # the same places in smaller workgroups
    for cap in (1024, 2048, 4096):
        sub = [p for p in places if p < cap]
        w = wl.make_workload(5, n_snapshots=len(sub), per_snapshot=cap)
        for u, p in enumerate(sub):
            j = u * cap + p
            w.deadline[j - 1] = w.deadline[j] + 1
            w.stage[j - 1] = w.stage[j]
        s, _ = check(gpu, oracle_mod, w)
        assert (marks(s) == 1).all(), (cap, marks(s))


@pytest.mark.parametrize("seed", range(8))
def test_in_order_random_plans(gpu, oracle_mod, seed):
    """Random pipelines of up to six stages with the requests arranged by deadline: heavy ties, every batch size
    and worker count, latency tables that are not monotone, the downstream latency given from outside."""
    S = 1 + seed % 6
    w = wl.in_deadline_order(wl.random_workload(4000 + seed, K=7, S=S, n_per_snapshot=1500, dag_shared=seed % 2,
                                                tie_heavy=(seed % 3 == 0), modes=(wl.MODE_LBF,), monotone=(seed % 2 == 0),
                                                max_workers=300 if seed == 5 else 16))
    s, ref = check(gpu, oracle_mod, w)
    assert (marks(s) == 0).all() or seed == 5          # seed 5 draws worker counts the short form does not cover
    check(gpu, oracle_mod, w, max_snap=8192)
    sub = np.random.default_rng(seed).integers(0, 60_000, size=w.K * w.S).astype(np.int64)
    check(gpu, oracle_mod, w, sub=sub)


def test_in_order_edge_values(gpu, oracle_mod):
    """Deadlines from the most negative value to INT32_MAX (never dropped), stage ids outside the pipeline,
    a time far in the past and one at the end of the range (saturated estimates)."""
    w = wl.make_workload(5, n_snapshots=5, per_snapshot=4000)
    for u in range(5):
        lo = u * 4000
        w.deadline[lo:lo + 300] = np.sort(np.random.default_rng(u).integers(-2**31, 0, 300)).astype(np.int32)
        w.deadline[lo + 3500:lo + 4000] = INT32_MAX
    w.stage[::11] = -7
    w.stage[5::13] = 1000
    s, ref = check(gpu, oracle_mod, w)
    assert not ref["drop"][w.deadline == INT32_MAX].any()
    w.now[:] = INT32_MAX
    check(gpu, oracle_mod, w)
    w.now[:] = -(2**31)
    check(gpu, oracle_mod, w)
    w.lat_us[:] = INT32_MAX                     # no stage admits the short form any more: the general kernel
    check(gpu, oracle_mod, w)


def test_plans_the_split_does_not_cover(gpu, oracle_mod):
    """Seven stages, high-budget-first and arrival order, more than 256 workers: the general kernel runs alone."""
    w = wl.in_deadline_order(wl.random_workload(77, K=9, S=7, n_per_snapshot=2000, dag_shared=0, modes=(wl.MODE_LBF,)))
    check(gpu, oracle_mod, w)
    for mode in (wl.MODE_HBF, wl.MODE_FCFS):
        check(gpu, oracle_mod, wl.make_workload(5, n_snapshots=5, per_snapshot=3000, order_mode=mode))
    w = wl.make_workload(5, n_snapshots=5, per_snapshot=3000)
    w.workers[::4] = 1000
    check(gpu, oracle_mod, w)


def test_in_order_snapshot_larger_than_promised(gpu):
    w = wl.make_workload(5, n_snapshots=4, per_snapshot=3000)
    s = gpu.Session(w, max_snapshot_requests=2000)
    s.run()
    s.results()
    assert s.status_word() & 1


def test_in_order_unaligned_buffers_and_graph(gpu, oracle_mod):
    """Views at odd offsets into larger allocations, and the calls recorded into a graph and replayed."""
    import torch
    w = wl.make_workload(5, n_snapshots=12, per_snapshot=6000)
    s, ref = check(gpu, oracle_mod, w)
    n = w.n
    for o32, o8 in ((1, 1), (2, 6), (4, 16)):
        def view32(src):
            big = torch.full((n + 32,), -7, dtype=torch.int32, device=s.dev)
            v = big[o32:o32 + n]
            if src is not None:
                v.copy_(src)
            return big, v
        _, deadline = view32(s.deadline)
        _, stage = view32(s.stage)
        est_big, est = view32(None)
        order_big, order = view32(None)
        drop_big = torch.full((n + 64,), 9, dtype=torch.uint8, device=s.dev)
        drop = drop_big[o8:o8 + n]
        gpu.pard_estimate_drop(s.plan, n, s.max_snap, None, deadline, stage, s.snap_ptr, s.now, est, drop, order, s.seg_ptr,
                               s.workspace)
        torch.cuda.synchronize()
        assert np.array_equal(est.cpu().numpy(), ref["est"]) and np.array_equal(drop.cpu().numpy(), ref["drop"])
        assert np.array_equal(order.cpu().numpy(), ref["order"]) and np.array_equal(s.seg_ptr.cpu().numpy(), ref["seg_ptr"])
        for big, off in ((est_big, o32), (order_big, o32)):
            h = big.cpu().numpy()
            assert (h[:off] == -7).all() and (h[off + n:] == -7).all()
        h = drop_big.cpu().numpy()
        assert (h[:o8] == 9).all() and (h[o8 + n:] == 9).all()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s.run()
    base_now = w.now.copy()
    for shift in (0, -150_000, -400_000, 0):
        w.now[:] = np.maximum(-2**31, base_now.astype(np.int64) + shift).astype(np.int32)
        s.now.copy_(torch.from_numpy(w.now).to(s.dev))
        s.est.zero_(); s.drop.zero_(); s.order.zero_(); s.surv_idx.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = s.results()
        want = oracle_mod.run(w, threads=8)
        for k in KEYS:
            assert np.array_equal(got[k], want[k]), (shift, k)
