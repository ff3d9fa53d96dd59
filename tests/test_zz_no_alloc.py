"""The entry point that allocates nothing: pard_estimate_drop_static runs pard_estimate_drop's kernels on the
scratch buffer that is part of the library's device image.  Its outputs must equal pard_estimate_drop's (and
the oracle's) bit for bit, on calls in a row that share the buffer, the later ones smaller than the first."""
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


def _both(gpu, oracle_mod, w, max_snap):
    import torch
    print(f"case {w.name} n={w.n} max_snap={max_snap}", flush=True)
    s = gpu.Session(w, max_snapshot_requests=max_snap)
    s.estimate_drop()
    want = {k: getattr(s, k).clone() for k in ("est", "drop", "order", "seg_ptr")}
    for t in (s.est, s.drop, s.order, s.seg_ptr):
        t.fill_(0x55)
    status = torch.full((1,), 77, dtype=torch.int32, device=s.dev)
    if not _both.warm:
        # the first call on a device looks up the buffer's address, and the runtime may place the library's
        # device image only then; every later call must leave the free device memory as it is
        gpu.pard_estimate_drop_static(s.plan, s.n, s.max_snap, s.arrival, s.deadline, s.stage, s.snap_ptr, s.now,
                                      s.est, s.drop, s.order, s.seg_ptr, None)
        torch.cuda.synchronize()
        _both.warm = True
    free_before = torch.cuda.mem_get_info()[0]
    gpu.pard_estimate_drop_static(s.plan, s.n, s.max_snap, s.arrival, s.deadline, s.stage, s.snap_ptr, s.now,
                                  s.est, s.drop, s.order, s.seg_ptr, status)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before        # nothing was allocated on the device
    for k, v in want.items():
        assert torch.equal(getattr(s, k), v), (w.name, k)
    assert int(status.item()) == 0
    ref = oracle_mod.run(w, threads=8)
    n = w.n
    assert np.array_equal(s.est[:n].cpu().numpy(), ref["est"]) and np.array_equal(s.drop[:n].cpu().numpy(), ref["drop"])
    assert np.array_equal(s.order[:n].cpu().numpy(), ref["order"]) and np.array_equal(s.seg_ptr.cpu().numpy(), ref["seg_ptr"])


_both.warm = False


def test_static_scratch_calls_in_a_row(gpu, oracle_mod):
    # large-snapshot path (the kernels keep keys, counters and partial results in the buffer): a call, then
    # smaller ones over the contents the first one left behind, then the on-chip path and the first size again
    first = wl.make_workload(3, n_requests=300_001, permute=True)
    first.now[:] = np.maximum(0, first.now.astype(np.int64) - 280000).astype(np.int32)
    first.lat_us[:] = np.maximum(1, first.lat_us // 400)
    _both(gpu, oracle_mod, first, FORCE_SORT)
    _both(gpu, oracle_mod, wl.make_workload(3, n_requests=70_001, permute=True), FORCE_SORT)
    _both(gpu, oracle_mod, wl.make_workload(4, n_requests=9_000, permute=True), FORCE_SORT)
    _both(gpu, oracle_mod, wl.make_workload(5, n_snapshots=7, per_snapshot=5000, permute=True), None)
    _both(gpu, oracle_mod, wl.make_workload(5, n_snapshots=3, per_snapshot=100, permute=True), None)
    _both(gpu, oracle_mod, first, FORCE_SORT)


def test_static_scratch_at_its_limit(gpu, oracle_mod):
    """The largest request count of the large-snapshot path the built-in buffer serves (found by asking: one request
    more is refused with PARD_E_SCRATCH before anything is launched): the call uses the buffer up to its last tables
    and gives the oracle's results; a smaller call right after it shares the buffer."""
    probe = gpu.Session(wl.make_workload(3, n_requests=1000), max_snapshot_requests=FORCE_SORT)

    def fits(n):
        return gpu.pard_estimate_drop_static(probe.plan, n, FORCE_SORT, probe.arrival, None, probe.stage, probe.snap_ptr,
                                             probe.now, probe.est, probe.drop, probe.order, probe.seg_ptr, None,
                                             check=False) != -12
    lo, hi = 1000, 4_000_000                       # fits(lo), not fits(hi); the null deadline keeps every probe from launching
    assert fits(lo) and not fits(hi)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if fits(mid):
            lo = mid
        else:
            hi = mid
    assert 1_000_000 < lo < 2_000_000, lo
    _both(gpu, oracle_mod, wl.make_workload(3, n_requests=lo, permute=True), None)      # one snapshot: the promise is its size
    _both(gpu, oracle_mod, wl.make_workload(4, n_requests=123_457, permute=True), FORCE_SORT)


def test_static_scratch_limits_and_status(gpu):
    import torch
    w = wl.make_workload(2, n_requests=1000)
    s = gpu.Session(w, max_snapshot_requests=FORCE_SORT)
    # a request count whose sort buffers exceed the built-in buffer is refused before anything is launched
    assert gpu.pard_estimate_drop_static(s.plan, 4_000_000, FORCE_SORT, s.arrival, s.deadline, s.stage, s.snap_ptr, s.now,
                                         s.est, s.drop, s.order, s.seg_ptr, None, check=False) == -12
    assert gpu.pard_estimate_drop_static(s.plan, -1, FORCE_SORT, s.arrival, s.deadline, s.stage, s.snap_ptr, s.now,
                                         s.est, s.drop, s.order, s.seg_ptr, None, check=False) == -2
    assert gpu.pard_estimate_drop_static(s.plan, s.n, FORCE_SORT, s.arrival, None, s.stage, s.snap_ptr, s.now,
                                         s.est, s.drop, s.order, s.seg_ptr, None, check=False) == -1
    assert b"scratch" in gpu.load_library().pard_strerror(-12)
    # on the on-chip path any request count fits: the buffer only holds the status word there
    big = wl.make_workload(5, n_snapshots=600, per_snapshot=8192)
    sb = gpu.Session(big)
    status = torch.zeros(1, dtype=torch.int32, device=sb.dev)
    gpu.pard_estimate_drop_static(sb.plan, sb.n, sb.max_snap, sb.arrival, sb.deadline, sb.stage, sb.snap_ptr, sb.now,
                                  sb.est, sb.drop, sb.order, sb.seg_ptr, status)
    got = {k: getattr(sb, k).clone() for k in ("est", "drop", "order", "seg_ptr")}
    sb.estimate_drop()
    torch.cuda.synchronize()
    for k, v in got.items():
        assert torch.equal(getattr(sb, k), v), k
    assert int(status.item()) == 0
    # a snapshot larger than promised raises bit 0 in the buffer; taking the status clears it for the next call
    small = wl.make_workload(5, n_snapshots=4, per_snapshot=500)
    ss = gpu.Session(small, max_snapshot_requests=100)
    gpu.pard_estimate_drop_static(ss.plan, ss.n, 100, ss.arrival, ss.deadline, ss.stage, ss.snap_ptr, ss.now,
                                  ss.est, ss.drop, ss.order, ss.seg_ptr, status)
    torch.cuda.synchronize()
    assert int(status.item()) & 1
    gpu.pard_estimate_drop_static(sb.plan, sb.n, sb.max_snap, sb.arrival, sb.deadline, sb.stage, sb.snap_ptr, sb.now,
                                  sb.est, sb.drop, sb.order, sb.seg_ptr, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
