"""Pins of the oracle's ranked variant (in later queues a request counts only the requests their
order serves before it).  Expected values come from a hand-worked pipeline, from the independent
brute force in tests/bruteforce.py (it inserts the newcomer into the later queue and sorts) and from
the cases in which the variant must equal the plain estimate - never from the C oracle itself."""
import numpy as np
import pytest

from tests import bruteforce
from paper_2602_08747_amd import workloads as wl


def two_stage(deadlines0, deadlines1, mode1, lat0=100, lat1=1000, now=0):
    """Chain 0 -> 1, B = 1, W = 1 everywhere: cost_s(a) = (a + 1) * lat_s."""
    rp, cl = wl.csr_from_edges(2, wl.chain_edges(2))
    n0, n1 = len(deadlines0), len(deadlines1)
    lat = np.concatenate([np.full(64, lat0), np.full(64, lat1)]).astype(np.int32)
    return dict(K=1, S=2, dag_shared=1, dag_row_ptr=rp, dag_col=cl, batch=np.ones(2, np.int32), workers=np.ones(2, np.int32),
                lat_us=lat, order_mode=np.array([0, mode1], np.int32), arrival=np.arange(n0 + n1, dtype=np.int32),
                deadline=np.asarray(list(deadlines0) + list(deadlines1), np.int32),
                stage=np.array([0] * n0 + [1] * n1, np.int32), snap_ptr=np.array([0, n0 + n1], np.int32),
                now=np.array([now], np.int32))


def test_hand_worked_two_stages(oracle_mod):
    """Stage 1 holds deadlines 3000, 5000, 5000, 9000.  A request of stage 0 with deadline d, at position p:
    est = (p + 1) * 100 + (ahead + 1) * 1000, ahead = requests of stage 1 served before a newcomer with d.
      low budget first at stage 1 (those with deadline <= d):   d = 2000: 0, 5000: 3, 8000: 3, 9000: 4
      high budget first (those with deadline >= d):             d = 2000: 4, 5000: 3, 8000: 1, 9000: 1
      arrival order: everybody, 4.
    Stage 0 (low budget first) is ordered 2000, 5000, 8000, 9000 -> positions 0..3."""
    own = [100, 200, 300, 400]
    for mode1, ahead in ((0, [0, 3, 3, 4]), (1, [4, 3, 1, 1]), (2, [4, 4, 4, 4])):
        w = two_stage([2000, 5000, 8000, 9000], [3000, 5000, 5000, 9000], mode1)
        est, drop, _, _ = oracle_mod.estimate_drop(**w, ranked=True)
        want = [o + (a + 1) * 1000 for o, a in zip(own, ahead)]
        assert est[:4].tolist() == want, (mode1, est[:4].tolist(), want)
        assert drop[:4].tolist() == [int(e > d) for e, d in zip(want, [2000, 5000, 8000, 9000])]
        # the requests of the last stage have nothing after them: as in the plain estimate
        plain, _, _, _ = oracle_mod.estimate_drop(**w)
        assert est[4:].tolist() == plain[4:].tolist()
        assert plain[:4].tolist() == [o + 5000 for o in own]


@pytest.mark.parametrize("seed", range(24))
def test_bruteforce_small_random(oracle_mod, seed):
    w = wl.random_workload(800 + seed, K=1 + seed % 3, S=1 + (seed * 7) % 6, n_per_snapshot=10 + seed,
                           monotone=(seed % 2 == 0), tie_heavy=(seed % 3 == 0))
    est, drop, order, seg_ptr = oracle_mod.estimate_drop(
        w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, w.order_mode,
        w.arrival, w.deadline, w.stage, w.snap_ptr, w.now, ranked=True)
    b_est, b_drop, _ = bruteforce.brute(w, ranked=True)
    assert est.tolist() == b_est
    assert drop.tolist() == b_drop
    plain = oracle_mod.estimate_drop(
        w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, w.order_mode,
        w.arrival, w.deadline, w.stage, w.snap_ptr, w.now)
    assert np.array_equal(order, plain[2]) and np.array_equal(seg_ptr, plain[3])      # the queues themselves do not change


def test_equals_the_plain_estimate_when_it_must(oracle_mod):
    """A request whose budget is the largest of the whole snapshot is last in every low-budget-first queue
    (ties go to the ones already there), so it sees whole queues; so does everybody in arrival order; and a
    single stage has no later queue at all."""
    w = wl.random_workload(850, K=2, S=5, n_per_snapshot=60, modes=(wl.MODE_LBF,), monotone=False)
    last = [int(np.argmax(np.where((np.arange(w.n) >= w.snap_ptr[u]) & (np.arange(w.n) < w.snap_ptr[u + 1]), w.deadline.astype(np.int64), -1)))
            for u in range(w.K)]
    r, p = oracle_mod.run(w, ranked=True), oracle_mod.run(w)
    for i in last:
        assert r["est"][i] == p["est"][i]
    w = wl.random_workload(851, K=2, S=5, n_per_snapshot=60, modes=(wl.MODE_FCFS,))
    assert np.array_equal(oracle_mod.run(w, ranked=True)["est"], oracle_mod.run(w)["est"])
    w = wl.random_workload(852, K=3, S=1, n_per_snapshot=40)
    assert np.array_equal(oracle_mod.run(w, ranked=True)["est"], oracle_mod.run(w)["est"])


def test_never_above_the_plain_estimate_with_rising_tables(oracle_mod):
    """Fewer requests ahead cannot cost more when the latency table rises with the batch size."""
    for seed in range(6):
        w = wl.random_workload(860 + seed, K=2, S=4 + seed, n_per_snapshot=80, monotone=True)
        r, p = oracle_mod.run(w, ranked=True), oracle_mod.run(w)
        assert (r["est"] <= p["est"]).all()
        assert (r["drop"] <= p["drop"]).all()
