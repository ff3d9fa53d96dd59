"""Pins of the oracle's sequentially consistent dropping (a dropped request frees its slot).

Expected values come from a hand-worked queue, from the independent brute force in
tests/bruteforce.py (Python's sorted(), unbounded integers, recursion over successors) and from
identities - never from the C oracle itself."""
import numpy as np
import pytest

from tests import bruteforce
from paper_2602_08747_amd import workloads as wl


def single_stage(deadlines, lat, now=0):
    n = len(deadlines)
    rp, cl = wl.csr_from_edges(1, [])
    return dict(K=1, S=1, dag_shared=1, dag_row_ptr=rp, dag_col=cl, batch=np.ones(1, np.int32), workers=np.ones(1, np.int32),
                lat_us=np.full(64, lat, np.int32), order_mode=np.zeros(1, np.int32), arrival=np.zeros(n, np.int32),
                deadline=np.asarray(deadlines, np.int32), stage=np.zeros(n, np.int32), snap_ptr=np.array([0, n], np.int32),
                now=np.array([now], np.int32))


def test_hand_worked_queue(oracle_mod):
    """One stage, B = 1, W = 1, every latency L = 100: cost(a) = (a + 1) * 100.  Deadlines ascending
    (LBF).  One pass uses the raw position; the broker's order gives every dropped request's slot
    to the next one:
        deadline   99  100  199  200  250  300  301
        one pass   est 100 200 300 400 500 600 700 -> drop 1 1 1 1 1 1 1 except 100? (200 > 100: dropped)
        in order   a=0: 100 > 99 drop | a=0: 100 <= 100 keep | a=1: 200 > 199 drop | a=1: 200 keep |
                   a=2: 300 > 250 drop | a=2: 300 keep | a=3: 400 > 301 drop
    """
    w = single_stage([99, 100, 199, 200, 250, 300, 301], 100)
    est, drop, order, _ = oracle_mod.estimate_drop(**w, consistent=True)
    assert est.tolist() == [100, 100, 200, 200, 300, 300, 400]
    assert drop.tolist() == [1, 0, 1, 0, 1, 0, 1]
    assert order.tolist() == list(range(7))
    est1, drop1, _, _ = oracle_mod.estimate_drop(**w)
    assert est1.tolist() == [100, 200, 300, 400, 500, 600, 700] and drop1.tolist() == [1, 1, 1, 1, 1, 1, 1]


@pytest.mark.parametrize("seed", range(20))
def test_brute_force(oracle_mod, seed):
    K = 1 + seed % 4
    S = 1 + (seed * 3) % 7
    w = wl.random_workload(900 + seed, K=K, S=S, n_per_snapshot=25 + 3 * seed, monotone=(seed % 2 == 0),
                           tie_heavy=(seed % 3 == 0), dag_shared=seed % 2)
    if seed % 5 == 0:
        w.order_mode[:] = np.arange(w.order_mode.size) % 3
    ref = oracle_mod.run(w, consistent=True)
    est, drop, _ = bruteforce.brute(w, consistent=True)
    assert ref["est"].tolist() == est and ref["drop"].tolist() == drop


def test_nothing_dropped_equals_one_pass(oracle_mod):
    w = wl.make_workload(5, n_snapshots=5, per_snapshot=700, permute=True)
    w.deadline[:] = 2**31 - 1
    a = oracle_mod.run(w)
    b = oracle_mod.run(w, consistent=True)
    assert not a["drop"].any()
    for k in a:
        assert np.array_equal(a[k], b[k])


def test_everything_dropped_sees_an_empty_queue(oracle_mod):
    w = wl.make_workload(3, n_requests=3000, permute=True)
    w.deadline[:] = -5
    b = oracle_mod.run(w, consistent=True)
    assert b["drop"].all()
    stage = np.clip(w.stage, 0, w.S - 1)
    for k in range(w.S):
        e = b["est"][stage == k]
        assert (e == e[0]).all()              # every request of a queue was evaluated at position 0


def test_monotone_tables_never_raise_an_estimate(oracle_mod):
    """With non-decreasing latency tables the cost is non-decreasing in the position, positions only
    shrink, so no estimate grows and nobody kept by the one-pass decision is dropped."""
    w = wl.make_workload(5, n_snapshots=6, per_snapshot=2500, permute=True)
    w.now[:] = np.maximum(0, w.now.astype(np.int64) - 250000).astype(np.int32)
    a = oracle_mod.run(w)
    b = oracle_mod.run(w, consistent=True)
    assert (b["est"] <= a["est"]).all() and (b["drop"] <= a["drop"]).all()
    assert b["drop"].sum() < a["drop"].sum()
    assert np.array_equal(a["order"], b["order"]) and np.array_equal(a["seg_ptr"], b["seg_ptr"])


def test_with_given_downstream_latency(oracle_mod):
    w = wl.make_workload(3, n_requests=2000, permute=True)
    qlen = np.bincount(np.clip(w.stage, 0, w.S - 1), minlength=w.S).astype(np.int32)
    lower = oracle_mod.sub_latency(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, qlen, 1)
    a = oracle_mod.run(w, consistent=True)
    b = oracle_mod.run(w, consistent=True, sub=lower)
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert 0 < a["drop"].mean() < 1
