"""Pins of the oracle's reactive baselines (Section 5.1 "Baselines": the Nexus window scan and the Clipper++
per-module SLO split).  Expected values come from hand-worked queues, closed forms and independent Python brute
forces written from the definitions (Python integers and Fractions) - never from the C oracle itself.
The paper prints no value for either rule."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

INT32_MAX = 2**31 - 1


def one_queue(deadlines, B, lat, now):
    """A single stage holding `deadlines` in scan order; lat: dict batch size -> latency (others 0)."""
    n = len(deadlines)
    table = np.zeros(64, np.int32)
    for b, v in lat.items():
        table[b - 1] = v
    return dict(K=1, S=1, dag_shared=1, batch=np.array([B], np.int32), lat_us=table, deadline=np.asarray(deadlines, np.int32),
                order=np.arange(n, dtype=np.int32), seg_ptr=np.array([0, n], np.int32), now=np.array([now], np.int32))


def test_nexus_hand_worked_queues(oracle_mod):
    """B = 2, a batch of two takes 150, a batch of one 100, now = 1000: a window of two meets the budget when both
    deadlines are >= 1150, the last window (one request) when its deadline is >= 1100.
        deadlines 1100 1200 1140 1160 1300 1090
        p=0 {1100,1200} no, p=1 {1200,1140} no, p=2 {1140,1160} no, p=3 {1160,1300} yes -> first_kept 3
    """
    drop, first = oracle_mod.nexus_drop(**one_queue([1100, 1200, 1140, 1160, 1300, 1090], 2, {1: 100, 2: 150}, 1000))
    assert first.tolist() == [3] and drop.tolist() == [1, 1, 1, 0, 0, 0]
    # only the cut-off last window fits: {1149, 1100}: p=0 needs both >= 1150, p=1 is a batch of one ending at 1100
    drop, first = oracle_mod.nexus_drop(**one_queue([1149, 1100], 2, {1: 100, 2: 150}, 1000))
    assert first.tolist() == [1] and drop.tolist() == [1, 0]
    # exactly on the deadline is in time; one microsecond less is not
    drop, first = oracle_mod.nexus_drop(**one_queue([1150, 1150], 2, {1: 100, 2: 150}, 1000))
    assert first.tolist() == [0] and not drop.any()
    drop, first = oracle_mod.nexus_drop(**one_queue([1150, 1149, 1099], 2, {1: 100, 2: 150}, 1000))
    assert first.tolist() == [3] and drop.tolist() == [1, 1, 1]          # no window fits: everything is dropped
    # the queue is scanned in the order given, not by request index
    q = one_queue([1300, 1100, 1160, 1200], 2, {1: 100, 2: 150}, 1000)
    q["order"] = np.array([1, 3, 2, 0], np.int32)                         # scan 1100 1200 1160 1300
    drop, first = oracle_mod.nexus_drop(**q)
    assert first.tolist() == [1] and drop.tolist() == [0, 1, 0, 0]


def test_nexus_closed_forms(oracle_mod):
    rng = np.random.default_rng(3)
    for B in (1, 2, 7, 16, 64):
        lat = {b: 1000 + 10 * b for b in range(1, 65)}
        n = 300
        good = np.full(n, 50_000, np.int32)
        # everybody in time: nothing dropped
        drop, first = oracle_mod.nexus_drop(**one_queue(good, B, lat, 0))
        assert first.tolist() == [0] and not drop.any()
        # everybody late: everything dropped
        drop, first = oracle_mod.nexus_drop(**one_queue(np.zeros(n, np.int32), B, lat, 0))
        assert first.tolist() == [n] and drop.all()
        # one late request at position i in a queue of requests in time: the first window without it starts at 0
        # when it lies beyond the first window, right behind it otherwise
        for i in (0, 1, B - 1, B, B + 1, n - 2, n - 1):
            if not 0 <= i < n:
                continue
            dl = good.copy()
            dl[i] = 0
            drop, first = oracle_mod.nexus_drop(**one_queue(dl, B, lat, 0))
            want = 0 if i >= B else i + 1
            assert first.tolist() == [want], (B, i)
            assert drop.tolist() == [1] * want + [0] * (n - want)
    # B = 1: the first request whose own deadline allows a batch of one
    dl = rng.integers(0, 3000, 200).astype(np.int32)
    drop, first = oracle_mod.nexus_drop(**one_queue(dl, 1, {1: 1500}, 0))
    ok = np.flatnonzero(dl >= 1500)
    assert first.tolist() == [int(ok[0]) if ok.size else 200]


def brute_nexus(K, S, dag_shared, batch, lat_us, deadline, order, seg_ptr, now):
    n = len(deadline)
    drop = [0] * n
    first = []
    for u in range(K):
        for s in range(S):
            g = u * S + s
            rec = s if dag_shared else g
            B = int(batch[rec])
            q = [int(deadline[int(r)]) for r in order[int(seg_ptr[g]):int(seg_ptr[g + 1])]]
            f = len(q)
            for p in range(len(q)):
                window = q[p:p + B]
                if min(window) >= int(now[u]) + int(lat_us[rec * 64 + len(window) - 1]):
                    f = p
                    break
            first.append(f)
            for j, r in enumerate(order[int(seg_ptr[g]):int(seg_ptr[g + 1])]):
                drop[int(r)] = 1 if j < f else 0
    return drop, first


@pytest.mark.parametrize("seed", range(16))
def test_nexus_brute_force(oracle_mod, seed):
    """Random pipelines and snapshots, queues in arrival order (the paper's baseline) or any other order."""
    modes = (wl.MODE_FCFS,) if seed % 2 == 0 else (wl.MODE_LBF, wl.MODE_HBF, wl.MODE_FCFS)
    w = wl.random_workload(7000 + seed, K=1 + seed % 4, S=1 + (seed * 3) % 7, n_per_snapshot=40 + 5 * seed, modes=modes,
                           monotone=(seed % 3 != 0), tie_heavy=(seed % 5 == 0), dag_shared=seed % 2,
                           slo_choices=(20000, 60000, 200000))
    _, _, order, seg_ptr = oracle_mod.estimate_drop(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers,
                                                    w.lat_us, w.order_mode, w.arrival, w.deadline, w.stage, w.snap_ptr, w.now)
    drop, first = oracle_mod.nexus_drop(w.K, w.S, w.dag_shared, w.batch, w.lat_us, w.deadline, order, seg_ptr, w.now)
    want_drop, want_first = brute_nexus(w.K, w.S, w.dag_shared, w.batch, w.lat_us, w.deadline, order, seg_ptr, w.now)
    assert first.tolist() == want_first and drop.tolist() == want_drop
    if seed in (1, 2, 3):
        assert 0 < sum(want_drop) < w.n             # not a vacuous comparison


def test_nexus_invariants(oracle_mod):
    w = wl.make_workload(5, n_snapshots=6, per_snapshot=900, order_mode=wl.MODE_FCFS)
    w.now[:] = w.now + 140_000                       # the older part of most queues is out of time
    _, _, order, seg_ptr = oracle_mod.estimate_drop(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers,
                                                    w.lat_us, w.order_mode, w.arrival, w.deadline, w.stage, w.snap_ptr, w.now)
    drop, first = oracle_mod.nexus_drop(w.K, w.S, w.dag_shared, w.batch, w.lat_us, w.deadline, order, seg_ptr, w.now)
    # the dropped requests of a queue are exactly its first first_kept ones
    for g in range(w.K * w.S):
        q = order[seg_ptr[g]:seg_ptr[g + 1]]
        assert drop[q].tolist() == [1] * first[g] + [0] * (len(q) - first[g])
    assert 0 < drop.mean() < 1
    # later deadlines never move the first kept position back
    drop2, first2 = oracle_mod.nexus_drop(w.K, w.S, w.dag_shared, w.batch, w.lat_us, w.deadline + 20_000, order, seg_ptr, w.now)
    assert (first2 <= first).all() and (first2 < first).any()


# ---- Clipper++ ------------------------------------------------------------------------------------

def chain(S, durations, B=1):
    rp, cl = wl.csr_from_edges(S, wl.chain_edges(S))
    lat = np.zeros((S, 64), np.int32)
    lat[:, B - 1] = durations
    return dict(K=1, S=S, dag_shared=1, dag_row_ptr=rp, dag_col=cl, batch=np.full(S, B, np.int32), lat_us=lat.reshape(-1))


def test_clipper_hand_worked(oracle_mod):
    """Four modules of equal duration, SLO 400: the budgets add up to 100, 200, 300, 400 through modules 0..3.
    A request sent at 0 that sits at module 2 is dropped once more than 300 have passed."""
    p = chain(4, [1000] * 4)
    req = dict(arrival=np.zeros(4, np.int32), deadline=np.full(4, 400, np.int32), stage=np.arange(4, dtype=np.int32),
               snap_ptr=np.array([0, 4], np.int32))
    for now, want in ((100, [0, 0, 0, 0]), (101, [1, 0, 0, 0]), (300, [1, 1, 0, 0]), (301, [1, 1, 1, 0]), (401, [1, 1, 1, 1])):
        assert oracle_mod.clipper_drop(**p, **req, now=np.array([now], np.int32)).tolist() == want, now
    # unequal durations 10, 20, 50, 20 (batch size 3, the table's third column), SLO 1000, sent at 5000:
    # budgets through the modules 100, 300, 800, 1000
    p = chain(4, [10, 20, 50, 20], B=3)
    req = dict(arrival=np.full(4, 5000, np.int32), deadline=np.full(4, 6000, np.int32), stage=np.arange(4, dtype=np.int32),
               snap_ptr=np.array([0, 4], np.int32))
    for now, want in ((5100, [0, 0, 0, 0]), (5101, [1, 0, 0, 0]), (5301, [1, 1, 0, 0]), (5800, [1, 1, 0, 0]), (5801, [1, 1, 1, 0]),
                      (6000, [1, 1, 1, 0]), (6001, [1, 1, 1, 1])):
        assert oracle_mod.clipper_drop(**p, **req, now=np.array([now], np.int32)).tolist() == want, now
    # a diamond 0 -> {1, 2} -> 3 with durations 10, 20, 50, 10: longest way in 10, 30, 60, 70; whole path through
    # each stage 70, 40, 70, 70; SLO 700 -> budgets 100, 525, 600, 700
    rp, cl = wl.csr_from_edges(4, [(0, 1), (0, 2), (1, 3), (2, 3)])
    lat = np.zeros((4, 64), np.int32)
    lat[:, 0] = [10, 20, 50, 10]
    p = dict(K=1, S=4, dag_shared=1, dag_row_ptr=rp, dag_col=cl, batch=np.ones(4, np.int32), lat_us=lat.reshape(-1))
    req = dict(arrival=np.zeros(4, np.int32), deadline=np.full(4, 700, np.int32), stage=np.arange(4, dtype=np.int32),
               snap_ptr=np.array([0, 4], np.int32))
    for now, want in ((100, [0, 0, 0, 0]), (101, [1, 0, 0, 0]), (525, [1, 0, 0, 0]), (526, [1, 1, 0, 0]), (601, [1, 1, 1, 0]),
                      (701, [1, 1, 1, 1])):
        assert oracle_mod.clipper_drop(**p, **req, now=np.array([now], np.int32)).tolist() == want, now


def test_clipper_single_module_is_the_plain_rule(oracle_mod):
    """One module: dropped exactly when the deadline has passed (Clipper's own rule); also the last module of any
    pipeline, whose budgets add up to the whole SLO; also when every duration is zero."""
    rng = np.random.default_rng(8)
    n = 500
    arrival = rng.integers(-1000, 50_000, n).astype(np.int32)
    deadline = (arrival + rng.integers(0, 30_000, n)).astype(np.int32)
    now = np.array([40_000], np.int32)
    p = chain(1, [777])
    got = oracle_mod.clipper_drop(**p, arrival=arrival, deadline=deadline, stage=np.zeros(n, np.int32),
                                  snap_ptr=np.array([0, n], np.int32), now=now)
    assert got.tolist() == (now[0] > deadline).astype(int).tolist()
    p = chain(5, [300, 10, 4000, 1, 90])
    got = oracle_mod.clipper_drop(**p, arrival=arrival, deadline=deadline, stage=np.full(n, 4, np.int32),
                                  snap_ptr=np.array([0, n], np.int32), now=now)
    assert got.tolist() == (now[0] > deadline).astype(int).tolist()
    p = chain(3, [0, 0, 0])
    got = oracle_mod.clipper_drop(**p, arrival=arrival, deadline=deadline, stage=rng.integers(0, 3, n).astype(np.int32),
                                  snap_ptr=np.array([0, n], np.int32), now=now)
    assert got.tolist() == (now[0] > deadline).astype(int).tolist()


def brute_clipper(w):
    D = 1 if w.dag_shared else w.K
    rows = w.dag_row_ptr.reshape(D, w.S + 1)
    cols = np.split(w.dag_col, np.cumsum(rows[:, -1])[:-1])
    drop = []
    for u in range(w.K):
        d = 0 if w.dag_shared else u
        succ = [[int(c) for c in cols[d][rows[d][v]:rows[d][v + 1]]] for v in range(w.S)]
        pred = [[a for a in range(w.S) if v in succ[a]] for v in range(w.S)]
        dur = [int(w.lat_us[(d * w.S + v) * 64 + int(w.batch[d * w.S + v]) - 1]) for v in range(w.S)]

        def way_in(v):
            return dur[v] + max([way_in(a) for a in pred[v]], default=0)

        def way_out(v):
            return max([dur[t] + way_out(t) for t in succ[v]], default=0)

        for r in range(int(w.snap_ptr[u]), int(w.snap_ptr[u + 1])):
            k = min(max(int(w.stage[r]), 0), w.S - 1)
            used = int(w.now[u]) - int(w.arrival[r])
            slo = int(w.deadline[r]) - int(w.arrival[r])
            P, T = way_in(k), way_in(k) + way_out(k)
            budget = Fraction(slo) if T == 0 else Fraction(slo * P, T)
            drop.append(1 if used > budget else 0)
    return drop


@pytest.mark.parametrize("seed", range(16))
def test_clipper_brute_force(oracle_mod, seed):
    w = wl.random_workload(7100 + seed, K=1 + seed % 4, S=1 + (seed * 3) % 7, n_per_snapshot=60, dag_shared=seed % 2,
                           monotone=(seed % 3 != 0), slo_choices=(20000, 60000, 200000))
    if seed % 4 == 0:
        w.stage[::7] = -3
        w.stage[3::11] = 99
    got = oracle_mod.clipper_drop(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.lat_us, w.arrival, w.deadline,
                                  w.stage, w.snap_ptr, w.now)
    want = brute_clipper(w)
    assert got.tolist() == want
    if seed in (1, 2, 3):
        assert 0 < sum(want) < w.n
