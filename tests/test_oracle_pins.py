"""Pins of the CPU oracle (no GPU): hand vector, brute force, closed forms, invariants.

The paper prints no number for the estimate/drop path, so the oracle is pinned by
what the definition and the mathematics fix.
"""
import json
import os

import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl
from tests.bruteforce import brute

INT32_MAX = 2**31 - 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _workload(S, edges, batch, workers, lat, mode, arrival, deadline, stage, now, K=1, snap_ptr=None):
    rp, cl = wl.csr_from_edges(S, edges)
    n = len(deadline)
    return wl.Workload(
        name="t", K=K, S=S, dag_shared=1, dag_row_ptr=rp, dag_col=cl,
        batch=np.asarray(batch, np.int32), workers=np.asarray(workers, np.int32),
        lat_us=np.asarray(lat, np.int32).reshape(-1), order_mode=np.asarray(mode, np.int32),
        arrival=np.asarray(arrival, np.int32), deadline=np.asarray(deadline, np.int32),
        stage=np.asarray(stage, np.int32),
        snap_ptr=np.asarray([0, n] if snap_ptr is None else snap_ptr, np.int32),
        now=np.asarray(now, np.int32).reshape(-1))


def test_hand_vector_diamond(oracle_mod):
    g = json.load(open(os.path.join(GOLDEN, "diamond_hand_vector.json")))
    b = np.arange(1, 65)
    lat = np.asarray(g["lat_affine_a"])[:, None] + np.asarray(g["lat_affine_c"])[:, None] * b[None, :]
    n = len(g["deadline"])
    w = _workload(g["S"], g["edges"], g["batch"], g["workers"], lat, [wl.MODE_LBF] * g["S"],
                  [0] * n, g["deadline"], g["stage"], [g["now"]])
    r = oracle_mod.run(w)
    assert r["est"].tolist() == g["expect_est"]
    assert r["drop"].tolist() == g["expect_drop"]
    assert r["order"].tolist() == g["expect_order"]
    assert r["seg_ptr"].tolist() == g["expect_seg_ptr"]
    assert r["surv_idx"].tolist() == g["expect_surv_idx"]
    assert r["surv_ptr"].tolist() == g["expect_surv_ptr"]


@pytest.mark.parametrize("seed", range(24))
def test_bruteforce_small_random(oracle_mod, seed):
    """Random DAGs, all order modes, ragged multi-snapshot batches, arbitrary tables."""
    K = 1 + seed % 3
    S = 1 + seed % 6
    w = wl.random_workload(seed, K=K, S=S, n_per_snapshot=10 + seed, monotone=(seed % 2 == 0),
                           tie_heavy=(seed % 4 == 3))
    r = oracle_mod.run(w)
    est, drop, pos = brute(w)
    assert r["est"].tolist() == est
    assert r["drop"].tolist() == drop
    # order: position inside its segment equals the number of requests ahead
    seg = r["seg_ptr"]
    for g in range(w.K * w.S):
        for j in range(seg[g], seg[g + 1]):
            assert pos[r["order"][j]] == j - seg[g]
    assert sorted(r["order"].tolist()) == list(range(w.n))


def test_paths_match_longest_path_dp(oracle_mod):
    """max over enumerated paths == longest-path dynamic programme; path counts by DP."""
    for seed in range(20):
        rng = np.random.default_rng(seed)
        S = int(rng.integers(1, 9))
        rp, cl = wl.random_dag(rng, S, 0.4)
        ptr, stg = oracle_mod.expand_paths(S, rp, cl)
        assert len(ptr) - 1 == wl.count_paths_any_order(S, rp, cl)
        weight = rng.integers(1, 1000, size=S)
        best_from = np.zeros(S, dtype=np.int64)      # heaviest path starting at s (DP, memoised DFS)
        done = [False] * S

        def go(s):
            if done[s]:
                return best_from[s]
            m = 0
            for e in range(rp[s], rp[s + 1]):
                m = max(m, go(int(cl[e])))
            best_from[s] = weight[s] + m
            done[s] = True
            return best_from[s]

        for s in range(S):
            go(s)
        for s in range(S):
            via_paths = 0
            for p in range(len(ptr) - 1):
                nodes = stg[ptr[p]:ptr[p + 1]].tolist()
                if s in nodes:
                    via_paths = max(via_paths, int(weight[nodes[nodes.index(s):]].sum()))
            assert via_paths == best_from[s]


def test_bad_dags_rejected(oracle_mod):
    with pytest.raises(ValueError):
        oracle_mod.expand_paths(3, *wl.csr_from_edges(3, [(0, 1), (1, 2), (2, 0)]))
    with pytest.raises(ValueError):     # cycle not reachable from the only source
        oracle_mod.expand_paths(3, *wl.csr_from_edges(3, [(1, 2), (2, 1)]))
    rp, cl = wl.csr_from_edges(2, [(0, 1)])
    with pytest.raises(ValueError):
        oracle_mod.expand_paths(2, rp, np.asarray([5], np.int32))


def test_stage_cost_against_batch_simulation(oracle_mod):
    """W=1: the wait equals the time a single worker needs to run the batches ahead,
    simulated batch by batch; execution uses the batch the request lands in."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        lat = np.sort(rng.integers(1, 50000, size=64)).astype(np.int32)
        B = int(rng.integers(1, 65))
        a = int(rng.integers(0, 500))
        t, left = 0, a
        while left > 0:          # batches of the configured size are charged at lat[B]
            left -= min(B, left)
            t += int(lat[B - 1])
        mine = min(B, a + 1)
        assert oracle_mod.stage_cost(lat, B, 1, a) == t + int(lat[mine - 1])
    # W workers: floor of the exact quotient, multiplied before dividing
    lat = np.full(64, 7, np.int32)
    assert oracle_mod.stage_cost(lat, 1, 2, 3) == (3 * 7) // 2 + 7
    assert oracle_mod.stage_cost(lat, 1, 4, 3) == 5 + 7
    assert oracle_mod.stage_cost(lat, 64, 3, 0) == 7
    big = np.full(64, INT32_MAX, np.int32)
    assert oracle_mod.stage_cost(big, 1, 1, INT32_MAX) == INT32_MAX * INT32_MAX + INT32_MAX


def test_linear_pipeline_is_single_suffix_sum(oracle_mod):
    """Chain: one path, so est = own-stage cost + sum of downstream costs at full queue length."""
    w = wl.make_workload(2, n_requests=3000)
    r = oracle_mod.run(w)
    S = w.S
    lat = w.lat_us.reshape(S, 64)
    qlen = np.bincount(w.stage, minlength=S)
    c_full = [oracle_mod.stage_cost(lat[s], w.batch[s], w.workers[s], int(qlen[s])) for s in range(S)]
    suffix = np.concatenate([np.cumsum(c_full[::-1])[::-1][1:], [0]])
    seg = r["seg_ptr"]
    for s in range(S):
        for j in range(seg[s], seg[s + 1]):
            rid = r["order"][j]
            own = oracle_mod.stage_cost(lat[s], w.batch[s], w.workers[s], j - seg[s])
            assert r["est"][rid] == min(own + suffix[s], INT32_MAX)


def test_lone_request_sees_batch1_latencies(oracle_mod):
    """One request, all queues otherwise empty: est = worst path sum of lat[1]."""
    w4 = wl.make_workload(4, n_requests=1)
    S = w4.S
    lat1 = w4.lat_us.reshape(S, 64)[:, 0].astype(np.int64)
    rp, cl = w4.dag_row_ptr, w4.dag_col

    def worst(s):
        return lat1[s] + max([worst(int(cl[e])) for e in range(rp[s], rp[s + 1])], default=0)

    for k in range(S):
        w4.stage[:] = k
        r = oracle_mod.run(w4)
        assert r["est"][0] == worst(k)


def test_single_stage_unit_batch_is_rank_times_latency(oracle_mod):
    """S=1, B=1, W=1, constant table: est = (rank+1)*lat with rank from a library sort."""
    rng = np.random.default_rng(11)
    n = 500
    deadline = rng.integers(0, 300, size=n)          # many ties
    w = _workload(1, [], [1], [1], np.full((1, 64), 37), [wl.MODE_LBF], np.zeros(n), deadline,
                  np.zeros(n), [0])
    r = oracle_mod.run(w)
    rank = np.empty(n, np.int64)
    rank[np.lexsort((np.arange(n), deadline))] = np.arange(n)
    assert np.array_equal(r["est"], (rank + 1) * 37)
    assert np.array_equal(r["order"], np.lexsort((np.arange(n), deadline)))
    # HBF: descending deadline, ties still by ascending index
    w.order_mode[:] = wl.MODE_HBF
    r = oracle_mod.run(w)
    assert np.array_equal(r["order"], np.lexsort((np.arange(n), -deadline)))
    # FCFS: arrival order
    w.order_mode[:] = wl.MODE_FCFS
    w.arrival[:] = rng.integers(0, 100, size=n)
    r = oracle_mod.run(w)
    assert np.array_equal(r["order"], np.lexsort((np.arange(n), w.arrival)))


def test_infinite_deadline_never_dropped_and_saturation(oracle_mod):
    n = 300
    lat = np.full((2, 64), INT32_MAX)
    w = _workload(2, [(0, 1)], [1, 1], [1, 1], lat, [0, 0], np.zeros(n), np.full(n, INT32_MAX),
                  np.arange(n) % 2, [INT32_MAX])
    r = oracle_mod.run(w)
    assert np.all(r["est"] == INT32_MAX) and not r["drop"].any()
    w.deadline[::3] = INT32_MAX - 1
    r = oracle_mod.run(w)
    assert np.array_equal(r["drop"], (w.deadline < INT32_MAX).astype(np.uint8))


def test_uniform_deadline_shift_is_monotone(oracle_mod):
    for cfg in (1, 3):
        w = wl.make_workload(cfg, n_requests=4000, permute=True)
        w.now[:] = int(np.median(w.deadline)) - 150000
        r0 = oracle_mod.run(w)
        prev = r0
        for delta in (1, 1000, 50000, 10**6):
            w2 = wl.make_workload(cfg, n_requests=4000, permute=True)
            w2.now[:] = w.now
            w2.deadline[:] = w.deadline + delta
            r = oracle_mod.run(w2)
            assert np.array_equal(r["order"], r0["order"]) and np.array_equal(r["est"], r0["est"])
            assert not np.any(r["drop"] & ~prev["drop"].astype(bool))   # drop set only shrinks
            prev = r
        assert 0 < r0["drop"].mean() < 1


def test_estimates_monotone_in_load(oracle_mod):
    """More latency, fewer workers or one more queued request never lowers an estimate."""
    w = wl.make_workload(3, n_requests=2000, permute=True)
    base = oracle_mod.run(w)["est"].astype(np.int64)
    w2 = wl.make_workload(3, n_requests=2000, permute=True)
    w2.lat_us[:] = w.lat_us + 17
    assert np.all(oracle_mod.run(w2)["est"] >= base)
    w3 = wl.make_workload(3, n_requests=2000, permute=True)
    w3.workers[:] = np.maximum(1, w.workers - 1)
    assert np.all(oracle_mod.run(w3)["est"] >= base)
    w4 = wl.make_workload(3, n_requests=2001, permute=False)
    w5 = wl.make_workload(3, n_requests=2001, permute=False)
    for a in ("arrival", "deadline", "stage"):       # same requests plus one more at the end
        getattr(w5, a)[:2000] = getattr(w4, a)[:2000]
    r4 = oracle_mod.estimate_drop(w4.K, w4.S, 1, w4.dag_row_ptr, w4.dag_col, w4.batch, w4.workers, w4.lat_us,
                                  w4.order_mode, w4.arrival[:2000], w4.deadline[:2000], w4.stage[:2000],
                                  np.asarray([0, 2000], np.int32), w4.now)[0]
    r5 = oracle_mod.run(w5)["est"][:2000]
    assert np.all(r5.astype(np.int64) >= r4)


def test_permutation_invariance(oracle_mod):
    """Shuffling the input changes nothing but the order of equal keys."""
    w = wl.make_workload(5, n_snapshots=3, per_snapshot=700)
    rng = np.random.default_rng(3)
    # make keys unique inside each snapshot so that tie order cannot differ
    for u in range(w.K):
        lo, hi = w.snap_ptr[u], w.snap_ptr[u + 1]
        w.deadline[lo:hi] = w.deadline[lo] + rng.permutation(hi - lo) * 13
    r = oracle_mod.run(w)
    perm = np.concatenate([w.snap_ptr[u] + rng.permutation(w.snap_ptr[u + 1] - w.snap_ptr[u])
                           for u in range(w.K)])
    w2 = wl.make_workload(5, n_snapshots=3, per_snapshot=700)
    w2.deadline[:] = w.deadline[perm]
    w2.arrival[:] = w.arrival[perm]
    w2.stage[:] = w.stage[perm]
    r2 = oracle_mod.run(w2)
    assert np.array_equal(r2["est"], r["est"][perm])
    assert np.array_equal(r2["drop"], r["drop"][perm])
    assert np.array_equal(perm[r2["order"]], r["order"])
    assert np.array_equal(perm[r2["surv_idx"]], r["surv_idx"])


def test_compaction_invariants(oracle_mod):
    for cfg, kw in ((1, {}), (5, dict(n_snapshots=5, per_snapshot=900)), (3, dict(n_requests=5000))):
        w = wl.make_workload(cfg, permute=True, **kw)
        w.now[:] = (w.now.astype(np.int64) - 250000).clip(0)
        r = oracle_mod.run(w)
        keep = ~r["drop"].astype(bool)
        assert r["surv_ptr"][-1] == keep.sum() == len(r["surv_idx"])
        assert np.array_equal(r["surv_idx"], r["order"][keep[r["order"]]])     # subsequence of order
        per_seg = np.add.reduceat(np.concatenate([keep[r["order"]].astype(np.int64), [0]]),
                                  np.minimum(r["seg_ptr"][:-1], w.n))
        per_seg[np.diff(r["seg_ptr"]) == 0] = 0
        assert np.array_equal(np.diff(r["surv_ptr"]), per_seg)


def test_out_of_range_stage_reads_as_nearest(oracle_mod):
    w = wl.make_workload(1, n_requests=200)
    w2 = wl.make_workload(1, n_requests=200)
    w2.stage[::7] = -5
    w2.stage[3::7] = 99
    w.stage[::7] = 0
    w.stage[3::7] = w.S - 1
    a, b = oracle_mod.run(w), oracle_mod.run(w2)
    for k in a:
        assert np.array_equal(a[k], b[k])


def test_empty_and_singleton(oracle_mod):
    w = wl.make_workload(3, n_requests=0)
    r = oracle_mod.run(w)
    assert r["est"].size == 0 and r["seg_ptr"].tolist() == [0] * (w.S + 1) and r["surv_ptr"].tolist() == [0] * (w.S + 1)
    w = wl.random_workload(1, K=4, S=3, n_per_snapshot=0, vary_sizes=False)
    r = oracle_mod.run(w)
    assert r["seg_ptr"].tolist() == [0] * 13


def test_threads_do_not_change_results(oracle_mod):
    w = wl.make_workload(5, n_snapshots=6, per_snapshot=500, permute=True)
    a, b = oracle_mod.run(w, threads=1), oracle_mod.run(w, threads=4)
    for k in a:
        assert np.array_equal(a[k], b[k])
