"""Seeded synthetic pipeline snapshots shaped like the paper's workloads.

The paper evaluates on 3- and 5-module chains and a fan-out/fan-in DAG
(Section 5.1, "Workload"), SLOs of 200-600 ms (Section 5.4) and bursty rate
traces.  None of those traces are available, so every input here is
synthetic: a pipeline description (DAG as successor CSR, batch sizes, worker
counts, 64-entry batch-latency tables, queue order mode) and one or more
queue snapshots (arrival, deadline, current stage per request, `now` per
snapshot).  All times are int32 microseconds.

This module only draws inputs.  It contains none of the estimator's
arithmetic; both the CPU oracle's tests and the GPU path's tests consume the
arrays it returns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import dataclasses

import numpy as np

BASE_SEED = 20260208

MODE_LBF = 0   # low budget first  : ascending deadline
MODE_HBF = 1   # high budget first : descending deadline
MODE_FCFS = 2  # arrival order     : ascending arrival

LAT_ENTRIES = 64


@dataclass
class Workload:
    """One plan (pipeline description) plus one batch of snapshots."""
    name: str
    K: int                      # snapshots
    S: int                      # stages per snapshot
    dag_shared: int             # 1: one DAG/tables for all snapshots
    dag_row_ptr: np.ndarray     # int32 [(shared?1:K)*(S+1)], offsets relative per DAG
    dag_col: np.ndarray         # int32 successor ids
    batch: np.ndarray           # int32 [D*S]
    workers: np.ndarray         # int32 [D*S]
    lat_us: np.ndarray          # int32 [D*S*64]
    order_mode: np.ndarray      # int32 [D*S]
    arrival: np.ndarray         # int32 [n]
    deadline: np.ndarray        # int32 [n]
    stage: np.ndarray           # int32 [n]
    snap_ptr: np.ndarray        # int32 [K+1]
    now: np.ndarray             # int32 [K]
    notes: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(self.arrival.shape[0])

    @property
    def num_dags(self) -> int:
        return 1 if self.dag_shared else self.K

    @property
    def max_snapshot_requests(self) -> int:
        if self.K == 0:
            return 0
        return int(np.max(np.diff(self.snap_ptr.astype(np.int64)))) if self.n else 0


def _rng(cfg: int, stream: int, seed: Optional[int] = None) -> np.random.Generator:
    base = BASE_SEED if seed is None else seed
    return np.random.default_rng([base + cfg, stream])


# --------------------------------------------------------------------------
# pipeline pieces
# --------------------------------------------------------------------------

def csr_from_edges(S: int, edges: Sequence[Sequence[int]]):
    """Successor CSR (row_ptr[S+1], col[E]) of one DAG given (src, dst) pairs."""
    succ: List[List[int]] = [[] for _ in range(S)]
    for a, b in edges:
        succ[a].append(b)
    row_ptr = np.zeros(S + 1, dtype=np.int32)
    col: List[int] = []
    for s in range(S):
        col.extend(succ[s])
        row_ptr[s + 1] = len(col)
    return row_ptr, np.asarray(col, dtype=np.int32)


def chain_edges(S: int):
    return [(i, i + 1) for i in range(S - 1)]


def affine_tables(rng: np.random.Generator, S: int) -> np.ndarray:
    """lat(b) = a + c*b, a in [2000,10000], c in [200,1500]  (config 1)."""
    a = rng.integers(2000, 10001, size=S)
    c = rng.integers(200, 1501, size=S)
    b = np.arange(1, LAT_ENTRIES + 1)
    return (a[:, None] + c[:, None] * b[None, :]).astype(np.int32)


def monotone_tables(rng: np.random.Generator, S: int) -> np.ndarray:
    """lat[1] in [2000,10000], non-negative increments in [0,1500], prefix-summed."""
    first = rng.integers(2000, 10001, size=(S, 1))
    inc = rng.integers(0, 1501, size=(S, LAT_ENTRIES - 1))
    return np.concatenate([first, first + np.cumsum(inc, axis=1)], axis=1).astype(np.int32)


def poisson_arrivals(rng: np.random.Generator, n: int, mean_gap_us: float) -> np.ndarray:
    """Cumulative sum of floor(Exp(mean gap)) -> non-decreasing int64 arrival times."""
    gaps = np.floor(rng.exponential(mean_gap_us, size=n)).astype(np.int64)
    return np.cumsum(gaps)


def mmpp_arrivals(rng: np.random.Generator, n: int, base_rate: float, burst_mult: float,
                  calm_ms: float, burst_ms: float) -> np.ndarray:
    """Two-state Markov-modulated Poisson process, times in integer microseconds.

    Sojourns alternate calm/burst with exponential durations (means calm_ms,
    burst_ms); inside a sojourn arrivals are Poisson at base_rate (calm) or
    burst_mult*base_rate (burst).  Returns the first n arrival times, sorted.
    """
    out: List[np.ndarray] = []
    have = 0
    t = 0.0
    burst = False
    while have < n:
        dur_us = rng.exponential((burst_ms if burst else calm_ms) * 1000.0)
        rate = base_rate * (burst_mult if burst else 1.0)  # per second
        cnt = int(rng.poisson(rate * dur_us * 1e-6))
        if cnt:
            ts = np.sort(np.floor(t + rng.random(cnt) * dur_us)).astype(np.int64)
            out.append(ts)
            have += cnt
        t += dur_us
        burst = not burst
    return np.concatenate(out)[:n]


def count_paths(S: int, row_ptr: np.ndarray, col: np.ndarray) -> int:
    """Number of source-to-sink paths (used only to accept/reject random DAGs)."""
    indeg = np.zeros(S, dtype=np.int64)
    for c in col:
        indeg[c] += 1
    ways = np.zeros(S, dtype=np.int64)
    # stage ids of the random layered DAGs are already topologically ordered
    total = 0
    for s in range(S):
        if indeg[s] == 0:
            ways[s] = 1
        lo, hi = int(row_ptr[s]), int(row_ptr[s + 1])
        if lo == hi:
            total += int(ways[s])
        for e in range(lo, hi):
            ways[int(col[e])] += ways[s]
    return total


def count_paths_any_order(S: int, row_ptr: np.ndarray, col: np.ndarray) -> int:
    """Source-to-sink path count of a DAG whose stage ids are in arbitrary order."""
    indeg = np.zeros(S, dtype=np.int64)
    for c in col:
        indeg[c] += 1
    ways = np.where(indeg == 0, 1, 0).astype(object)
    left = indeg.copy()
    ready = [s for s in range(S) if left[s] == 0]
    total = 0
    while ready:
        s = ready.pop()
        lo, hi = int(row_ptr[s]), int(row_ptr[s + 1])
        if lo == hi:
            total += int(ways[s])
        for e in range(lo, hi):
            t = int(col[e])
            ways[t] += ways[s]
            left[t] -= 1
            if left[t] == 0:
                ready.append(t)
    return total


def random_layered_dag(rng: np.random.Generator, S: int, min_paths: int, max_paths: int):
    """Random layered DAG on S stages whose path count lies in [min_paths, max_paths]."""
    while True:
        L = int(rng.integers(3, min(S, 5) + 1)) if S >= 3 else S
        # split S nodes into L non-empty consecutive layers
        cuts = np.sort(rng.choice(np.arange(1, S), size=L - 1, replace=False)) if L > 1 else np.array([], dtype=int)
        bounds = np.concatenate([[0], cuts, [S]]).astype(int)
        layers = [list(range(bounds[i], bounds[i + 1])) for i in range(L)]
        edges = set()
        for li in range(L - 1):
            cur, nxt = layers[li], layers[li + 1]
            for v in nxt:                      # every node has a predecessor in the layer above
                edges.add((int(rng.choice(cur)), v))
            for u in cur:                      # every node has a successor in the layer below
                if not any(e[0] == u for e in edges):
                    edges.add((u, int(rng.choice(nxt))))
            for u in cur:                      # a few extra edges
                for v in nxt:
                    if rng.random() < 0.25:
                        edges.add((u, v))
        if L >= 3 and rng.random() < 0.3:      # occasional layer-skipping edge
            li = int(rng.integers(0, L - 2))
            edges.add((int(rng.choice(layers[li])), int(rng.choice(layers[li + 2]))))
        row_ptr, col = csr_from_edges(S, sorted(edges))
        p = count_paths(S, row_ptr, col)
        if min_paths <= p <= max_paths:
            return row_ptr, col, p


def _permute_within_snapshots(rng, snap_ptr, *arrays):
    out = [a.copy() for a in arrays]
    for u in range(len(snap_ptr) - 1):
        lo, hi = int(snap_ptr[u]), int(snap_ptr[u + 1])
        perm = rng.permutation(hi - lo)
        for a_out, a in zip(out, arrays):
            a_out[lo:hi] = a[lo:hi][perm]
    return out


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------

CONFIG_NAMES = {
    1: "cfg1-linear3-1k",
    2: "cfg2-linear5-1m",
    3: "cfg3-dag8-4paths-4m",
    4: "cfg4-bursty-dag12-16paths-16m",
    5: "cfg5-sweep-4096x8192",
}

FULL_N = {1: 1024, 2: 1 << 20, 3: 1 << 22, 4: 1 << 24, 5: 4096 * 8192}


def make_workload(cfg: int, n_requests: Optional[int] = None, n_snapshots: Optional[int] = None,
                  per_snapshot: Optional[int] = None, permute: bool = False,
                  seed: Optional[int] = None, order_mode: Optional[int] = None) -> Workload:
    """Build benchmark configuration `cfg` (1..5).

    n_requests / n_snapshots / per_snapshot shrink the workload for tests (the
    shape stays the same).  permute=True shuffles request order inside each
    snapshot (arrival-ordered input is nearly sorted by deadline; tests must
    not depend on that).  order_mode overrides the per-stage queue order.
    """
    if cfg not in CONFIG_NAMES:
        raise ValueError(f"unknown config {cfg}")
    notes = {}
    if cfg == 1:
        S, K = 3, 1
        n = 1024 if n_requests is None else int(n_requests)
        row_ptr, col = csr_from_edges(S, chain_edges(S))
        batch = np.full(S, 8, np.int32)
        workers = np.full(S, 2, np.int32)
        lat = affine_tables(_rng(cfg, 1, seed), S)
        arrival = _rng(cfg, 2, seed).integers(0, 100000, size=n).astype(np.int64)
        deadline = arrival + 200000
        stage = _rng(cfg, 3, seed).integers(0, S, size=n).astype(np.int32)
        now = np.array([100000], dtype=np.int64)
        mode = np.full(S, MODE_LBF, np.int32)
    elif cfg == 2:
        S, K = 5, 1
        n = (1 << 20) if n_requests is None else int(n_requests)
        row_ptr, col = csr_from_edges(S, chain_edges(S))
        batch = _rng(cfg, 4, seed).choice([4, 8, 16, 32], size=S).astype(np.int32)
        workers = _rng(cfg, 5, seed).integers(1, 9, size=S).astype(np.int32)
        lat = monotone_tables(_rng(cfg, 1, seed), S)
        arrival = poisson_arrivals(_rng(cfg, 2, seed), n, 20.0)
        deadline = arrival + 300000
        stage = _rng(cfg, 3, seed).integers(0, S, size=n).astype(np.int32)
        now = np.array([arrival.max() if n else 0], dtype=np.int64)
        mode = np.full(S, MODE_LBF, np.int32)
    elif cfg == 3:
        S, K = 8, 1
        n = (1 << 22) if n_requests is None else int(n_requests)
        edges = [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (3, 5), (4, 6), (5, 6), (6, 7)]
        row_ptr, col = csr_from_edges(S, edges)
        batch = _rng(cfg, 4, seed).choice([4, 8, 16, 32], size=S).astype(np.int32)
        workers = _rng(cfg, 5, seed).integers(1, 9, size=S).astype(np.int32)
        lat = monotone_tables(_rng(cfg, 1, seed), S)
        arrival = poisson_arrivals(_rng(cfg, 2, seed), n, 20.0)
        slo = _rng(cfg, 6, seed).choice([150000, 250000, 400000], size=n).astype(np.int64)
        deadline = arrival + slo
        stage = _rng(cfg, 3, seed).integers(0, S, size=n).astype(np.int32)
        now = np.array([arrival.max() if n else 0], dtype=np.int64)
        mode = np.full(S, MODE_LBF, np.int32)
    elif cfg == 4:
        S, K = 12, 1
        n = (1 << 24) if n_requests is None else int(n_requests)
        edges = [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (3, 5), (4, 6), (5, 6),
                 (6, 7), (6, 8), (7, 9), (8, 9), (9, 10), (9, 11)]
        row_ptr, col = csr_from_edges(S, edges)
        batch = _rng(cfg, 4, seed).choice([4, 8, 16, 32], size=S).astype(np.int32)
        workers = _rng(cfg, 5, seed).integers(1, 9, size=S).astype(np.int32)
        lat = monotone_tables(_rng(cfg, 1, seed), S)
        arrival = mmpp_arrivals(_rng(cfg, 2, seed), n, base_rate=200000.0, burst_mult=10.0,
                                calm_ms=950.0, burst_ms=50.0)
        deadline = arrival + 300000
        # skewed stage occupancy: Zipf(1.5) weights over a seeded permutation of the stages
        w = 1.0 / np.power(np.arange(1, S + 1, dtype=np.float64), 1.5)
        w /= w.sum()
        perm = _rng(cfg, 7, seed).permutation(S)
        p = np.empty(S)
        p[perm] = w
        stage = _rng(cfg, 3, seed).choice(S, size=n, p=p).astype(np.int32)
        now = np.array([arrival.max() if n else 0], dtype=np.int64)
        mode = np.full(S, MODE_HBF, np.int32)
        notes["stage_weights"] = p.tolist()
    else:  # cfg == 5
        S = 6
        K = 4096 if n_snapshots is None else int(n_snapshots)
        per = 8192 if per_snapshot is None else int(per_snapshot)
        if n_requests is not None:
            per = max(1, int(n_requests) // K)
        n = K * per
        drng = _rng(cfg, 8, seed)
        row_ptrs, cols, npaths = [], [], []
        for _ in range(K):
            rp, cl, p = random_layered_dag(drng, S, 2, 8)
            row_ptrs.append(rp)
            cols.append(cl)
            npaths.append(p)
        row_ptr = np.concatenate(row_ptrs).astype(np.int32)
        col = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
        batch = _rng(cfg, 4, seed).choice([4, 8, 16, 32], size=K * S).astype(np.int32)
        workers = _rng(cfg, 5, seed).integers(1, 17, size=K * S).astype(np.int32)
        lat = monotone_tables(_rng(cfg, 1, seed), K * S)
        rate = _rng(cfg, 9, seed).uniform(5000.0, 50000.0, size=K)
        gaps = np.floor(_rng(cfg, 2, seed).exponential(1.0, size=(K, per)) * (1e6 / rate)[:, None]).astype(np.int64)
        arr2 = np.cumsum(gaps, axis=1)
        slo = _rng(cfg, 6, seed).choice([150000, 250000, 400000], size=K).astype(np.int64)
        arrival = arr2.reshape(-1)
        deadline = (arr2 + slo[:, None]).reshape(-1)
        stage = _rng(cfg, 3, seed).integers(0, S, size=n).astype(np.int32)
        now = arr2.max(axis=1) if per else np.zeros(K, np.int64)
        mode = np.full(K * S, MODE_LBF, np.int32)
        notes["paths_per_snapshot"] = (int(min(npaths)), int(max(npaths))) if npaths else (0, 0)

    if cfg != 5:
        snap_ptr = np.array([0, n], dtype=np.int32)
        dag_shared = 1
    else:
        snap_ptr = (np.arange(K + 1, dtype=np.int64) * per).astype(np.int32)
        dag_shared = 0

    if order_mode is not None:
        mode = np.full_like(mode, order_mode)

    assert arrival.size == 0 or (deadline.max() < 2**31 and arrival.min() >= 0), "times must fit int32"
    arrival = arrival.astype(np.int32)
    deadline = deadline.astype(np.int32)
    if permute:
        arrival, deadline, stage = _permute_within_snapshots(_rng(cfg, 10, seed), snap_ptr,
                                                             arrival, deadline, stage)
    return Workload(
        name=CONFIG_NAMES[cfg] + ("" if n == FULL_N[cfg] else f"@n={n}") + ("-permuted" if permute else ""),
        K=K, S=S, dag_shared=dag_shared,
        dag_row_ptr=np.ascontiguousarray(row_ptr, np.int32), dag_col=np.ascontiguousarray(col, np.int32),
        batch=np.ascontiguousarray(batch, np.int32), workers=np.ascontiguousarray(workers, np.int32),
        lat_us=np.ascontiguousarray(lat.reshape(-1), np.int32), order_mode=np.ascontiguousarray(mode, np.int32),
        arrival=np.ascontiguousarray(arrival), deadline=np.ascontiguousarray(deadline),
        stage=np.ascontiguousarray(stage, np.int32), snap_ptr=snap_ptr, now=now.astype(np.int32), notes=notes)


def in_deadline_order(w: Workload) -> Workload:
    """The same snapshots with the requests of every snapshot arranged by rising deadline (what a queue
    snapshot taken in arrival order looks like when the pipeline has one SLO)."""
    idx = np.arange(w.n, dtype=np.int64)
    snap = np.repeat(np.arange(w.K, dtype=np.int64), np.diff(w.snap_ptr.astype(np.int64)))
    perm = np.lexsort((idx, w.deadline, snap))
    return dataclasses.replace(w, name=w.name + "-by-deadline", arrival=np.ascontiguousarray(w.arrival[perm]),
                               deadline=np.ascontiguousarray(w.deadline[perm]), stage=np.ascontiguousarray(w.stage[perm]))


def half_survivors(w: Workload) -> Workload:
    """A labelled variant of a single-snapshot workload (not one of the five configurations): the SLO is
    half the arrival span, `now` sits in the middle of it and the latency tables are scaled down by 200,
    so that roughly half of the queue is still in time and the drop mask is mixed.  The deep-overload
    snapshots of configurations 2-4 drop nearly everything; this one exercises estimates below the
    saturation value and a compaction that keeps a large part of every queue."""
    span = int(w.arrival.max()) if w.n else 0
    deadline = (w.arrival.astype(np.int64) + span // 2).astype(np.int32)
    return dataclasses.replace(w, name=w.name + "-half-survivors", deadline=deadline,
                               now=np.full_like(w.now, span // 2),
                               lat_us=np.maximum(1, w.lat_us // 200).astype(np.int32))


# --------------------------------------------------------------------------
# small random cases for brute-force pins and adversarial parity tests
# --------------------------------------------------------------------------

def with_snapshot_sizes(w: Workload, sizes) -> Workload:
    """The same plan with snapshot u cut down to its first sizes[u] requests (ragged batches)."""
    have = np.diff(w.snap_ptr.astype(np.int64))
    sizes = np.minimum(np.asarray(sizes, np.int64), have)
    keep = (np.concatenate([np.arange(w.snap_ptr[u], w.snap_ptr[u] + sizes[u]) for u in range(w.K)])
            if w.K else np.zeros(0, np.int64)).astype(np.int64)
    snap_ptr = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    return dataclasses.replace(w, name=w.name + "-ragged", arrival=np.ascontiguousarray(w.arrival[keep]),
                               deadline=np.ascontiguousarray(w.deadline[keep]),
                               stage=np.ascontiguousarray(w.stage[keep]), snap_ptr=snap_ptr)


def random_dag(rng: np.random.Generator, S: int, p_edge: float = 0.35):
    """Random DAG on S stages: edge a->b only for a<b under a random relabelling."""
    label = rng.permutation(S)
    edges = []
    for a in range(S):
        for b in range(a + 1, S):
            if rng.random() < p_edge:
                edges.append((int(label[a]), int(label[b])))
    rng.shuffle(edges)
    return csr_from_edges(S, edges)


def random_workload(seed: int, K: int = 1, S: int = 4, n_per_snapshot=16, dag_shared: Optional[int] = None,
                    time_span: int = 50000, slo_choices=(5000, 20000, 60000), tie_heavy: bool = False,
                    modes=(MODE_LBF, MODE_HBF, MODE_FCFS), max_batch: int = 64, max_workers: int = 16,
                    monotone: bool = True, vary_sizes: bool = True) -> Workload:
    """Small random plan + snapshots: random DAGs, all order modes, ragged snapshot sizes."""
    rng = np.random.default_rng([BASE_SEED, 777, seed])
    if dag_shared is None:
        dag_shared = int(rng.integers(0, 2)) if K > 1 else 1
    D = 1 if dag_shared else K
    rps, cls = [], []
    for _ in range(D):
        rp, cl = random_dag(rng, S, float(rng.uniform(0.15, 0.6)))
        rps.append(rp)
        cls.append(cl)
    batch = rng.integers(1, max_batch + 1, size=D * S).astype(np.int32)
    workers = rng.integers(1, max_workers + 1, size=D * S).astype(np.int32)
    if monotone:
        lat = monotone_tables(rng, D * S)
    else:
        lat = rng.integers(0, 20000, size=(D * S, LAT_ENTRIES)).astype(np.int32)
    mode = rng.choice(np.asarray(modes), size=D * S).astype(np.int32)
    if vary_sizes and K > 1:
        sizes = rng.integers(0, 2 * n_per_snapshot + 1, size=K)
    else:
        sizes = np.full(K, n_per_snapshot)
    snap_ptr = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    n = int(snap_ptr[-1])
    if tie_heavy:
        arrival = rng.integers(0, 8, size=n).astype(np.int64) * 1000
        slo = np.full(n, slo_choices[0], dtype=np.int64)
    else:
        arrival = rng.integers(0, max(1, time_span), size=n).astype(np.int64)
        slo = rng.choice(np.asarray(slo_choices), size=n).astype(np.int64)
    deadline = arrival + slo
    stage = rng.integers(0, S, size=n).astype(np.int32)
    now = rng.integers(0, max(1, time_span), size=K).astype(np.int32)
    return Workload(
        name=f"random-seed{seed}-K{K}-S{S}", K=K, S=S, dag_shared=int(dag_shared),
        dag_row_ptr=np.concatenate(rps).astype(np.int32),
        dag_col=(np.concatenate(cls) if cls else np.zeros(0)).astype(np.int32),
        batch=batch, workers=workers, lat_us=np.ascontiguousarray(lat.reshape(-1), np.int32),
        order_mode=mode, arrival=arrival.astype(np.int32), deadline=deadline.astype(np.int32),
        stage=stage, snap_ptr=snap_ptr, now=now)
