"""Pins of the oracle's adaptive priority (Section 3.3: load factor, thresholds 1 +- epsilon, delayed
transition).  Expected values: hand-worked series, closed forms, and an independent brute force
with exact rationals - never the C oracle itself."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

LBF, HBF = 0, 1


def one_stage(B, W, latB):
    lat = np.full(64, latB, np.int32)
    return np.array([B], np.int32), np.array([W], np.int32), lat


def brute(K, S, shared, batch, workers, lat, rate, window, prev):
    rate = np.asarray(rate).reshape(K * S, -1)
    out = []
    for g in range(K * S):
        rec = g % S if shared else g
        B, W, latB = int(batch[rec]), int(workers[rec]), int(lat[rec * 64 + int(batch[rec]) - 1])
        r = [int(x) for x in rate[g]]
        ts = [sum(r[max(0, t - window + 1):t + 1]) // (t - max(0, t - window + 1) + 1) for t in range(len(r))]
        total = sum(r)
        eps = Fraction(sum(abs(a - b) for a, b in zip(r, ts)), total) if total else Fraction(0)
        mode = LBF if prev is None else int(prev[g])
        for x in r:
            if latB == 0:
                mu = Fraction(0)
            else:
                mu = Fraction(x) / Fraction(W * B * 1_000_000, latB)
            if mu > 1 + eps:
                mode = HBF
            elif mu < 1 - eps:
                mode = LBF
        out.append(mode)
    return np.array(out, np.int32)


def test_hand_worked_series(oracle_mod):
    """B = 4, W = 2, lat[B] = 8000 us: T_m = 2 * 4 / 8 ms = 1000 requests/s.
    Series 1000 x 6 then one sample: window 3.
      ..., 1300: T_s = floor(3300/3) = 1100, dev = 200, sum = 7300, eps = 200/7300 = 0.0274;
            mu = 1.3 > 1.0274 -> HBF
      ..., 1020: T_s = 1006, dev = 14, eps = 14/7020 = 0.0020; mu = 1.02 > 1.002 -> HBF
      ..., 1001: T_s = 1000, dev = 1, eps = 1/7001; mu = 1.001 > 1.00014 -> HBF
      ..., 1000 only: eps = 0, mu = 1: neither -> keeps the previous priority
      ..., 700: T_s = 900, dev = 200, eps = 200/6700 = 0.0299; mu = 0.7 < 0.9701 -> LBF"""
    B, W, lat = one_stage(4, 2, 8000)
    for last, prev, want in ((1300, LBF, HBF), (1020, LBF, HBF), (1001, LBF, HBF), (1000, LBF, LBF), (1000, HBF, HBF),
                             (700, HBF, LBF)):
        rate = np.array([1000] * 6 + [last], np.int32)
        got = oracle_mod.priority_modes(1, 1, 1, B, W, lat, rate, 3, np.array([prev], np.int32))
        assert got[0] == want, (last, prev)


def test_delayed_transition_holds_inside_the_band(oracle_mod):
    """A burst switches to HBF; afterwards the load returns to just under capacity, inside
    [1 - eps, 1 + eps], and the priority stays HBF; without the burst it would have stayed LBF."""
    B, W, lat = one_stage(1, 1, 1000)                         # T_m = 1000 requests/s
    calm = [990] * 20
    burst = [990] * 5 + [3000] * 3 + [990] * 12
    assert oracle_mod.priority_modes(1, 1, 1, B, W, lat, np.array(calm, np.int32), 4)[0] == LBF
    assert oracle_mod.priority_modes(1, 1, 1, B, W, lat, np.array(burst, np.int32), 4)[0] == HBF
    # far below capacity at the end: back to LBF
    assert oracle_mod.priority_modes(1, 1, 1, B, W, lat, np.array(burst + [100], np.int32), 4)[0] == LBF


def test_constant_load_closed_form(oracle_mod):
    """A constant series has eps = 0: HBF iff rate > T_m, LBF iff rate < T_m, unchanged at equality."""
    for B, W, latB, tm in ((8, 2, 4000, 4000), (1, 3, 1500, 2000), (64, 1, 64000, 1000)):
        b, w, lat = one_stage(B, W, latB)
        for rate, prev, want in ((tm + 1, LBF, HBF), (tm - 1, HBF, LBF), (tm, LBF, LBF), (tm, HBF, HBF), (0, HBF, LBF)):
            got = oracle_mod.priority_modes(1, 1, 1, b, w, lat, np.full(9, rate, np.int32), 5, np.array([prev], np.int32))
            assert got[0] == want, (B, W, latB, rate, prev)


@pytest.mark.parametrize("seed", range(12))
def test_brute_force(oracle_mod, seed):
    rng = np.random.default_rng(4000 + seed)
    K, S, shared = 1 + seed % 4, 1 + seed % 5, seed % 2
    w = wl.random_workload(800 + seed, K=K, S=S, n_per_snapshot=5, dag_shared=shared)
    lat = w.lat_us.copy()
    if seed % 3 == 0:
        lat[::64] = 0
    T = int(rng.integers(1, 60))
    window = int(rng.integers(1, 12))
    cap = (w.workers.astype(np.int64) * w.batch * 1_000_000 // np.maximum(1, lat.reshape(-1, 64)[np.arange(w.batch.size), w.batch - 1]))
    base = np.repeat(cap[np.arange(K * S) % S if shared else np.arange(K * S)], T).reshape(K * S, T)
    rate = np.clip(base * rng.uniform(0.5, 1.6, (K * S, T)), 0, 2**31 - 1).astype(np.int32)
    rate[rng.random((K * S, T)) < 0.1] = 0
    prev = rng.integers(0, 2, K * S).astype(np.int32) if seed % 2 else None
    got = oracle_mod.priority_modes(K, S, shared, w.batch, w.workers, lat, rate, window, prev)
    assert np.array_equal(got, brute(K, S, shared, w.batch, w.workers, lat, rate, window, prev))


def test_extremes_and_bad_arguments(oracle_mod):
    B, W, lat = one_stage(64, 1 << 20, 2**31 - 1)
    rate = np.full(2048, 2**31 - 1, np.int32)
    assert oracle_mod.priority_modes(1, 1, 1, B, W, lat, rate, 7)[0] == brute(1, 1, 1, B, W, lat, rate, 7, None)[0]
    with pytest.raises(ValueError):
        oracle_mod.priority_modes(1, 1, 1, B, W, lat, rate, 0)
