"""Pins of the oracle's monitored queueing delay (Section 3.2, State Planner: q_i from a sliding
window over the recent delays, linearly weighted) and of its use in the downstream latency.
Expected values: hand-worked windows, the closed form of a linearly weighted mean over equally
spaced samples, and an independent brute force with exact rationals - never the C oracle itself."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl


def brute(K, S, time, delay, now, window):
    time = np.asarray(time).reshape(K * S, -1)
    delay = np.asarray(delay).reshape(K * S, -1)
    out = []
    for g in range(K * S):
        num, den = Fraction(0), Fraction(0)
        for t, x in zip(time[g], delay[g]):
            age = int(now[g // S]) - int(t)
            if 0 <= age < window:
                num += (window - age) * max(int(x), 0)
                den += window - age
        out.append(int(num / den // 1) if den else 0)
    return np.array(out, np.int32)


def test_hand_worked_windows(oracle_mod):
    """now = 10, window = 10: a sample aged 5 weighs 5, one aged 1 weighs 9:
    (5*100 + 9*200) / 14 = 164.28 -> 164.  The newest sample dominates."""
    q = oracle_mod.queue_delay(1, 1, [[5, 9]], [[100, 200]], [10], 10)
    assert q[0] == 164
    # age 0 weighs the whole window, age window-1 weighs 1, age window weighs nothing
    q = oracle_mod.queue_delay(1, 1, [[10, 1, 0]], [[0, 1100, 10 ** 9]], [10], 10)
    assert q[0] == (10 * 0 + 1 * 1100) // 11 == 100
    # a sample later than now is not part of the window; negative delays read as 0
    q = oracle_mod.queue_delay(1, 1, [[11, 8]], [[10 ** 9, 700]], [10], 10)
    assert q[0] == 700
    q = oracle_mod.queue_delay(1, 1, [[9, 8]], [[-50, 900]], [10], 10)
    assert q[0] == (9 * 0 + 8 * 900) // 17
    # nothing inside the window, or no samples at all: 0
    assert oracle_mod.queue_delay(1, 1, [[0, -5]], [[5, 5]], [10], 10)[0] == 0
    assert oracle_mod.queue_delay(1, 2, np.zeros((2, 0), np.int32), np.zeros((2, 0), np.int32), [10], 10).tolist() == [0, 0]


def test_constant_delay_is_its_own_mean(oracle_mod):
    rng = np.random.default_rng(5)
    time = rng.integers(0, 5_000_000, size=(6, 200))
    delay = np.full((6, 200), 12345)
    q = oracle_mod.queue_delay(2, 3, time, delay, [5_000_000, 4_000_000], 5_000_000)
    assert (q == 12345).all()


def test_equally_spaced_linear_trend_closed_form(oracle_mod):
    """N samples one step apart, the newest at now, window = N steps: weights N, N-1, ..., 1 (the
    textbook linearly weighted moving average).  For delay = a + b * j (j = age in steps):
    mean = a + b * sum (N - j) j / sum (N - j) = a + b * (N - 1) / 3."""
    for N, step, a, b in ((4, 1000, 500, 30), (10, 250, 7000, 9), (100, 50_000, 20, 3), (7, 1, 0, 300)):
        now = 3_000_000
        ages = np.arange(N) * step
        q = oracle_mod.queue_delay(1, 1, [now - ages], [a + b * np.arange(N)], [now], N * step)
        assert q[0] == (3 * a + b * (N - 1)) // 3, (N, step, a, b)


def test_order_and_padding_do_not_matter(oracle_mod):
    rng = np.random.default_rng(11)
    K, S, L = 3, 2, 50
    now = rng.integers(1_000_000, 2_000_000, size=K)
    time = rng.integers(0, 2_000_000, size=(K * S, L))
    delay = rng.integers(0, 100_000, size=(K * S, L))
    base = oracle_mod.queue_delay(K, S, time, delay, now, 700_000)
    perm = rng.permutation(L)
    assert (oracle_mod.queue_delay(K, S, time[:, perm], delay[:, perm], now, 700_000) == base).all()
    # samples that lie outside every window (too old, or in the future) change nothing
    pad_t = np.concatenate([time, np.full((K * S, 5), 2**31 - 1), np.full((K * S, 5), -2**31)], axis=1)
    pad_d = np.concatenate([delay, np.full((K * S, 10), 77_777_777)], axis=1)
    assert (oracle_mod.queue_delay(K, S, pad_t, pad_d, now, 700_000) == base).all()


@pytest.mark.parametrize("seed", range(12))
def test_brute_force(oracle_mod, seed):
    rng = np.random.default_rng(1000 + seed)
    K, S = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    L = int(rng.integers(1, 40))
    window = int(rng.choice([1, 2, 7, 1000, 5_000_000, 2**31 - 1]))
    now = rng.integers(0, 2**31 - 1, size=K)
    span = min(window * 2, 2**31 - 1)
    time = (now.repeat(S)[:, None] - rng.integers(-span // 8 - 1, span, size=(K * S, L))).clip(-2**31, 2**31 - 1)
    delay = rng.integers(-1000, 2**31 - 1, size=(K * S, L))
    want = brute(K, S, time, delay, now, window)
    got = oracle_mod.queue_delay(K, S, time, delay, now, window)
    assert (got == want).all()


def test_extreme_values_do_not_overflow(oracle_mod):
    """Every sample at the largest delay and the largest weight: the mean is that delay."""
    L = 1000
    q = oracle_mod.queue_delay(1, 1, np.full((1, L), 2**31 - 1), np.full((1, L), 2**31 - 1), [2**31 - 1], 2**31 - 1)
    assert q[0] == 2**31 - 1


def test_monitored_delay_replaces_the_queue_term(oracle_mod):
    """Chain 0 -> 1 -> 2, monitored q = (q0, q1, q2): L_sub(0) = q1 + q2 + d1 + d2 + w with
    d_i = lat_i[min(B_i, n_i + 1)], whatever the queue lengths say about waiting."""
    S = 3
    rp, col = wl.csr_from_edges(S, wl.chain_edges(S))
    batch = np.array([4, 2, 8], np.int32)
    workers = np.array([1, 3, 2], np.int32)
    lat = np.zeros((S, 64), np.int32)
    for s in range(S):
        lat[s] = 1000 * (s + 1) + 10 * np.arange(1, 65)
    qlen = np.array([50, 0, 3], np.int32)              # d_1 = lat_1[1] = 2010, d_2 = lat_2[4] = 3040
    qd = np.array([999_999, 120, -7], np.int32)        # the negative one reads as 0
    d1, d2 = 2010, 3040
    lower = oracle_mod.sub_latency(1, S, 1, rp, col, batch, workers, lat.ravel(), qlen, variant=oracle_mod.VARIANT_LOWER, qdelay=qd)
    assert lower.tolist() == [120 + 0 + d1 + d2, 0 + d2, 0]
    upper = oracle_mod.sub_latency(1, S, 1, rp, col, batch, workers, lat.ravel(), qlen, variant=oracle_mod.VARIANT_UPPER, qdelay=qd)
    assert upper.tolist() == [120 + 2 * (d1 + d2), 2 * d2, 0]
    sf = oracle_mod.sub_latency(1, S, 1, rp, col, batch, workers, lat.ravel(), qlen, variant=oracle_mod.VARIANT_SF, qdelay=qd)
    assert sf.tolist() == [d1 + d2, d2, 0]
    # the sampled batch wait does not depend on where q comes from
    rng = np.random.default_rng(3)
    M = 200
    samples = rng.integers(0, 10**7, size=M).astype(np.int32)
    picks = rng.integers(0, 2**32, size=M * S, dtype=np.uint64).astype(np.uint32)
    full_q = oracle_mod.sub_latency(1, S, 1, rp, col, batch, workers, lat.ravel(), qlen, lam=(1, 10), samples=samples, picks=picks, qdelay=qd)
    full_n = oracle_mod.sub_latency(1, S, 1, rp, col, batch, workers, lat.ravel(), qlen, lam=(1, 10), samples=samples, picks=picks)
    lower_n = oracle_mod.sub_latency(1, S, 1, rp, col, batch, workers, lat.ravel(), qlen, variant=oracle_mod.VARIANT_LOWER)
    assert ((full_q - lower) == (full_n - lower_n)).all()
