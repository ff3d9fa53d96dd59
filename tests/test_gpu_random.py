"""Randomised differential test: many small random plans and snapshots through every variant of the
estimate (plain, given downstream latency, sequentially consistent, ranked) on both kernel paths, C-ABI vs the
CPU oracle, bit for bit."""
import numpy as np
import pytest

from paper_2602_08747_amd import workloads as wl

pytestmark = pytest.mark.gpu

FORCE_SORT = 1 << 20
KEYS = ("est", "drop", "order", "seg_ptr", "surv_idx", "surv_ptr")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libpard.so")
    from paper_2602_08747_amd import binding
    binding.load_library()
    return binding


def draw_case(seed):
    rng = np.random.default_rng([4711, seed])
    K = int(rng.integers(1, 10))
    S = int(rng.integers(1, 17))
    per = int(rng.choice([0, 1, 7, 64, 300, 1500, 4000, 9000]))
    modes = [(wl.MODE_LBF,), (wl.MODE_HBF,), (wl.MODE_LBF, wl.MODE_HBF), (wl.MODE_LBF, wl.MODE_HBF, wl.MODE_FCFS)][int(rng.integers(0, 4))]
    w = wl.random_workload(9000 + seed, K=K, S=S, n_per_snapshot=per, monotone=bool(rng.integers(0, 2)),
                           tie_heavy=bool(rng.integers(0, 4) == 0), modes=modes,
                           time_span=int(rng.choice([1, 1000, 50_000, 5_000_000])),
                           slo_choices=tuple(int(x) for x in rng.choice([0, 2000, 30_000, 400_000, 9_000_000], size=3)),
                           max_batch=int(rng.choice([1, 4, 64])), max_workers=int(rng.choice([1, 16, 1 << 20])))
    if rng.integers(0, 3) == 0 and w.n:
        w.deadline[rng.integers(0, w.n, size=max(1, w.n // 10))] = 2**31 - 1
    if rng.integers(0, 3) == 0 and w.n:
        w.stage[rng.integers(0, w.n, size=max(1, w.n // 20))] = rng.integers(-5, S + 5)
    sub = None
    if rng.integers(0, 2):
        sub = rng.choice([0, 1, 5000, 90_000, 1 << 33, 1 << 45], size=K * S).astype(np.int64)
    return w, sub


@pytest.mark.parametrize("seed", range(64))
def test_random_case(gpu, oracle_mod, seed):
    import torch
    w, sub = draw_case(seed)
    print("case", seed, w.name, "n", w.n, "K", w.K, "S", w.S, "sub", sub is not None, flush=True)
    for variant in ("plain", "consistent", "ranked"):
        if variant == "ranked" and sub is not None:
            continue                                   # the ranked variant computes the downstream part itself
        consistent, ranked = variant == "consistent", variant == "ranked"
        ref = oracle_mod.run(w, threads=8, sub=sub, consistent=consistent, ranked=ranked)
        # the tight promise picks the one-wave kernel for snapshots of at most 128: those also run under a
        # promise of 256 and of 512 (the smallest workgroup kernels)
        promises = (None, FORCE_SORT) + ((256, 512) if w.max_snapshot_requests <= 128 else ())
        for max_snap in promises:
            s = gpu.Session(w, max_snapshot_requests=None if max_snap is None else max(max_snap, w.max_snapshot_requests))
            s.run(sub=None if sub is None else torch.from_numpy(sub).to(s.dev), consistent=consistent, ranked=ranked)
            got = s.results()
            for k in KEYS:
                assert np.array_equal(got[k], ref[k]), (seed, variant, max_snap, k, np.flatnonzero(got[k] != ref[k])[:5])
            assert s.status_word() == 0


@pytest.mark.parametrize("seed", range(64))
def test_random_case_in_deadline_order(gpu, oracle_mod, seed):
    """The same random cases with every snapshot arranged by rising deadline: snapshots that arrive in queue order take
    the kernels without a sort (on chip and, under the forced promise, the split of the large-snapshot path) whenever
    the plan qualifies, and the general kernels otherwise; plain estimate with and without a given downstream latency."""
    import torch
    w, sub = draw_case(seed)
    w = wl.in_deadline_order(w)
    print("case", seed, w.name, "n", w.n, "K", w.K, "S", w.S, "sub", sub is not None, flush=True)
    ref = oracle_mod.run(w, threads=8, sub=sub)
    for max_snap in (None, FORCE_SORT):
        s = gpu.Session(w, max_snapshot_requests=None if max_snap is None else max(max_snap, w.max_snapshot_requests))
        s.run(sub=None if sub is None else torch.from_numpy(sub).to(s.dev))
        got = s.results()
        for k in KEYS:
            assert np.array_equal(got[k], ref[k]), (seed, max_snap, k, np.flatnonzero(got[k] != ref[k])[:5])
        assert s.status_word() == 0
        if sub is None:
            s.run_one_call()
            again = s.results()
            for k in KEYS:
                assert np.array_equal(again[k], ref[k]), (seed, max_snap, "one call", k)
