"""CPU-only checks of the GPU library: it loads, exports the declared symbols, and its
host-side logic (validation, DAG -> path expansion, invariant-divisor constants) is right.
No kernel is launched here."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

from paper_2602_08747_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pard.h")).read()
    declared = set(re.findall(r"\b(pard_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = binding.load_library()
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.pard_strerror(0) == b"ok" and b"workspace" in lib.pard_strerror(-8)


def _check(w, **over):
    a = dict(K=w.K, S=w.S, dag_shared=w.dag_shared, dag_row_ptr=w.dag_row_ptr, dag_col=w.dag_col, batch=w.batch,
             workers=w.workers, lat_us=w.lat_us, order_mode=w.order_mode)
    a.update(over)
    return binding.pard_plan_check(**a)


def test_plan_check_counts_paths(oracle_mod):
    for cfg, paths, longest in ((1, 1, 3), (2, 1, 5), (3, 4, 6), (4, 16, 8)):
        w = wl.make_workload(cfg, n_requests=4)
        assert _check(w) == (0, paths, longest)
    w = wl.make_workload(5, n_snapshots=40, per_snapshot=2)
    rc, total, longest = _check(w)
    want = 0
    col_base = 0
    for u in range(w.K):
        rp = w.dag_row_ptr[u * 7:(u + 1) * 7]
        want += wl.count_paths_any_order(6, rp, w.dag_col[col_base:col_base + rp[6]])
        col_base += rp[6]
    assert rc == 0 and total == want
    for seed in range(30):      # agrees with the oracle's independent enumeration on random DAGs
        rng = np.random.default_rng(seed)
        S = int(rng.integers(1, 10))
        rp, cl = wl.random_dag(rng, S, 0.4)
        ptr, stg = oracle_mod.expand_paths(S, rp, cl)
        one = np.ones(S, np.int32)
        rc, total, longest = binding.pard_plan_check(1, S, 1, rp, cl, one, one, np.ones(S * 64, np.int32), one * 0)
        assert (rc, total, longest) == (0, len(ptr) - 1, int(np.diff(ptr).max()))


def test_plan_check_error_codes():
    w = wl.make_workload(3, n_requests=4)
    assert _check(w, K=0)[0] == -2
    assert _check(w, S=65)[0] == -2
    b = w.batch.copy(); b[2] = 0
    assert _check(w, batch=b)[0] == -3
    b[2] = 65
    assert _check(w, batch=b)[0] == -3
    x = w.workers.copy(); x[0] = 0
    assert _check(w, workers=x)[0] == -4
    x[0] = (1 << 20) + 1
    assert _check(w, workers=x)[0] == -4
    l = w.lat_us.copy(); l[100] = -1
    assert _check(w, lat_us=l)[0] == -5
    m = w.order_mode.copy(); m[1] = 3
    assert _check(w, order_mode=m)[0] == -10
    c = w.dag_col.copy(); c[0] = 8
    assert _check(w, dag_col=c)[0] == -6                      # edge out of range
    c = w.dag_col.copy(); c[0] = 0
    assert _check(w, dag_col=c)[0] == -6                      # self loop
    rp, cl = wl.csr_from_edges(3, [(0, 1), (1, 2), (2, 0)])
    one = np.ones(3, np.int32)
    assert binding.pard_plan_check(1, 3, 1, rp, cl, one, one, np.ones(192, np.int32), one * 0)[0] == -6   # cycle
    rp, cl = wl.csr_from_edges(3, [(1, 2), (2, 1)])
    assert binding.pard_plan_check(1, 3, 1, rp, cl, one, one, np.ones(192, np.int32), one * 0)[0] == -6   # unreachable cycle
    rp2 = rp.copy(); rp2[1] = 5
    assert binding.pard_plan_check(1, 3, 1, rp2, cl, one, one, np.ones(192, np.int32), one * 0)[0] == -6  # offsets not monotone
    # exponential DAG: 12 diamonds in series = 4096 paths > limit
    S, edges = 37, []
    for d in range(12):
        a = 3 * d
        edges += [(a, a + 1), (a, a + 2), (a + 1, a + 3), (a + 2, a + 3)]
    rp, cl = wl.csr_from_edges(S, edges)
    one = np.ones(S, np.int32)
    assert binding.pard_plan_check(1, S, 1, rp, cl, one, one, np.ones(S * 64, np.int32), one * 0)[0] == -7
    lib = binding.load_library()
    assert lib.pard_plan_check(None, None, None) == -1
    assert lib.pard_plan_destroy(None) == 0


@pytest.fixture(scope="module")
def host_shim(tmp_path_factory):
    """The library's host-only header compiled on its own with g++ (no HIP)."""
    d = tmp_path_factory.mktemp("shim")
    src = d / "shim.cpp"
    src.write_text('#include "paper_2602_08747_amd/csrc/pard_host.hpp"\n'
                   'extern "C" unsigned shim_div(unsigned n, unsigned d) {\n'
                   '  return pard::magic_div(n, pard::magic_u32(d)); }\n'
                   'extern "C" long shim_sweep(unsigned d, unsigned lo, unsigned count) {\n'
                   '  pard::Magic32 k = pard::magic_u32(d); long bad = 0;\n'
                   '  for (unsigned i = 0; i < count; ++i) { unsigned n = lo + i; bad += pard::magic_div(n, k) != n / d; }\n'
                   '  return bad; }\n')
    so = d / "shim.so"
    subprocess.run(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-I", ROOT, str(src), "-o", str(so)], check=True)
    lib = ctypes.CDLL(str(so))
    lib.shim_div.restype = ctypes.c_uint32
    lib.shim_div.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
    lib.shim_sweep.restype = ctypes.c_long
    lib.shim_sweep.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
    return lib


def test_invariant_division_is_exact(host_shim):
    """floor(n/d) through the multiply-high constants equals n/d: every batch size, worker
    counts up to the limit, numerators at both ends of the 32-bit range and around multiples."""
    rng = np.random.default_rng(0)
    divisors = list(range(1, 130)) + [255, 256, 257, 1000, 4095, 4096, 65535, 65536, 65537, (1 << 20) - 1, 1 << 20] \
        + rng.integers(1, 1 << 20, size=200).tolist()
    for d in divisors:
        assert host_shim.shim_sweep(d, 0, 70000) == 0
        assert host_shim.shim_sweep(d, 2**32 - 70000, 70000) == 0
        assert host_shim.shim_sweep(d, 2**31 - 35000, 70000) == 0
        for q in rng.integers(0, 2**32 // d, size=50).tolist():
            base = q * d
            for n in (base - 1, base, base + 1, base + d - 1):
                if 0 <= n < 2**32:
                    assert host_shim.shim_div(n, d) == n // d


def test_short_queue_float_reciprocals_are_exact():
    """The on-chip kernel forms ceil(a/B) and floor(p/W) for short queues with one float32
    multiply each: trunc((x + 0.5) * fl(1/d)).  Replayed here in IEEE float32 (numpy) over the
    whole domain the kernel uses it on: x = a + B - 1 < 2^13 + 64 for every B, and
    p = q * (latB mod W) < 2^21 for every W <= 256."""
    f32 = np.float32
    for B in range(1, 65):
        x = np.arange(0, 8192 + B, dtype=np.int64)
        got = ((x.astype(f32) + f32(0.5)) * (f32(1.0) / f32(B))).astype(np.int64)
        assert np.array_equal(got, x // B), B
    for W in range(1, 257):
        p = np.arange(0, 8192 * (W - 1) + 1, dtype=np.int64) if W > 1 else np.zeros(1, np.int64)
        assert p.max() < 2**21
        got = ((p.astype(f32) + f32(0.5)) * (f32(1.0) / f32(W))).astype(np.int64)
        assert np.array_equal(got, p // W), W


def test_stale_library_is_detected(tmp_path, monkeypatch):
    """The digest written beside the library at build time covers every source, header and flag: a tree whose
    sources differ from the ones the library was built from is reported stale whatever the file times say."""
    from paper_2602_08747_amd import build
    binding.load_library()                       # builds when needed
    assert not build.is_stale()
    assert set(os.path.basename(d) for d in build.dependencies()) >= {"pard_api.hip", "pard_device.hpp", "pard.h"}
    recorded = open(build.HASH_PATH).read().strip()
    assert recorded == build.source_hash()
    fake = tmp_path / "libpard.srchash"
    fake.write_text("0" * 64 + "\n")
    monkeypatch.setattr(build, "HASH_PATH", str(fake))
    assert build.is_stale()
    monkeypatch.setattr(build, "HASH_PATH", str(tmp_path / "missing"))
    assert build.is_stale()


SANITIZE = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]
SAN_ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1")
SAN_ENV.pop("LD_PRELOAD", None)


def _run_sanitized(exe):
    res = subprocess.run([str(exe)], env=SAN_ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-3000:]
    assert "ERROR: AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout, res.stdout[-3000:]
    return res.stdout


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    """The oracle's C source built with AddressSanitizer and UndefinedBehaviorSanitizer and driven through every entry
    point on small random pipelines (including out-of-range stages, empty snapshots and extreme times)."""
    driver = tmp_path / "driver.c"
    driver.write_text(r'''
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
int pard_oracle_estimate_drop(int32_t, int32_t, int32_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*,
    const int32_t*, int64_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int32_t*, uint8_t*, int32_t*,
    int32_t*, int32_t);
int pard_oracle_estimate_drop_consistent(int32_t, int32_t, int32_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*,
    const int32_t*, const int32_t*, int64_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int64_t*,
    int32_t*, uint8_t*, int32_t*, int32_t*, int32_t);
int pard_oracle_estimate_drop_ranked(int32_t, int32_t, int32_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*,
    const int32_t*, int64_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int32_t*, uint8_t*, int32_t*,
    int32_t*, int32_t);
int pard_oracle_compact(int32_t, int32_t, int64_t, const int32_t*, const int32_t*, const uint8_t*, int32_t*, int32_t*);
int pard_oracle_nexus_drop(int32_t, int32_t, int32_t, const int32_t*, const int32_t*, int64_t, const int32_t*, const int32_t*, const int32_t*,
    const int32_t*, uint8_t*, int32_t*);
int pard_oracle_clipper_drop(int32_t, int32_t, int32_t, const int32_t*, const int32_t*, const int32_t*, const int32_t*, int64_t,
    const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*, uint8_t*);
static uint64_t state = 88172645463325252ull;
static uint32_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (uint32_t)(state >> 16); }
int main(void) {
    for (int round = 0; round < 40; ++round) {
        const int K = 1 + rnd() % 4, S = 1 + rnd() % 6;
        /* a diamond-ish DAG: stage s -> s+1 and sometimes s -> s+2 */
        int32_t* rp = calloc((size_t)K * (S + 1), 4); int32_t* col = calloc((size_t)K * 2 * S + 1, 4);
        int32_t* B = malloc((size_t)K * S * 4); int32_t* W = malloc((size_t)K * S * 4); int32_t* M = malloc((size_t)K * S * 4);
        int32_t* L = malloc((size_t)K * S * 64 * 4);
        int nc = 0;
        for (int u = 0; u < K; ++u) {
            int local = 0;
            for (int s = 0; s < S; ++s) {
                rp[u * (S + 1) + s] = local;
                if (s + 1 < S) { col[nc++] = s + 1; ++local; }
                if (s + 2 < S && rnd() % 2) { col[nc++] = s + 2; ++local; }
            }
            rp[u * (S + 1) + S] = local;
        }
        for (int i = 0; i < K * S; ++i) {
            B[i] = 1 + rnd() % 64; W[i] = 1 + rnd() % 9; M[i] = rnd() % 3;
            for (int b = 0; b < 64; ++b) L[i * 64 + b] = round % 5 == 4 ? 2147483647 : (int32_t)(rnd() % 20000);
        }
        int32_t* sp = malloc((size_t)(K + 1) * 4); sp[0] = 0;
        for (int u = 0; u < K; ++u) sp[u + 1] = sp[u] + (rnd() % 3 == 0 ? 0 : (int32_t)(rnd() % 300));
        const int64_t n = sp[K];
        int32_t* arr = malloc((size_t)(n + 1) * 4); int32_t* dl = malloc((size_t)(n + 1) * 4); int32_t* st = malloc((size_t)(n + 1) * 4);
        int32_t* now = malloc((size_t)K * 4);
        for (int64_t r = 0; r < n; ++r) {
            arr[r] = (int32_t)(rnd() % 100000) - 500; dl[r] = rnd() % 7 == 0 ? 2147483647 : arr[r] + (int32_t)(rnd() % 90000);
            st[r] = (int32_t)(rnd() % (S + 2)) - 1;
        }
        for (int u = 0; u < K; ++u) now[u] = round % 7 == 6 ? -2147483647 - 1 : (int32_t)(rnd() % 120000);
        int32_t* est = malloc((size_t)(n + 1) * 4); uint8_t* drop = malloc((size_t)n + 1); int32_t* order = malloc((size_t)(n + 1) * 4);
        int32_t* seg = malloc((size_t)(K * S + 1) * 4); int32_t* surv = malloc((size_t)(n + 1) * 4); int32_t* sptr = malloc((size_t)(K * S + 1) * 4);
        int32_t* first = malloc((size_t)K * S * 4);
        if (pard_oracle_estimate_drop(K, S, 0, rp, col, B, W, L, M, n, arr, dl, st, sp, now, est, drop, order, seg, 2)) return 2;
        if (pard_oracle_compact(K, S, n, order, seg, drop, surv, sptr)) return 3;
        if (pard_oracle_estimate_drop_consistent(K, S, 0, rp, col, B, W, L, M, n, arr, dl, st, sp, now, NULL, est, drop, order, seg, 1)) return 4;
        if (pard_oracle_estimate_drop_ranked(K, S, 0, rp, col, B, W, L, M, n, arr, dl, st, sp, now, est, drop, order, seg, 1)) return 5;
        if (pard_oracle_nexus_drop(K, S, 0, B, L, n, dl, order, seg, now, drop, first)) return 6;
        if (pard_oracle_clipper_drop(K, S, 0, rp, col, B, L, n, arr, dl, st, sp, now, drop)) return 7;
        free(rp); free(col); free(B); free(W); free(M); free(L); free(sp); free(arr); free(dl); free(st); free(now); free(est); free(drop);
        free(order); free(seg); free(surv); free(sptr); free(first);
    }
    puts("oracle driver done");
    return 0;
}
''')
    exe = tmp_path / "oracle_san"
    subprocess.run(["gcc", "-std=gnu99", *SANITIZE, "-fopenmp", os.path.join(ROOT, "oracle", "pard_oracle.c"), str(driver), "-o", str(exe)],
                   check=True)
    assert "oracle driver done" in _run_sanitized(exe)


def test_host_plan_builder_under_address_and_undefined_sanitizers(tmp_path):
    """The library's host-side plan builder (validation, path expansion, constants) built on its own with the sanitizers and
    fed valid, malformed and exploding pipeline descriptions."""
    driver = tmp_path / "driver.cpp"
    driver.write_text(r'''
#include <cstdio>
#include <vector>
#include "paper_2602_08747_amd/csrc/pard_host.hpp"
static unsigned long long state = 88172645463325252ull;
static unsigned rnd() { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (unsigned)(state >> 16); }
int main() {
    int ok = 0, rejected = 0;
    for (int round = 0; round < 400; ++round) {
        const int K = 1 + rnd() % 3, S = 1 + rnd() % 12, shared = rnd() % 2, D = shared ? 1 : K;
        std::vector<int32_t> rp, col, B(D * S), W(D * S), M(D * S), L((size_t)D * S * 64);
        for (int d = 0; d < D; ++d) {
            int local = 0;
            for (int s = 0; s < S; ++s) {
                rp.push_back(local);
                for (int t = s + 1; t < S; ++t)
                    if (rnd() % 3 == 0) { col.push_back(round % 11 == 10 && rnd() % 9 == 0 ? (int)(rnd() % (S + 2)) - 1 : t); ++local; }
            }
            rp.push_back(local);
        }
        for (int i = 0; i < D * S; ++i) {
            B[i] = round % 13 == 12 ? (int)(rnd() % 70) : 1 + rnd() % 64;
            W[i] = round % 17 == 16 ? (int)(rnd() % 3) : 1 + rnd() % 300;
            M[i] = round % 19 == 18 ? (int)(rnd() % 5) : rnd() % 3;
            for (int b = 0; b < 64; ++b) L[(size_t)i * 64 + b] = round % 23 == 22 ? -(int)(rnd() % 3) : (int)(rnd() % 2000000);
        }
        pard_plan_desc_t d{K, S, shared, rp.data(), col.empty() ? nullptr : col.data(), B.data(), W.data(), L.data(), M.data()};
        pard::HostPlan hp;
        const int rc = pard::build_host_plan(&d, hp);
        if (rc == PARD_OK) {
            ++ok;
            if (hp.split_in.size() != (size_t)D * S || hp.entry_end.size() != hp.entry_stage.size()) return 2;
        } else {
            ++rejected;
        }
    }
    // twelve diamonds in series: 4096 paths, refused
    {
        const int S = 37;
        std::vector<int32_t> rp(S + 1, 0), col, one(S, 1), zero(S, 0), L((size_t)S * 64, 5);
        for (int s = 0; s < S; ++s) {
            rp[s] = (int32_t)col.size();
            if (s % 3 == 0 && s + 3 < S) { col.push_back(s + 1); col.push_back(s + 2); }
            else if (s % 3 == 1 && s + 2 < S) col.push_back(s + 2);
            else if (s % 3 == 2 && s + 1 < S) col.push_back(s + 1);
        }
        rp[S] = (int32_t)col.size();
        pard_plan_desc_t d{1, S, 1, rp.data(), col.data(), one.data(), one.data(), L.data(), zero.data()};
        pard::HostPlan hp;
        if (pard::build_host_plan(&d, hp) != PARD_E_TOO_MANY_PATHS) return 3;
    }
    std::printf("host driver done: %d accepted, %d rejected\n", ok, rejected);
    return ok > 50 && rejected > 20 ? 0 : 4;
}
''')
    exe = tmp_path / "host_san"
    subprocess.run(["g++", "-std=c++17", *SANITIZE, "-I", ROOT, str(driver), "-o", str(exe)], check=True)
    assert "host driver done" in _run_sanitized(exe)
