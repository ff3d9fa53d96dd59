"""ctypes binding of oracle/pard_oracle.c (TEST INFRASTRUCTURE, CPU only).

`build_oracle()` compiles the C file with gcc into oracle/libpard_oracle.so; the
other functions marshal numpy arrays and call it.  Nothing here computes: every
step of the oracle's arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pard_oracle.c")
_LIB = os.path.join(_HERE, "libpard_oracle.so")
_lib: Optional[ctypes.CDLL] = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def build_oracle(force: bool = False) -> str:
    """Compile the oracle (gcc -O2 -fopenmp).  Rebuilds when the source is newer."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        lib.pard_oracle_estimate_drop.restype = ctypes.c_int
        lib.pard_oracle_estimate_drop.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            _i32p, _i32p, _i32p, _i32p, _i32p, _i32p,
            ctypes.c_int64, _i32p, _i32p, _i32p, _i32p, _i32p,
            _i32p, _u8p, _i32p, _i32p, ctypes.c_int32]
        lib.pard_oracle_estimate_drop_ranked.restype = ctypes.c_int
        lib.pard_oracle_estimate_drop_ranked.argtypes = lib.pard_oracle_estimate_drop.argtypes
        lib.pard_oracle_estimate_drop_sub.restype = ctypes.c_int
        lib.pard_oracle_estimate_drop_sub.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            _i32p, _i32p, _i32p, _i32p, _i32p, _i32p,
            ctypes.c_int64, _i32p, _i32p, _i32p, _i32p, _i32p, _i64p,
            _i32p, _u8p, _i32p, _i32p, ctypes.c_int32]
        lib.pard_oracle_estimate_drop_consistent.restype = ctypes.c_int
        lib.pard_oracle_estimate_drop_consistent.argtypes = lib.pard_oracle_estimate_drop_sub.argtypes
        lib.pard_oracle_sub_latency.restype = ctypes.c_int
        lib.pard_oracle_sub_latency.argtypes = [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            _i32p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p,
            ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, _i32p, ctypes.POINTER(ctypes.c_uint32),
            _i64p, ctypes.c_int32]
        lib.pard_oracle_priority_modes.restype = ctypes.c_int
        lib.pard_oracle_priority_modes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _i32p, _i32p, _i32p,
                                                   ctypes.c_int32, ctypes.c_int32, _i32p, _i32p, _i32p]
        lib.pard_oracle_queue_delay.restype = ctypes.c_int
        lib.pard_oracle_queue_delay.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                                _i32p, _i32p, _i32p, _i32p]
        lib.pard_oracle_compact.restype = ctypes.c_int
        lib.pard_oracle_compact.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                            _i32p, _i32p, _u8p, _i32p, _i32p]
        lib.pard_oracle_nexus_drop.restype = ctypes.c_int
        lib.pard_oracle_nexus_drop.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _i32p, _i32p, ctypes.c_int64,
                                               _i32p, _i32p, _i32p, _i32p, _u8p, _i32p]
        lib.pard_oracle_clipper_drop.restype = ctypes.c_int
        lib.pard_oracle_clipper_drop.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _i32p, _i32p, _i32p, _i32p,
                                                 ctypes.c_int64, _i32p, _i32p, _i32p, _i32p, _i32p, _u8p]
        lib.pard_oracle_paths.restype = ctypes.c_int
        lib.pard_oracle_paths.argtypes = [ctypes.c_int32, _i32p, _i32p, _i64p, _i64p,
                                          _i32p, ctypes.c_int64, _i32p, ctypes.c_int64]
        lib.pard_oracle_stage_cost.restype = ctypes.c_int64
        lib.pard_oracle_stage_cost.argtypes = [_i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64]
        _lib = lib
    return _lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p32(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


VARIANT_FULL, VARIANT_LOWER, VARIANT_UPPER, VARIANT_SF, VARIANT_BACK = range(5)


def sub_latency(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, qlen, variant=VARIANT_FULL,
                lam=(1, 10), samples=None, picks=None, threads: int = 1, qdelay=None):
    """Downstream latency L_sub per (snapshot, stage): int64[K*S].  qdelay: monitored q_i, int32[K*S]."""
    lib = _load()
    rp, cl, B, W, L, q = map(_i32, (dag_row_ptr, dag_col, batch, workers, lat_us, qlen))
    if cl.size == 0:
        cl = np.zeros(1, np.int32)
    M = 0 if samples is None else int(np.asarray(samples).shape[0])
    smp = _i32(samples) if M else np.zeros(1, np.int32)
    pk = np.ascontiguousarray(picks, dtype=np.uint32) if M else np.zeros(1, np.uint32)
    if M:
        assert pk.size == M * S
    qd = None if qdelay is None else _i32(qdelay)
    if qd is not None:
        assert qd.size == K * S
    out = np.zeros(K * S, np.int64)
    rc = lib.pard_oracle_sub_latency(
        K, S, int(dag_shared), _p32(rp), _p32(cl), _p32(B), _p32(W), _p32(L), _p32(q),
        None if qd is None else _p32(qd),
        int(variant), int(lam[0]), int(lam[1]), M, _p32(smp), pk.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
        out.ctypes.data_as(_i64p), int(threads))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return out


def queue_delay(K, S, time, delay, now, window):
    """Linearly weighted sliding-window mean of the delay samples per (snapshot, stage): int32[K*S].
    time, delay: int32[K*S, len]; now: int32[K]."""
    lib = _load()
    tm = np.ascontiguousarray(_i32(time).reshape(K * S, -1))
    dl = np.ascontiguousarray(_i32(delay).reshape(K * S, -1))
    assert tm.shape == dl.shape
    nw = _i32(now)
    assert nw.size == K
    out = np.zeros(K * S, np.int32)
    if tm.shape[1] == 0:
        tm = np.zeros((K * S, 1), np.int32); dl = tm.copy(); length = 0
    else:
        length = int(tm.shape[1])
    rc = lib.pard_oracle_queue_delay(K, S, length, int(window), _p32(tm), _p32(dl), _p32(nw), _p32(out))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return out


def priority_modes(K, S, dag_shared, batch, workers, lat_us, rate, window, prev_mode=None):
    """Priority (0 = LBF, 1 = HBF) in force per (snapshot, stage) after the rate series: int32[K*S].
    rate: int32[K*S, T]."""
    lib = _load()
    B, W, L = map(_i32, (batch, workers, lat_us))
    rt = _i32(rate).reshape(K * S, -1)
    T = int(rt.shape[1])
    pm = None if prev_mode is None else _i32(prev_mode)
    out = np.zeros(K * S, np.int32)
    rc = lib.pard_oracle_priority_modes(K, S, int(dag_shared), _p32(B), _p32(W), _p32(L), T, int(window),
                                        _p32(np.ascontiguousarray(rt)), None if pm is None else _p32(pm), _p32(out))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return out


def estimate_drop(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, order_mode,
                  arrival, deadline, stage, snap_ptr, now, threads: int = 1, sub=None, consistent: bool = False,
                  ranked: bool = False):
    """Returns (est int32[n], drop uint8[n], order int32[n], seg_ptr int32[K*S+1]).
    With `sub` (int64[K*S]) the downstream part of every estimate is taken from it.
    `consistent`: positions count only the kept requests ahead (sequentially consistent dropping).
    `ranked`: in later queues a request counts only the requests their order serves before it."""
    lib = _load()
    rp, cl, B, W, L, M = map(_i32, (dag_row_ptr, dag_col, batch, workers, lat_us, order_mode))
    if cl.size == 0:
        cl = np.zeros(1, np.int32)
    arr, ddl, stg, sp, nw = map(_i32, (arrival, deadline, stage, snap_ptr, now))
    n = int(arr.shape[0])
    est = np.zeros(max(n, 1), np.int32)
    drop = np.zeros(max(n, 1), np.uint8)
    order = np.zeros(max(n, 1), np.int32)
    seg_ptr = np.zeros(K * S + 1, np.int32)
    pad = lambda a: a if a.size else np.zeros(1, np.int32)  # noqa: E731
    if ranked:
        assert sub is None and not consistent
        rc = lib.pard_oracle_estimate_drop_ranked(
            K, S, int(dag_shared), _p32(rp), _p32(cl), _p32(B), _p32(W), _p32(L), _p32(M),
            n, _p32(pad(arr)), _p32(pad(ddl)), _p32(pad(stg)), _p32(sp), _p32(pad(nw)),
            _p32(est), drop.ctypes.data_as(_u8p), _p32(order), _p32(seg_ptr), int(threads))
    elif consistent:
        sb = None if sub is None else np.ascontiguousarray(sub, dtype=np.int64)
        rc = lib.pard_oracle_estimate_drop_consistent(
            K, S, int(dag_shared), _p32(rp), _p32(cl), _p32(B), _p32(W), _p32(L), _p32(M),
            n, _p32(pad(arr)), _p32(pad(ddl)), _p32(pad(stg)), _p32(sp), _p32(pad(nw)),
            None if sb is None else sb.ctypes.data_as(_i64p),
            _p32(est), drop.ctypes.data_as(_u8p), _p32(order), _p32(seg_ptr), int(threads))
    elif sub is None:
        rc = lib.pard_oracle_estimate_drop(
            K, S, int(dag_shared), _p32(rp), _p32(cl), _p32(B), _p32(W), _p32(L), _p32(M),
            n, _p32(pad(arr)), _p32(pad(ddl)), _p32(pad(stg)), _p32(sp), _p32(pad(nw)),
            _p32(est), drop.ctypes.data_as(_u8p), _p32(order), _p32(seg_ptr), int(threads))
    else:
        sb = np.ascontiguousarray(sub, dtype=np.int64)
        assert sb.size == K * S
        rc = lib.pard_oracle_estimate_drop_sub(
            K, S, int(dag_shared), _p32(rp), _p32(cl), _p32(B), _p32(W), _p32(L), _p32(M),
            n, _p32(pad(arr)), _p32(pad(ddl)), _p32(pad(stg)), _p32(sp), _p32(pad(nw)), sb.ctypes.data_as(_i64p),
            _p32(est), drop.ctypes.data_as(_u8p), _p32(order), _p32(seg_ptr), int(threads))
    if rc != 0:
        raise ValueError(f"oracle rejected the DAG (code {rc})")
    return est[:n], drop[:n], order[:n], seg_ptr


def compact(K, S, order, seg_ptr, drop):
    """Returns (surv_idx int32[count], surv_ptr int32[K*S+1])."""
    lib = _load()
    order = _i32(order)
    seg_ptr = _i32(seg_ptr)
    drop = np.ascontiguousarray(drop, np.uint8)
    n = int(order.shape[0])
    surv = np.zeros(max(n, 1), np.int32)
    surv_ptr = np.zeros(K * S + 1, np.int32)
    o = order if n else np.zeros(1, np.int32)
    d = drop if n else np.zeros(1, np.uint8)
    lib.pard_oracle_compact(K, S, n, _p32(o), _p32(seg_ptr), d.ctypes.data_as(_u8p),
                            _p32(surv), _p32(surv_ptr))
    return surv[:int(surv_ptr[-1])], surv_ptr


def nexus_drop(K, S, dag_shared, batch, lat_us, deadline, order, seg_ptr, now):
    """Reactive window scan over the given queues: (drop uint8[n], first_kept int32[K*S])."""
    lib = _load()
    B, L, ddl, od, sp, nw = map(_i32, (batch, lat_us, deadline, order, seg_ptr, now))
    n = int(ddl.shape[0])
    drop = np.zeros(max(n, 1), np.uint8)
    first = np.zeros(K * S, np.int32)
    pad = lambda a: a if a.size else np.zeros(1, np.int32)  # noqa: E731
    rc = lib.pard_oracle_nexus_drop(K, S, int(dag_shared), _p32(B), _p32(L), n, _p32(pad(ddl)), _p32(pad(od)), _p32(sp),
                                    _p32(nw), drop.ctypes.data_as(_u8p), _p32(first))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return drop[:n], first


def clipper_drop(K, S, dag_shared, dag_row_ptr, dag_col, batch, lat_us, arrival, deadline, stage, snap_ptr, now):
    """Per-module SLO split: drop uint8[n]."""
    lib = _load()
    rp, cl, B, L = map(_i32, (dag_row_ptr, dag_col, batch, lat_us))
    if cl.size == 0:
        cl = np.zeros(1, np.int32)
    arr, ddl, stg, sp, nw = map(_i32, (arrival, deadline, stage, snap_ptr, now))
    n = int(arr.shape[0])
    drop = np.zeros(max(n, 1), np.uint8)
    pad = lambda a: a if a.size else np.zeros(1, np.int32)  # noqa: E731
    rc = lib.pard_oracle_clipper_drop(K, S, int(dag_shared), _p32(rp), _p32(cl), _p32(B), _p32(L), n, _p32(pad(arr)),
                                      _p32(pad(ddl)), _p32(pad(stg)), _p32(sp), _p32(nw), drop.ctypes.data_as(_u8p))
    if rc != 0:
        raise ValueError(f"oracle rejected the arguments (code {rc})")
    return drop[:n]


def expand_paths(S, dag_row_ptr, dag_col):
    """All source-to-sink paths of one DAG: (path_ptr, path_stage); raises on a bad DAG."""
    lib = _load()
    rp, cl = _i32(dag_row_ptr), _i32(dag_col)
    if cl.size == 0:
        cl = np.zeros(1, np.int32)
    P = ctypes.c_int64(0)
    mx = ctypes.c_int64(0)
    rc = lib.pard_oracle_paths(S, _p32(rp), _p32(cl), ctypes.byref(P), ctypes.byref(mx), None, 0, None, 0)
    if rc:
        raise ValueError(f"bad DAG (code {rc})")
    ptr = np.zeros(P.value + 1, np.int32)
    stg = np.zeros(max(1, P.value * max(1, mx.value)), np.int32)
    rc = lib.pard_oracle_paths(S, _p32(rp), _p32(cl), ctypes.byref(P), ctypes.byref(mx),
                               _p32(ptr), ptr.size, _p32(stg), stg.size)
    if rc:
        raise ValueError(f"bad DAG (code {rc})")
    return ptr, stg[:int(ptr[-1])]


def stage_cost(lat64, B: int, W: int, a: int) -> int:
    lib = _load()
    L = _i32(lat64)
    return int(lib.pard_oracle_stage_cost(_p32(L), int(B), int(W), int(a)))


def run(w, threads: int = 1, sub=None, consistent: bool = False, ranked: bool = False):
    """Whole path on a workloads.Workload: dict of est, drop, order, seg_ptr, surv_idx, surv_ptr."""
    est, drop, order, seg_ptr = estimate_drop(
        w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers, w.lat_us, w.order_mode,
        w.arrival, w.deadline, w.stage, w.snap_ptr, w.now, threads=threads, sub=sub, consistent=consistent,
        ranked=ranked)
    surv_idx, surv_ptr = compact(w.K, w.S, order, seg_ptr, drop)
    return dict(est=est, drop=drop, order=order, seg_ptr=seg_ptr, surv_idx=surv_idx, surv_ptr=surv_ptr)
