"""Thin ctypes binding of libpard.so: same names as the C entry points, argument
marshalling only.  Device buffers are torch tensors on a ROCm device (torch is used for
device memory and streams, nothing else); every step of the path runs in the library's
kernels.  There is no CPU fallback: if the library cannot be loaded the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import build as _build

_i32p = ctypes.POINTER(ctypes.c_int32)
_lib: Optional[ctypes.CDLL] = None

PARD_OK = 0
PARD_FUSED_SNAPSHOT_CAPACITY = 8192
STATUS_NAMES = {
    0: "PARD_OK", -1: "PARD_E_NULL", -2: "PARD_E_BAD_SHAPE", -3: "PARD_E_BAD_BATCH", -4: "PARD_E_BAD_WORKERS",
    -5: "PARD_E_BAD_LATENCY", -6: "PARD_E_BAD_DAG", -7: "PARD_E_TOO_MANY_PATHS", -8: "PARD_E_WORKSPACE",
    -9: "PARD_E_HIP", -10: "PARD_E_BAD_MODE", -11: "PARD_E_UNSUPPORTED", -12: "PARD_E_SCRATCH",
}
EXPORTS = ["pard_plan_check", "pard_plan_create", "pard_plan_destroy", "pard_plan_info",
           "pard_workspace_bytes", "pard_estimate_drop", "pard_estimate_drop_sub", "pard_estimate_drop_consistent",
           "pard_estimate_drop_ranked", "pard_estimate_drop_static", "pard_estimate_drop_compact", "pard_reactive_drop",
           "pard_queue_lengths", "pard_priority_modes", "pard_plan_set_modes",
           "pard_sub_latency", "pard_sub_latency_q", "pard_queue_delay", "pard_compact", "pard_strerror"]
SUB_FULL, SUB_LOWER, SUB_UPPER, SUB_SF, SUB_BACK = range(5)
REACTIVE_WINDOW_SCAN, REACTIVE_SLO_SPLIT = 0, 1


class PardError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load_library().pard_strerror(code).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(code, code)} ({msg})")


class PlanDesc(ctypes.Structure):
    _fields_ = [("num_snapshots", ctypes.c_int32), ("num_stages", ctypes.c_int32), ("dag_shared", ctypes.c_int32),
                ("dag_row_ptr", _i32p), ("dag_col", _i32p), ("batch", _i32p), ("workers", _i32p),
                ("lat_us", _i32p), ("order_mode", _i32p)]


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads the built library.  The in-tree library is rebuilt first when it is missing or was built
    from other sources than the ones in the tree (a stale binary is never loaded silently)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or os.environ.get("PARD_LIBRARY") or _build.LIB_PATH
    if p == _build.LIB_PATH and _build.is_stale():
        _build.build_library(incremental=True)
    lib = ctypes.CDLL(p)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.pard_plan_check.argtypes = [ctypes.POINTER(PlanDesc), ctypes.POINTER(i64), ctypes.POINTER(i32)]
    lib.pard_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(PlanDesc)]
    lib.pard_plan_destroy.argtypes = [vp]
    lib.pard_plan_info.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i32)]
    lib.pard_workspace_bytes.argtypes = [vp, i64, i64, ctypes.POINTER(i64)]
    lib.pard_estimate_drop.argtypes = [vp, i64, i64] + [vp] * 9 + [vp, i64, vp]
    lib.pard_estimate_drop_ranked.argtypes = lib.pard_estimate_drop.argtypes
    lib.pard_estimate_drop_static.argtypes = [vp, i64, i64] + [vp] * 9 + [vp, vp]
    lib.pard_estimate_drop_compact.argtypes = [vp, i64, i64] + [vp] * 11 + [vp, i64, vp, vp]
    lib.pard_compact.argtypes = [vp, i64, i64] + [vp] * 5 + [vp, i64, vp]
    lib.pard_reactive_drop.argtypes = [vp, i32, i64] + [vp] * 10
    lib.pard_estimate_drop_sub.argtypes = [vp, i64, i64] + [vp] * 10 + [vp, i64, vp]
    lib.pard_estimate_drop_consistent.argtypes = [vp, i64, i64] + [vp] * 10 + [vp, i64, vp]
    lib.pard_queue_lengths.argtypes = [vp, i64, vp, vp, vp, vp]
    lib.pard_priority_modes.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp]
    lib.pard_plan_set_modes.argtypes = [vp, vp, vp]
    lib.pard_sub_latency.argtypes = [vp, vp, ctypes.c_int32, i64, i64, ctypes.c_int32, vp, vp, vp, vp]
    lib.pard_sub_latency_q.argtypes = [vp, vp, vp, ctypes.c_int32, i64, i64, ctypes.c_int32, vp, vp, vp, vp]
    lib.pard_queue_delay.argtypes = [vp, ctypes.c_int32, i64, vp, vp, vp, vp, vp]
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ctypes.c_int
    lib.pard_strerror.argtypes = [ctypes.c_int]
    lib.pard_strerror.restype = ctypes.c_char_p
    if path is None:
        _lib = lib
    return lib


def _desc(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, order_mode):
    keep = [np.ascontiguousarray(a, dtype=np.int32) for a in (dag_row_ptr, dag_col, batch, workers, lat_us, order_mode)]
    ptr = [a.ctypes.data_as(_i32p) if a.size else None for a in keep]
    d = PlanDesc(int(K), int(S), int(dag_shared), *ptr)
    return d, keep


def pard_plan_check(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, order_mode):
    """Host-only validation + path expansion.  Returns (status, total_paths, max_path_len)."""
    lib = load_library()
    d, keep = _desc(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, order_mode)
    tp, ml = ctypes.c_int64(0), ctypes.c_int32(0)
    rc = lib.pard_plan_check(ctypes.byref(d), ctypes.byref(tp), ctypes.byref(ml))
    del keep
    return rc, tp.value, ml.value


class Plan:
    """Owner of a pard_plan_t*."""

    def __init__(self, handle: int, K: int, S: int):
        self.handle = ctypes.c_void_p(handle)
        self.K, self.S = K, S

    def destroy(self):
        if self.handle:
            load_library().pard_plan_destroy(self.handle)
            self.handle = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def pard_plan_create(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, order_mode) -> Plan:
    lib = load_library()
    d, keep = _desc(K, S, dag_shared, dag_row_ptr, dag_col, batch, workers, lat_us, order_mode)
    h = ctypes.c_void_p(None)
    rc = lib.pard_plan_create(ctypes.byref(h), ctypes.byref(d))
    del keep
    if rc != PARD_OK:
        raise PardError(rc, "pard_plan_create")
    return Plan(h.value, int(K), int(S))


def pard_plan_info(plan: Plan):
    tp, ml = ctypes.c_int64(0), ctypes.c_int32(0)
    rc = load_library().pard_plan_info(plan.handle, ctypes.byref(tp), ctypes.byref(ml))
    if rc != PARD_OK:
        raise PardError(rc, "pard_plan_info")
    return tp.value, ml.value


def pard_workspace_bytes(plan: Plan, max_requests: int, max_snapshot_requests: int) -> int:
    b = ctypes.c_int64(0)
    rc = load_library().pard_workspace_bytes(plan.handle, int(max_requests), int(max_snapshot_requests), ctypes.byref(b))
    if rc != PARD_OK:
        raise PardError(rc, "pard_workspace_bytes")
    return b.value


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else ctypes.c_void_p(None)


def _stream_handle(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def pard_estimate_drop(plan: Plan, n: int, max_snapshot_requests: int, arrival, deadline, stage, snap_ptr, now,
                       est, drop, order, seg_ptr, workspace, stream=None, check: bool = True) -> int:
    """Enqueues the estimate + drop kernels on `stream` (default: torch's current stream)."""
    rc = load_library().pard_estimate_drop(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(arrival), _ptr(deadline), _ptr(stage),
        _ptr(snap_ptr), _ptr(now), _ptr(est), _ptr(drop), _ptr(order), _ptr(seg_ptr),
        _ptr(workspace), int(workspace.numel() * workspace.element_size()), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_estimate_drop")
    return rc


def pard_estimate_drop_static(plan: Plan, n: int, max_snapshot_requests: int, arrival, deadline, stage, snap_ptr, now,
                              est, drop, order, seg_ptr, status=None, stream=None, check: bool = True) -> int:
    """pard_estimate_drop on the library's built-in scratch buffer (no workspace, nothing allocated)."""
    rc = load_library().pard_estimate_drop_static(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(arrival), _ptr(deadline), _ptr(stage),
        _ptr(snap_ptr), _ptr(now), _ptr(est), _ptr(drop), _ptr(order), _ptr(seg_ptr), _ptr(status),
        _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_estimate_drop_static")
    return rc


def pard_estimate_drop_compact(plan: Plan, n: int, max_snapshot_requests: int, arrival, deadline, stage, snap_ptr, now,
                               est, drop, order, seg_ptr, surv_idx, surv_ptr, workspace, between_event=None, stream=None,
                               check: bool = True) -> int:
    """The whole path in one call (estimate, drop decision, survivor queues).  between_event: a raw hipEvent_t
    handle (int) recorded between the two steps, or None."""
    rc = load_library().pard_estimate_drop_compact(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(arrival), _ptr(deadline), _ptr(stage),
        _ptr(snap_ptr), _ptr(now), _ptr(est), _ptr(drop), _ptr(order), _ptr(seg_ptr), _ptr(surv_idx), _ptr(surv_ptr),
        _ptr(workspace), int(workspace.numel() * workspace.element_size()),
        ctypes.c_void_p(between_event) if between_event else ctypes.c_void_p(None), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_estimate_drop_compact")
    return rc


def pard_estimate_drop_ranked(plan: Plan, n: int, max_snapshot_requests: int, arrival, deadline, stage, snap_ptr, now,
                              est, drop, order, seg_ptr, workspace, stream=None, check: bool = True) -> int:
    """pard_estimate_drop with ranked positions in the later queues."""
    rc = load_library().pard_estimate_drop_ranked(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(arrival), _ptr(deadline), _ptr(stage),
        _ptr(snap_ptr), _ptr(now), _ptr(est), _ptr(drop), _ptr(order), _ptr(seg_ptr),
        _ptr(workspace), int(workspace.numel() * workspace.element_size()), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_estimate_drop_ranked")
    return rc


def pard_estimate_drop_sub(plan: Plan, n: int, max_snapshot_requests: int, arrival, deadline, stage, snap_ptr, now, sub,
                           est, drop, order, seg_ptr, workspace, stream=None, check: bool = True) -> int:
    """pard_estimate_drop with the downstream latency per (snapshot, stage) given."""
    rc = load_library().pard_estimate_drop_sub(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(arrival), _ptr(deadline), _ptr(stage), _ptr(snap_ptr),
        _ptr(now), _ptr(sub), _ptr(est), _ptr(drop), _ptr(order), _ptr(seg_ptr),
        _ptr(workspace), int(workspace.numel() * workspace.element_size()), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_estimate_drop_sub")
    return rc


def pard_estimate_drop_consistent(plan: Plan, n: int, max_snapshot_requests: int, arrival, deadline, stage, snap_ptr, now,
                                  sub, est, drop, order, seg_ptr, workspace, stream=None, check: bool = True) -> int:
    """Sequentially consistent dropping (positions count kept requests only); `sub` may be None."""
    rc = load_library().pard_estimate_drop_consistent(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(arrival), _ptr(deadline), _ptr(stage), _ptr(snap_ptr),
        _ptr(now), _ptr(sub), _ptr(est), _ptr(drop), _ptr(order), _ptr(seg_ptr),
        _ptr(workspace), int(workspace.numel() * workspace.element_size()), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_estimate_drop_consistent")
    return rc


def pard_queue_lengths(plan: Plan, n: int, stage, snap_ptr, qlen, stream=None, check: bool = True) -> int:
    """Enqueues the queue-length count on `stream`."""
    rc = load_library().pard_queue_lengths(plan.handle, int(n), _ptr(stage), _ptr(snap_ptr), _ptr(qlen),
                                           _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_queue_lengths")
    return rc


def pard_priority_modes(plan: Plan, series_len: int, window: int, rate, prev_mode, mode, stream=None, check: bool = True) -> int:
    """Enqueues the adaptive-priority decision (one mode per (snapshot, stage)) on `stream`."""
    rc = load_library().pard_priority_modes(plan.handle, int(series_len), int(window), _ptr(rate), _ptr(prev_mode), _ptr(mode),
                                            _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_priority_modes")
    return rc


def pard_plan_set_modes(plan: Plan, mode, stream=None, check: bool = True) -> int:
    """Installs per-stage queue orders (device int32 array) in the plan."""
    rc = load_library().pard_plan_set_modes(plan.handle, _ptr(mode), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_plan_set_modes")
    return rc


def pard_sub_latency(plan: Plan, qlen, variant: int, lambda_num: int, lambda_den: int, num_samples: int, samples, picks,
                     sub, stream=None, check: bool = True) -> int:
    """Enqueues the downstream-latency kernels on `stream`."""
    rc = load_library().pard_sub_latency(plan.handle, _ptr(qlen), int(variant), int(lambda_num), int(lambda_den),
                                         int(num_samples), _ptr(samples), _ptr(picks), _ptr(sub), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_sub_latency")
    return rc


def pard_sub_latency_q(plan: Plan, qlen, qdelay, variant: int, lambda_num: int, lambda_den: int, num_samples: int, samples,
                       picks, sub, stream=None, check: bool = True) -> int:
    """pard_sub_latency with monitored queueing delays (device int32[K*S]) for the q_i."""
    rc = load_library().pard_sub_latency_q(plan.handle, _ptr(qlen), _ptr(qdelay), int(variant), int(lambda_num),
                                           int(lambda_den), int(num_samples), _ptr(samples), _ptr(picks), _ptr(sub),
                                           _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_sub_latency_q")
    return rc


def pard_queue_delay(plan: Plan, series_len: int, window_us: int, time, delay, now, q, stream=None, check: bool = True) -> int:
    """Enqueues the sliding-window queueing delay (one value per (snapshot, stage)) on `stream`."""
    rc = load_library().pard_queue_delay(plan.handle, int(series_len), int(window_us), _ptr(time), _ptr(delay), _ptr(now),
                                         _ptr(q), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_queue_delay")
    return rc


def pard_reactive_drop(plan: Plan, policy: int, n: int, arrival, deadline, stage, snap_ptr, now, order, seg_ptr, drop,
                       first_kept, stream=None, check: bool = True) -> int:
    """Enqueues a reactive dropping policy (window scan or per-module SLO split) on `stream`."""
    rc = load_library().pard_reactive_drop(plan.handle, int(policy), int(n), _ptr(arrival), _ptr(deadline), _ptr(stage),
                                           _ptr(snap_ptr), _ptr(now), _ptr(order), _ptr(seg_ptr), _ptr(drop), _ptr(first_kept),
                                           _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_reactive_drop")
    return rc


def pard_compact(plan: Plan, n: int, max_snapshot_requests: int, order, seg_ptr, drop, surv_idx, surv_ptr, workspace,
                 stream=None, check: bool = True) -> int:
    """Enqueues the survivor-compaction kernels on `stream`."""
    rc = load_library().pard_compact(
        plan.handle, int(n), int(max_snapshot_requests), _ptr(order), _ptr(seg_ptr), _ptr(drop), _ptr(surv_idx),
        _ptr(surv_ptr),
        _ptr(workspace), int(workspace.numel() * workspace.element_size()), _stream_handle(stream))
    if check and rc != PARD_OK:
        raise PardError(rc, "pard_compact")
    return rc


class Session:
    """Device buffers for one workload: inputs uploaded once, outputs and workspace allocated
    with torch.  run() is the whole hot path: pard_estimate_drop followed by pard_compact."""

    def __init__(self, w, device="cuda:0", max_snapshot_requests: Optional[int] = None):
        import torch
        self.torch = torch
        self.w = w
        self.dev = torch.device(device)
        self.plan = pard_plan_create(w.K, w.S, w.dag_shared, w.dag_row_ptr, w.dag_col, w.batch, w.workers,
                                     w.lat_us, w.order_mode)
        self.n = w.n
        self.max_snap = w.max_snapshot_requests if max_snapshot_requests is None else max_snapshot_requests
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)  # noqa: E731
        self.arrival, self.deadline, self.stage = up(w.arrival), up(w.deadline), up(w.stage)
        self.snap_ptr, self.now = up(w.snap_ptr), up(w.now)
        n1 = max(self.n, 1)
        self.est = torch.empty(n1, dtype=torch.int32, device=self.dev)
        self.drop = torch.empty(n1, dtype=torch.uint8, device=self.dev)
        self.order = torch.empty(n1, dtype=torch.int32, device=self.dev)
        self.seg_ptr = torch.empty(w.K * w.S + 1, dtype=torch.int32, device=self.dev)
        self.surv_idx = torch.empty(n1, dtype=torch.int32, device=self.dev)
        self.surv_ptr = torch.empty(w.K * w.S + 1, dtype=torch.int32, device=self.dev)
        self.ws_bytes = pard_workspace_bytes(self.plan, self.n, self.max_snap)
        self.workspace = torch.zeros(self.ws_bytes // 4 + 64, dtype=torch.int32, device=self.dev)
        assert self.workspace.data_ptr() % 256 == 0

    def estimate_drop(self, stream=None, sub=None, consistent=False, ranked=False):
        if ranked:
            pard_estimate_drop_ranked(self.plan, self.n, self.max_snap, self.arrival, self.deadline, self.stage, self.snap_ptr,
                                      self.now, self.est, self.drop, self.order, self.seg_ptr, self.workspace, stream)
        elif consistent:
            pard_estimate_drop_consistent(self.plan, self.n, self.max_snap, self.arrival, self.deadline, self.stage,
                                          self.snap_ptr, self.now, sub, self.est, self.drop, self.order, self.seg_ptr,
                                          self.workspace, stream)
        elif sub is None:
            pard_estimate_drop(self.plan, self.n, self.max_snap, self.arrival, self.deadline, self.stage, self.snap_ptr,
                               self.now, self.est, self.drop, self.order, self.seg_ptr, self.workspace, stream)
        else:
            pard_estimate_drop_sub(self.plan, self.n, self.max_snap, self.arrival, self.deadline, self.stage,
                                   self.snap_ptr, self.now, sub, self.est, self.drop, self.order, self.seg_ptr,
                                   self.workspace, stream)

    def planner(self, variant=SUB_FULL, lam=(1, 10), samples=None, picks=None, stream=None, qdelay=None):
        """Queue lengths, then the downstream latency per (snapshot, stage) (device int64[K*S]).
        qdelay: monitored queueing delays (device int32[K*S]) to use for the q_i."""
        torch = self.torch
        if not hasattr(self, "qlen"):
            self.qlen = torch.empty(self.w.K * self.w.S, dtype=torch.int32, device=self.dev)
            self.sub = torch.empty(self.w.K * self.w.S, dtype=torch.int64, device=self.dev)
        pard_queue_lengths(self.plan, self.n, self.stage, self.snap_ptr, self.qlen, stream)
        m = 0 if samples is None else int(samples.numel())
        if qdelay is None:
            pard_sub_latency(self.plan, self.qlen, variant, lam[0], lam[1], m, samples, picks, self.sub, stream)
        else:
            pard_sub_latency_q(self.plan, self.qlen, qdelay, variant, lam[0], lam[1], m, samples, picks, self.sub, stream)
        return self.sub

    def compact(self, stream=None):
        pard_compact(self.plan, self.n, self.max_snap, self.order, self.seg_ptr, self.drop, self.surv_idx, self.surv_ptr,
                     self.workspace, stream)

    def run(self, stream=None, sub=None, consistent=False, ranked=False):
        self.estimate_drop(stream, sub, consistent, ranked)
        self.compact(stream)

    def run_one_call(self, stream=None, between_event=None):
        """The whole path through pard_estimate_drop_compact."""
        pard_estimate_drop_compact(self.plan, self.n, self.max_snap, self.arrival, self.deadline, self.stage, self.snap_ptr,
                                   self.now, self.est, self.drop, self.order, self.seg_ptr, self.surv_idx, self.surv_ptr,
                                   self.workspace, between_event, stream)

    def status_word(self) -> int:
        return int(self.workspace[0].item())

    def results(self):
        """Host copies of every output (synchronises)."""
        self.torch.cuda.synchronize(self.dev)
        n = self.n
        sp = self.surv_ptr.cpu().numpy()
        return dict(est=self.est[:n].cpu().numpy(), drop=self.drop[:n].cpu().numpy(),
                    order=self.order[:n].cpu().numpy(), seg_ptr=self.seg_ptr.cpu().numpy(),
                    surv_idx=self.surv_idx[:int(sp[-1])].cpu().numpy(), surv_ptr=sp)
