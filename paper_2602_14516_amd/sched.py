"""ctypes binding of libampd_sched.so (host-only): adaptive routing and prefill reordering."""
from __future__ import annotations

import ctypes
import os

import numpy as np

SCHED_LIB_PATH = os.environ.get("AMPD_SCHED_LIB_PATH") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libampd_sched.so")
SCHED_SYMBOLS = ["ampd_t_pre", "ampd_route", "ampd_reorder"]
ROUTE_LOCAL, ROUTE_ERROR = -1, -2
MAX_WINDOW = 8


class _Task(ctypes.Structure):
    _fields_ = [("l_hist", ctypes.c_int32), ("l_incr", ctypes.c_int32)]


class _TPre(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("l_incr", ctypes.c_void_p), ("alpha", ctypes.c_void_p), ("beta", ctypes.c_void_p)]


class _TKv(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("beta", ctypes.c_double)]


class _RouteIn(ctypes.Structure):
    _fields_ = [("n_prefill_workers", ctypes.c_int32), ("ttft_hat", ctypes.c_void_p), ("itl_hat", ctypes.c_double),
                ("ttft_thres", ctypes.c_double), ("itl_thres", ctypes.c_double), ("alpha", ctypes.c_double),
                ("beta", ctypes.c_double), ("visit_order", ctypes.c_void_p), ("decode_model", ctypes.POINTER(_TPre)),
                ("prefill_models", ctypes.POINTER(_TPre)), ("kv_d2p", ctypes.POINTER(_TKv)), ("kv_p2d", ctypes.POINTER(_TKv)),
                ("local_queue", ctypes.POINTER(_Task)), ("local_queue_len", ctypes.c_int32),
                ("remote_queues", ctypes.POINTER(ctypes.POINTER(_Task))), ("remote_queue_len", ctypes.c_void_p)]


class _QTask(ctypes.Structure):
    _fields_ = [("t_pre", ctypes.c_double), ("enqueue_time", ctypes.c_double), ("postponed", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


def _load():
    if not os.path.exists(SCHED_LIB_PATH):
        raise ImportError(f"{SCHED_LIB_PATH} is missing: build it with `python -m paper_2602_14516_amd.build`")
    L = ctypes.CDLL(SCHED_LIB_PATH)
    L.ampd_t_pre.restype = ctypes.c_double
    L.ampd_t_pre.argtypes = [ctypes.POINTER(_TPre), ctypes.c_int32, ctypes.c_int32]
    L.ampd_route.restype = ctypes.c_int32
    L.ampd_route.argtypes = [ctypes.POINTER(_RouteIn), _Task, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)]
    L.ampd_reorder.restype = ctypes.c_int32
    L.ampd_reorder.argtypes = [ctypes.POINTER(_QTask), ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                               ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)]
    return L


lib = _load()


class TPreModel:
    """(l_incr buckets, alpha, beta) -> C struct; keeps the arrays alive."""

    def __init__(self, l_incr, alpha, beta):
        self.a = [np.ascontiguousarray(x, dtype=np.float64) for x in (l_incr, alpha, beta)]
        self.c = _TPre(len(self.a[0]), *(x.ctypes.data for x in self.a))


def t_pre(model: TPreModel, l_hist: int, l_incr: int) -> float:
    return float(lib.ampd_t_pre(ctypes.byref(model.c), int(l_hist), int(l_incr)))


def route(task, ttft_hat, itl_hat, ttft_thres, itl_thres, alpha, beta, visit_order, decode_model, prefill_models,
          kv_d2p, kv_p2d, local_queue, remote_queues):
    """Algorithm 1.  Returns (route, costs, reason): route = 'local' or a prefill-worker index."""
    n = len(prefill_models)
    th = np.ascontiguousarray(ttft_hat, dtype=np.float64)
    vo = np.ascontiguousarray(visit_order, dtype=np.int32)
    pm = (_TPre * max(n, 1))(*[m.c for m in prefill_models])
    d2p = (_TKv * max(n, 1))(*[_TKv(*x) for x in kv_d2p])
    p2d = (_TKv * max(n, 1))(*[_TKv(*x) for x in kv_p2d])
    lq = (_Task * max(len(local_queue), 1))(*[_Task(*x) for x in local_queue])
    rqs = [(_Task * max(len(q), 1))(*[_Task(*x) for x in q]) for q in remote_queues]
    rq_ptrs = (ctypes.POINTER(_Task) * max(n, 1))(*[ctypes.cast(q, ctypes.POINTER(_Task)) for q in rqs])
    rlen = np.array([len(q) for q in remote_queues], dtype=np.int32)
    inp = _RouteIn(n, th.ctypes.data, itl_hat, ttft_thres, itl_thres, alpha, beta, vo.ctypes.data,
                   ctypes.pointer(decode_model.c), pm, d2p, p2d, lq, len(local_queue), rq_ptrs, rlen.ctypes.data)
    costs = np.full(n + 1, np.nan)
    reason = ctypes.c_int32(-1)
    r = lib.ampd_route(ctypes.byref(inp), _Task(*task), costs.ctypes.data, ctypes.byref(reason))
    if r == ROUTE_ERROR:
        raise ValueError("ampd_route rejected its input")
    return ("local" if r == ROUTE_LOCAL else int(r)), (costs.tolist() if reason.value == 2 else None), reason.value


def reorder(window, w, now, ttft_thres):
    """Algorithm 2.  window: list of (t_pre, enqueue_time, postponed).  Returns (ordering, counters, S)."""
    n = len(window)
    arr = (_QTask * max(n, 1))(*[_QTask(t, e, p, 0) for t, e, p in window])
    perm = np.zeros(max(n, 1), dtype=np.int32)
    post = np.zeros(max(n, 1), dtype=np.int32)
    s = ctypes.c_int32(0)
    rc = lib.ampd_reorder(arr, n, w, now, ttft_thres, perm.ctypes.data, post.ctypes.data, ctypes.byref(s))
    if rc != 0:
        raise ValueError("ampd_reorder rejected its input")
    return perm[:n].tolist(), post[:n].tolist(), int(s.value)
