"""Adaptive routing (paper Algorithm 1, Eq. 1-2) and prefill reordering (Algorithm 2, Eq. 3-4): pins of the
Python reference against hand-worked cases, then the C library against the reference.  CPU only."""
import itertools

import numpy as np
import pytest

from oracle import sched_reference as R
from paper_2602_14516_amd import sched as S

M_FAST = ([16.0, 1024.0], [1e-3, 2e-3], [1e-6, 4e-6])      # T_pre lines: alpha + beta * l_hist per l_incr bucket
M_SLOW = ([16.0, 1024.0], [2e-3, 4e-3], [2e-6, 8e-6])


# ---- pins of the reference ----------------------------------------------------------------------------

def test_t_pre_model_interpolates_in_log_l_incr():
    assert R.t_pre(M_FAST, 1000, 16) == pytest.approx(1e-3 + 1e-3)
    assert R.t_pre(M_FAST, 1000, 1024) == pytest.approx(2e-3 + 4e-3)
    assert R.t_pre(M_FAST, 1000, 128) == pytest.approx(0.5 * (2e-3 + 6e-3))       # 128 is the log-midpoint of 16 and 1024
    assert R.t_pre(M_FAST, 1000, 4) == R.t_pre(M_FAST, 1000, 16) and R.t_pre(M_FAST, 0, 9999) == pytest.approx(2e-3)


def test_routing_three_branches_by_hand():
    kw = dict(ttft_thres=1.0, itl_thres=0.05, alpha=0.9, beta=0.85, decode_model=M_SLOW, prefill_models=[M_FAST, M_FAST],
              kv_d2p=[(1e-3, 1e-6), (1e-3, 1e-6)], kv_p2d=[(1e-3, 1e-6), (1e-3, 1e-6)], local_queue=[], remote_queues=[[], []])
    # worker 1 has TTFT slack (0.5 <= 0.9); visiting order 1,0 returns 1; order 0,1 also 1 because 0 has none
    assert R.route((1000, 16), [0.95, 0.5], 0.06, visit_order=[1, 0], **kw)[0] == 1
    assert R.route((1000, 16), [0.95, 0.5], 0.06, visit_order=[0, 1], **kw)[0] == 1
    # both have slack: the random order decides
    assert R.route((1000, 16), [0.2, 0.5], 0.06, visit_order=[1, 0], **kw)[0] == 1
    assert R.route((1000, 16), [0.2, 0.5], 0.06, visit_order=[0, 1], **kw)[0] == 0
    # nobody has TTFT slack, decode worker has ITL slack (0.04 <= 0.0425): local
    assert R.route((1000, 16), [0.95, 0.99], 0.04, visit_order=[0, 1], **kw)[0] == "local"
    # no slack anywhere: cost comparison.  local = 2e-3 + 2e-6*1000 = 4e-3;
    # remote_i = (1e-3 + 1e-6*1000) + (1e-3 + 1e-6*1000) + (1e-3 + 1e-6*16) = 5.016e-3  -> local
    r, costs = R.route((1000, 16), [0.95, 0.99], 0.06, visit_order=[0, 1], **kw)
    assert r == "local" and costs == pytest.approx([4e-3, 5.016e-3, 5.016e-3])
    # a queue on the decode worker (Eq. 1, second term) tips it to remote; the longer remote queue loses
    kw2 = dict(kw, local_queue=[(500, 16)], remote_queues=[[(0, 16)], []])
    r, costs = R.route((1000, 16), [0.95, 0.99], 0.06, visit_order=[0, 1], **kw2)
    assert costs == pytest.approx([4e-3 + 3e-3, 5.016e-3 + 1e-3, 5.016e-3]) and r == 1


def test_reordering_by_hand():
    # A: long and relaxed, B: short and close to its deadline.  FIFO satisfies only A; B-first satisfies both.
    window = [(0.5, 0.0, 0), (0.1, 0.0, 0)]                    # (t_pre, enqueue time, postponed)
    order, counters, s = R.reorder(window, w=3, now=0.35, ttft_thres=1.0)
    # FIFO: A done at 0.5 -> 0.85 ok; B at 0.6 -> 0.95 ok: both fine already -> identity kept (first best)
    assert order == [0, 1] and s == 2 and counters == [0, 0]
    order, counters, s = R.reorder(window, w=3, now=0.45, ttft_thres=1.0)
    # FIFO: A 0.95 ok, B 0.45+0.6 = 1.05 late -> S=1;  B first: B 0.55 ok, A 0.45+0.6 = 1.05 late -> S=1: tie -> identity
    assert order == [0, 1] and s == 1
    window = [(0.5, 0.3, 0), (0.1, 0.0, 0)]                    # A arrived later, so it has more room
    order, counters, s = R.reorder(window, w=3, now=0.45, ttft_thres=1.0)
    # FIFO: A 0.15+0.5 ok, B 0.45+0.6 late -> 1;  B first: B 0.55 ok, A 0.15+0.6 ok -> 2
    assert order == [1, 0] and s == 2 and counters == [1, 0]
    # once A's postponement counter is exhausted the swap is forbidden
    window = [(0.5, 0.3, 3), (0.1, 0.0, 0)]
    order, counters, s = R.reorder(window, w=3, now=0.45, ttft_thres=1.0)
    assert order == [0, 1] and s == 1 and counters == [3, 0]
    assert R.reorder([], 3, 0.0, 1.0) == ([], [], 0)


def test_reference_reordering_is_optimal_and_respects_caps():
    # 200 random windows against an enumeration written out here: count the TTFT-satisfying tasks of every ordering
    # that moves no task with an exhausted counter backwards; the result must reach the best count, be feasible
    # itself, be the identity when the identity is already best, and raise exactly the counters of the tasks it moved back
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(1, 6)); w = int(rng.integers(n, 6))
        window = [(float(rng.uniform(0.01, 0.5)), float(rng.uniform(-1, 0)), int(rng.integers(0, w + 1))) for _ in range(n)]
        thres = float(rng.uniform(0.3, 1.5))
        order, counters, s = R.reorder(window, w, 0.0, thres)

        def count(p):
            t, cnt = 0.0, 0
            for r in p:
                t += window[r][0]
                cnt += (0.0 - window[r][1]) + t <= thres
            return cnt

        def feasible(p):
            return all(not (pos > r and window[r][2] >= w) for pos, r in enumerate(p))

        best = max(count(p) for p in itertools.permutations(range(n)) if feasible(p))
        assert sorted(order) == list(range(n)) and feasible(order)
        assert s == best == count(order)
        if count(tuple(range(n))) == best:
            assert order == list(range(n))
        assert counters == [window[i][2] + (order.index(i) > i) for i in range(n)]
    # independent exhaustive check on a fixed instance: S of the result equals the max over feasible orders
    window = [(0.3, -0.2, 0), (0.2, -0.5, 2), (0.1, -0.6, 0), (0.25, -0.1, 1)]
    order, counters, s = R.reorder(window, 4, 0.0, 0.8)
    best = 0
    for p in itertools.permutations(range(4)):
        t, cnt = 0.0, 0
        for r in p:
            t += window[r][0]
            cnt += (0.0 - window[r][1]) + t <= 0.8
        best = max(best, cnt)
    assert s == best and sorted(order) == [0, 1, 2, 3]
    assert all(c == window[i][2] + (order.index(i) > i) for i, c in enumerate(counters))


# ---- the C library against the reference -------------------------------------------------------------

def test_library_loads_and_exports_symbols():
    import os, re
    hdr = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "ampd_sched.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ampd_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(S.SCHED_SYMBOLS)
    for name in S.SCHED_SYMBOLS:
        assert hasattr(S.lib, name)


def test_decision_cost_is_far_below_a_millisecond():
    # the paper reports 0.39 ms / 0.45 ms per routing / reordering decision on its CPU (Section 6.4);
    # here a window of 5 (120 orderings) including the Python call overhead
    import time
    window = [(0.1 * (i + 1), -0.1 * i, 0) for i in range(5)]
    t0 = time.perf_counter()
    for _ in range(200):
        S.reorder(window, 5, 0.0, 1.0)
    assert (time.perf_counter() - t0) / 200 < 1e-3


def test_c_t_pre_matches_reference():
    m = S.TPreModel(*M_FAST)
    for lh, li in [(0, 1), (1000, 16), (1000, 128), (77, 500), (5000, 4096), (3, 1024)]:
        assert S.t_pre(m, lh, li) == pytest.approx(R.t_pre(M_FAST, lh, li), rel=1e-12)


def test_c_routing_matches_reference_on_random_instances():
    rng = np.random.default_rng(1)
    models = [M_FAST, M_SLOW, ([64.0], [5e-4], [3e-6])]
    for trial in range(300):
        n = int(rng.integers(0, 4))
        pm = [models[int(rng.integers(3))] for _ in range(n)]
        dm = models[int(rng.integers(3))]
        args = dict(task=(int(rng.integers(0, 20000)), int(rng.integers(1, 5000))),
                    ttft_hat=rng.uniform(0.5, 1.5, n).tolist(), itl_hat=float(rng.uniform(0.02, 0.08)),
                    ttft_thres=1.0, itl_thres=0.05, alpha=0.9, beta=0.85, visit_order=rng.permutation(n).tolist(),
                    kv_d2p=[(float(rng.uniform(0, 2e-3)), float(rng.uniform(0, 2e-6))) for _ in range(n)],
                    kv_p2d=[(float(rng.uniform(0, 2e-3)), float(rng.uniform(0, 2e-6))) for _ in range(n)],
                    local_queue=[(int(rng.integers(0, 9000)), int(rng.integers(1, 3000))) for _ in range(int(rng.integers(0, 4)))],
                    remote_queues=[[(int(rng.integers(0, 9000)), int(rng.integers(1, 3000))) for _ in range(int(rng.integers(0, 5)))] for _ in range(n)])
        want, wcosts = R.route(decode_model=dm, prefill_models=pm, **args)
        got, gcosts, reason = S.route(decode_model=S.TPreModel(*dm), prefill_models=[S.TPreModel(*m) for m in pm], **args)
        assert got == want, (trial, got, want)
        if wcosts is not None:
            assert gcosts == pytest.approx(wcosts, rel=1e-12) and reason == 2


def test_c_reordering_matches_reference_on_random_instances():
    rng = np.random.default_rng(2)
    for trial in range(500):
        w = int(rng.integers(1, 7)); n = int(rng.integers(0, w + 1))
        window = [(float(rng.uniform(0.01, 0.5)), float(rng.uniform(-1, 0)), int(rng.integers(0, w + 1))) for _ in range(n)]
        thres = float(rng.uniform(0.3, 1.5))
        assert S.reorder(window, w, 0.0, thres) == tuple(R.reorder(window, w, 0.0, thres)), trial
    with pytest.raises(ValueError):
        S.reorder([(0.1, 0.0, 0)] * 3, 2, 0.0, 1.0)              # window longer than w
