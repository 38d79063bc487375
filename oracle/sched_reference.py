"""TEST INFRASTRUCTURE -- not the product.

Plain Python statements of the two scheduling decisions, in the paper's notation:
adaptive routing (paper Section 4.1, Algorithm 1, Eq. 1 and Eq. 2) and prefill reordering
(Section 4.2, Algorithm 2, Eq. 3 and Eq. 4).  Brute force over all orderings; nothing is
optimised.  Readings where the paper leaves a choice open (tie-breaks, what "postponed"
means) are listed in include/ampd_sched.h and repeated here where they are applied.

Pinned by tests/test_sched.py: hand-worked examples, the no-reordering and no-slack special
cases, and optimality against an independent exhaustive count.
"""
from __future__ import annotations

import itertools
import math


def t_pre(model, l_hist, l_incr):
    """model = (l_incr buckets, alpha, beta): one line in l_hist per bucket, interpolated in log(l_incr)."""
    bs, al, be = model
    q = math.log(max(l_incr, 1e-30))
    hi = 0
    while hi < len(bs) and math.log(bs[hi]) < q:
        hi += 1
    if hi == 0:
        return al[0] + be[0] * l_hist
    if hi == len(bs):
        return al[-1] + be[-1] * l_hist
    lo = hi - 1
    a, b = math.log(bs[lo]), math.log(bs[hi])
    w = (q - a) / (b - a) if b > a else 0.0
    return (1 - w) * (al[lo] + be[lo] * l_hist) + w * (al[hi] + be[hi] * l_hist)


def route(task, ttft_hat, itl_hat, ttft_thres, itl_thres, alpha, beta, visit_order,
          decode_model, prefill_models, kv_d2p, kv_p2d, local_queue, remote_queues):
    """Returns (route, costs): route = 'local' or the index of a prefill worker."""
    for i in visit_order:                                        # a prefill worker with TTFT slack
        if ttft_hat[i] <= alpha * ttft_thres:
            return i, None
    if itl_hat <= beta * itl_thres:                              # the decode worker has ITL slack
        return "local", None
    l_hist, l_incr = task
    t_local = t_pre(decode_model, l_hist, l_incr) + sum(t_pre(decode_model, h, n) for h, n in local_queue)      # Eq. 1
    costs = [t_local]
    for i, m in enumerate(prefill_models):                       # Eq. 2
        t = t_pre(m, l_hist, l_incr)
        t += kv_d2p[i][0] + kv_d2p[i][1] * l_hist
        t += kv_p2d[i][0] + kv_p2d[i][1] * l_incr
        t += sum(t_pre(m, h, n) for h, n in remote_queues[i])
        costs.append(t)
    best = min(range(len(costs)), key=lambda j: (costs[j], j))   # ties: local first, then lower index
    return ("local" if best == 0 else best - 1), costs


def satisfied_count(order, window, now, ttft_thres):
    """Eq. 3 and Eq. 4 for one ordering (a sequence of window indices)."""
    c, s = 0.0, 0
    for r in order:
        c += window[r][0]                                        # C^(pi(k)) = sum of t_pre up to k
        if (now - window[r][1]) + c <= ttft_thres:
            s += 1
    return s


def reorder(window, w, now, ttft_thres):
    """window: list of (t_pre, enqueue_time, postponed) in queue order, len <= w.
    Returns (ordering, updated counters, S of the ordering)."""
    n = len(window)
    best, best_s = None, None
    for order in itertools.permutations(range(n)):               # lexicographic, identity first
        if any(k > r and window[r][2] >= w for k, r in enumerate(order)):
            continue                                             # would postpone a task whose counter is exhausted
        s = satisfied_count(order, window, now, ttft_thres)
        if best is None or s > best_s:
            best, best_s = order, s
    counters = [t[2] for t in window]
    for k, r in enumerate(best):
        if k > r:
            counters[r] += 1
    return list(best), counters, best_s
