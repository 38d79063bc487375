"""Discrete-event simulator of multi-round serving on a prefill / decode disaggregated deployment, driven by
the cost model of the attention path and by the two scheduling decisions of libampd_sched (host only).

What is simulated (paper Section 3: workflow of a multi-round request; Section 4.1: adaptive routing, Algorithm 1;
Section 4.2: prefill reordering, Algorithm 2):

* a session is a sequence of rounds; round r appends ``l_incr`` tokens (tool or retrieval output; the first round is
  the initial prefill, history 0) to the session's context, then decodes ``n_dec`` tokens, then waits for a tool;
* every session is bound to one decode worker, which holds all of its KV;
* a prefill task either runs **locally** on that decode worker (it takes the worker before the next decode step, so
  the worker's decode rows stall for its duration) or **remotely** on a prefill worker (history KV travels decode ->
  prefill first, the incremental KV travels back afterwards; the decode rows do not stall);
* a decode worker advances all of its active sessions by one token per step, the step costing T_dec(b, sum C);
* the first token of a round is produced when its prefill finishes: TTFT = that time - arrival of the round; ITL
  samples are the gaps between consecutive tokens of a session within a round.

Readings of what the paper leaves open: the windowed TTFT / ITL statistics that Algorithm 1 consults are the means of
the last ``stat_window`` samples of that worker (0 before the first sample); the always-remote baseline sends a task
to the prefill worker with the least estimated backlog; a decode worker serves its local prefill queue before
decoding (prefill priority); tool delays are exponential with a given mean.

The cost model is that of ONE attention layer as measured on the device; ``layers`` scales it to a stack, and
``other_s_per_token`` adds a per-token cost for everything that is not attention (0 by default: attention only).
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field

import numpy as np

from . import sched
from .perf_model import AlphaBetaFamily


@dataclass
class CostModel:
    """T_pre(l_hist; l_incr) and T_dec(sum C; b) as alpha-beta families (seconds), T_kv(tokens) = alpha + beta * tokens."""
    tpre_l_incr: np.ndarray
    tpre_alpha: np.ndarray
    tpre_beta: np.ndarray
    tdec_b: np.ndarray
    tdec_alpha: np.ndarray
    tdec_beta: np.ndarray
    kv_alpha: float = 20e-6                  # per transfer: pack + unpack launches and the link's latency
    kv_beta: float = 4096 / 100e9            # per token and layer: pack + unpack + bytes of K and V / link bandwidth
    layers: int = 32
    other_s_per_token: float = 0.0
    prefill_speed: float = 1.0               # prefill workers relative to the decode worker's device

    def __post_init__(self):
        self._tpre = sched.TPreModel(self.tpre_l_incr, self.tpre_alpha, self.tpre_beta)
        self._tpre_p = sched.TPreModel(self.tpre_l_incr, np.asarray(self.tpre_alpha) / self.prefill_speed,
                                       np.asarray(self.tpre_beta) / self.prefill_speed)
        self._tdec = AlphaBetaFamily(np.asarray(self.tdec_b, float), np.asarray(self.tdec_alpha, float),
                                     np.asarray(self.tdec_beta, float))

    # whole-stack times
    def t_pre(self, l_hist: int, l_incr: int, remote: bool) -> float:
        one = sched.t_pre(self._tpre_p if remote else self._tpre, l_hist, l_incr)
        other = self.other_s_per_token * l_incr / (self.prefill_speed if remote else 1.0)
        return self.layers * one + other

    def t_dec(self, b: int, sum_ctx: int) -> float:
        return self.layers * float(self._tdec(b, sum_ctx)[0]) + self.other_s_per_token * b

    def t_kv(self, tokens: int) -> float:
        return 0.0 if tokens <= 0 else self.kv_alpha + self.layers * self.kv_beta * tokens

    # what Algorithm 1 is given: per-layer lines scaled to the stack
    def sched_models(self):
        scale = lambda m, s: sched.TPreModel(m.a[0], m.a[1] * self.layers / s, m.a[2] * self.layers / s)
        return scale(self._tpre, 1.0), scale(self._tpre, self.prefill_speed)


# One MI355X, one attention layer (T_pre: Hq=32 Hkv=8 d=128; T_dec: Hq=64 Hkv=8 d=128; bf16 cache): the lines fitted by
# `bench.py --only model` to whole C-ABI calls, and T_kv as pack + wire + unpack with the two GPU halves fitted from
# ampd_kv_pack / ampd_kv_unpack timings.  The numbers live in mi355x_cost_model.json, which
# `python -m paper_2602_14516_amd.perf_model <sweep output>` writes; nothing is typed in by hand.
def mi355x_attention() -> dict:
    from .perf_model import load_cost_model
    m = load_cost_model()
    return dict(tpre_l_incr=np.array(m["tpre_l_incr"]), tpre_alpha=np.array(m["tpre_alpha"]), tpre_beta=np.array(m["tpre_beta"]),
                tdec_b=np.array(m["tdec_b"]), tdec_alpha=np.array(m["tdec_alpha"]), tdec_beta=np.array(m["tdec_beta"]),
                kv_alpha=float(m["kv_alpha"]), kv_beta=float(m["kv_beta"]))


MI355X_ATTENTION = mi355x_attention()


@dataclass
class Round:
    l_incr: int
    n_dec: int
    tool_delay: float


@dataclass
class _Task:
    session: int
    l_hist: int
    l_incr: int
    arrival: float
    postponed: int = 0
    worker: int = -1          # prefill worker, or -1 for local
    first_token: float = 0.0  # when the prefill finished


@dataclass
class SimResult:
    ttft: np.ndarray
    itl: np.ndarray
    makespan: float
    routed_local: int
    routed_remote: int
    reorders: int
    ttft_attainment: float = 0.0
    itl_attainment: float = 0.0
    per_worker_busy: dict = field(default_factory=dict)

    def summary(self) -> dict:
        q = lambda a, p: float(np.percentile(a, p)) if len(a) else 0.0
        return {"ttft_attainment": self.ttft_attainment, "itl_attainment": self.itl_attainment,
                "ttft_p50_s": q(self.ttft, 50), "ttft_p99_s": q(self.ttft, 99), "itl_p50_s": q(self.itl, 50),
                "itl_p99_s": q(self.itl, 99), "makespan_s": self.makespan, "routed_local": self.routed_local,
                "routed_remote": self.routed_remote, "reorders": self.reorders}


def make_sessions(seed: int, num_sessions: int = 64, rounds: int = 8, median: float = 512.0, sigma: float = 1.0,
                  lo: int = 16, hi: int = 8192, dec_lo: int = 64, dec_hi: int = 256, tool_delay_mean: float = 0.2,
                  arrival_span: float = 1.0):
    """Sessions with the length distributions of the multi-round trace configuration: lognormal incremental lengths,
    uniform decode lengths, exponential tool delays; session start times uniform in [0, arrival_span)."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 300])))
    L = np.clip(np.rint(np.exp(g.normal(np.log(median), sigma, size=(num_sessions, rounds)))), lo, hi).astype(int)
    D = g.integers(dec_lo, dec_hi, size=(num_sessions, rounds), endpoint=True)
    T = g.exponential(tool_delay_mean, size=(num_sessions, rounds))
    starts = np.sort(g.uniform(0.0, arrival_span, size=num_sessions))
    return [(float(starts[s]), [Round(int(L[s, r]), int(D[s, r]), float(T[s, r])) for r in range(rounds)])
            for s in range(num_sessions)]


def simulate(sessions, model: CostModel, *, n_prefill: int, n_decode: int, policy: str = "adaptive",
             reorder_window: int = 0, ttft_thres: float = 0.5, itl_thres: float = 0.05, alpha: float = 0.9,
             beta: float = 0.85, stat_window: int = 32, seed: int = 0) -> SimResult:
    """policy: 'adaptive' (Algorithm 1), 'remote' (always a prefill worker), 'local' (always the decode worker).
    reorder_window: 0 = first come first served; w >= 2 = Algorithm 2 over the first w queued tasks."""
    assert policy in ("adaptive", "remote", "local") and n_decode >= 1
    assert policy != "remote" or n_prefill >= 1
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 301])))
    m_dec, m_pre = model.sched_models()
    kv_line = (model.kv_alpha, model.layers * model.kv_beta)

    events = []                                   # (time, sequence number, kind, payload)
    seq = [0]

    def push(t, kind, payload):
        heapq.heappush(events, (t, seq[0], kind, payload))
        seq[0] += 1

    ctx = [0] * len(sessions)                     # tokens of context held by the decode worker
    next_round = [0] * len(sessions)
    p_queue = [[] for _ in range(n_prefill)]
    p_busy = [False] * n_prefill
    p_ttft = [[] for _ in range(n_prefill)]
    d_queue = [[] for _ in range(n_decode)]
    d_busy = [False] * n_decode
    d_active = [dict() for _ in range(n_decode)]  # session -> [remaining tokens, time of last token]
    d_itl = [[] for _ in range(n_decode)]
    busy_time = {("p", i): 0.0 for i in range(n_prefill)}
    busy_time.update({("d", i): 0.0 for i in range(n_decode)})
    ttft_all, itl_all = [], []
    counts = {"local": 0, "remote": 0, "reorders": 0}
    now = 0.0

    def mean_tail(xs):
        return float(np.mean(xs[-stat_window:])) if xs else 0.0

    def pick(queue, worker_is_remote):
        """Next task of a queue: first come first served, or Algorithm 2 over the head window."""
        if reorder_window < 2 or len(queue) < 2:
            return queue.pop(0)
        w = min(reorder_window, sched.MAX_WINDOW)
        head = queue[:w]
        window = [(model.t_pre(t.l_hist, t.l_incr, worker_is_remote), t.arrival, t.postponed) for t in head]
        perm, post, _ = sched.reorder(window, w, now, ttft_thres)
        for t, pcount in zip(head, post):
            t.postponed = pcount
        if perm[0] != 0:
            counts["reorders"] += 1
        return queue.pop(perm[0])

    def kick_prefill(i):
        if p_busy[i] or not p_queue[i]:
            return
        t = pick(p_queue[i], True)
        dur = model.t_pre(t.l_hist, t.l_incr, True)
        p_busy[i] = True
        busy_time[("p", i)] += dur
        push(now + dur, "p_done", t)

    def kick_decode(j):
        if d_busy[j]:
            return
        if d_queue[j]:
            t = pick(d_queue[j], False)
            dur = model.t_pre(t.l_hist, t.l_incr, False)
            d_busy[j] = True
            busy_time[("d", j)] += dur
            push(now + dur, "d_prefill_done", t)
        elif d_active[j]:
            members = list(d_active[j].keys())
            dur = model.t_dec(len(members), sum(ctx[s] for s in members))
            d_busy[j] = True
            busy_time[("d", j)] += dur
            push(now + dur, "d_step_done", (j, members))

    def route(t: _Task, j: int):
        if policy == "local" or n_prefill == 0:
            return "local"
        if policy == "remote":
            backlog = [sum(model.t_pre(x.l_hist, x.l_incr, True) for x in p_queue[i]) + (1e-9 if p_busy[i] else 0.0)
                       for i in range(n_prefill)]
            return int(np.argmin(backlog))
        r, _, _ = sched.route((t.l_hist, t.l_incr), [mean_tail(x) for x in p_ttft], mean_tail(d_itl[j]), ttft_thres,
                              itl_thres, alpha, beta, rng.permutation(n_prefill), m_dec, [m_pre] * n_prefill,
                              [kv_line] * n_prefill, [kv_line] * n_prefill,
                              [(x.l_hist, x.l_incr) for x in d_queue[j]],
                              [[(x.l_hist, x.l_incr) for x in q] for q in p_queue])
        return r

    for s, (start, _) in enumerate(sessions):
        push(start, "arrive", s)

    while events:
        now, _, kind, payload = heapq.heappop(events)
        if kind == "arrive":
            s = payload
            rnd = sessions[s][1][next_round[s]]
            j = s % n_decode
            t = _Task(s, ctx[s], rnd.l_incr, now)
            r = route(t, j)
            if r == "local":
                counts["local"] += 1
                d_queue[j].append(t)
                kick_decode(j)
            else:
                counts["remote"] += 1
                t.worker = r
                push(now + model.t_kv(t.l_hist), "p_enqueue", t)       # history KV: decode -> prefill worker
        elif kind == "p_enqueue":
            t = payload
            p_queue[t.worker].append(t)
            kick_prefill(t.worker)
        elif kind == "p_done":
            t = payload
            p_busy[t.worker] = False
            ttft = now - t.arrival
            t.first_token = now
            ttft_all.append(ttft)
            p_ttft[t.worker].append(ttft)
            push(now + model.t_kv(t.l_incr), "join", t)                 # incremental KV: prefill -> decode worker
            kick_prefill(t.worker)
        elif kind == "d_prefill_done":
            t = payload
            j = t.session % n_decode
            d_busy[j] = False
            t.first_token = now
            ttft_all.append(now - t.arrival)
            push(now, "join", t)
        elif kind == "join":
            t = payload
            s, j = t.session, t.session % n_decode
            ctx[s] += t.l_incr
            rnd = sessions[s][1][next_round[s]]
            d_active[j][s] = [rnd.n_dec, t.first_token]
            kick_decode(j)
        elif kind == "d_step_done":
            j, members = payload
            d_busy[j] = False
            for s in members:
                st = d_active[j][s]
                gap = now - st[1]
                itl_all.append(gap)
                d_itl[j].append(gap)
                st[1] = now
                st[0] -= 1
                ctx[s] += 1
                if st[0] == 0:
                    del d_active[j][s]
                    rnd = sessions[s][1][next_round[s]]
                    next_round[s] += 1
                    if next_round[s] < len(sessions[s][1]):
                        push(now + rnd.tool_delay, "arrive", s)
            kick_decode(j)

    ttft_a, itl_a = np.array(ttft_all), np.array(itl_all)
    res = SimResult(ttft_a, itl_a, now, counts["local"], counts["remote"], counts["reorders"])
    res.ttft_attainment = float(np.mean(ttft_a <= ttft_thres)) if len(ttft_a) else 1.0
    res.itl_attainment = float(np.mean(itl_a <= itl_thres)) if len(itl_a) else 1.0
    res.per_worker_busy = {f"{k}{i}": v / now if now > 0 else 0.0 for (k, i), v in busy_time.items()}
    return res
