"""Multi-round session trace (benchmark configuration 5): a deterministic replay schedule.

Every session alternates "append a tool output of L tokens" (an incremental prefill; the
first round has no history, i.e. an initial prefill) with D single-token decode steps, as
in the interleaved prefill/decode pattern of multi-round inference (paper Section 1 and
Section 3, steps 2-4).  All sessions advance in lock-step ticks; at every tick each active
session contributes one row to one mixed batch, which is how a decode instance that
executes incremental prefills locally sees them (paper Section 3, "Local execution").

The module only draws lengths, hands out pages from a free list and draws per-tick tensors;
it contains none of the attention / append / quantisation arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from .batches import f32_to_bf16_bits


@dataclass
class Tick:
    sessions: np.ndarray      # int32 [n] session id of each row
    ctx_len: np.ndarray       # int32 [n]
    incr_len: np.ndarray      # int32 [n]


@dataclass
class SessionTrace:
    Hq: int
    Hkv: int
    d: int
    P: int
    seed: int
    num_sessions: int
    ticks: list = field(default_factory=list)
    block_table: np.ndarray = None      # int32 [num_sessions, max_pages]: final table, pages in order of allocation
    num_pages: int = 0

    def tick_block_table(self, t: int) -> np.ndarray:
        """Block-table rows of tick t (a view of the final table: pages are never moved)."""
        return np.ascontiguousarray(self.block_table[self.ticks[t].sessions])


def make_trace_schedule(seed: int, *, num_sessions=32, rounds=8, Hq=32, Hkv=8, d=128, P=16,
                        median=512.0, sigma=1.0, lo=16, hi=8192, dec_lo=64, dec_hi=256,
                        stagger=8, pool_slack=0.10) -> SessionTrace:
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 200])))
    L = np.clip(np.rint(np.exp(g.normal(np.log(median), sigma, size=(num_sessions, rounds)))), lo, hi).astype(np.int64)
    D = g.integers(dec_lo, dec_hi, size=(num_sessions, rounds), endpoint=True)
    # per-session list of (L) per tick
    seqs = []
    for s in range(num_sessions):
        steps = [0] * (s % stagger)          # 0 = idle tick (staggered start)
        for r in range(rounds):
            steps.append(int(L[s, r]))
            steps.extend([1] * int(D[s, r]))
        seqs.append(steps)
    nticks = max(len(x) for x in seqs)
    final_tokens = np.array([sum(x) for x in seqs], dtype=np.int64)
    pages_final = (final_tokens + P - 1) // P
    num_pages = int(np.ceil(pages_final.sum() * (1.0 + pool_slack)))
    free = g.permutation(num_pages).astype(np.int32).tolist()      # free list in a seeded order
    max_pages = int(pages_final.max())
    bt = np.full((num_sessions, max_pages), -1, dtype=np.int32)
    have = np.zeros(num_sessions, dtype=np.int64)                 # pages owned
    ctx = np.zeros(num_sessions, dtype=np.int64)
    tr = SessionTrace(Hq, Hkv, d, P, seed, num_sessions)
    for t in range(nticks):
        ids, cs, ls = [], [], []
        for s in range(num_sessions):
            if t < len(seqs[s]) and seqs[s][t] > 0:
                l = seqs[s][t]
                need = (ctx[s] + l + P - 1) // P
                while have[s] < need:                             # allocate pages on demand
                    bt[s, have[s]] = free.pop()
                    have[s] += 1
                ids.append(s); cs.append(ctx[s]); ls.append(l)
                ctx[s] += l
        if ids:
            tr.ticks.append(Tick(np.array(ids, np.int32), np.array(cs, np.int32), np.array(ls, np.int32)))
    tr.block_table = bt
    tr.num_pages = num_pages
    return tr


def draw_tick_tensors(tr: SessionTrace, t: int):
    """q [sumL,Hq,d], k_new, v_new [sumL,Hkv,d] bf16 bits of tick t from a counter-based stream."""
    n = int(tr.ticks[t].incr_len.sum())
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([tr.seed, 300, t])))
    q = f32_to_bf16_bits(g.standard_normal((n, tr.Hq, tr.d), dtype=np.float32))
    k = f32_to_bf16_bits(g.standard_normal((n, tr.Hkv, tr.d), dtype=np.float32))
    v = f32_to_bf16_bits(g.standard_normal((n, tr.Hkv, tr.d), dtype=np.float32))
    return q, k, v
