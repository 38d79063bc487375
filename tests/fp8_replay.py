"""Replay of a multi-round session trace (benchmark configuration 5) through one persistent 8-bit page pool, with
the oracle's mirrors kept in lock-step on the host.  The GPU side is a callable, so that the bookkeeping can be
exercised without a GPU; the GPU tests pass the C-ABI call.

Host state per session (preallocated for the session's final length, fp64): the unquantised history K/V (what the
oracle for the stated 8-bit tolerance reads) and the dequantised cache contents (what the oracle for the kernel's own
error reads); the latter is refreshed for the pages a tick touched, since an append may re-encode the old slots of
a partly filled page.
"""
import numpy as np

import oracle
import workloads as W
from gpu_util import Fp8UnquantisedCheck, TOL_BF16


class HostMirror:
    """Codes and scales of the whole pool as the oracle's append reference leaves them, plus fp64 histories."""

    def __init__(self, tr, poison=True):
        shape = (tr.num_pages, tr.Hkv, tr.P, tr.d)
        fill = 0x7F if poison else 0                              # 0x7F decodes to NaN
        self.k = np.full(shape, fill, np.uint8)
        self.v = np.full(shape, fill, np.uint8)
        self.ks = np.full((tr.num_pages, tr.Hkv), np.nan if poison else 1.0, np.float32)
        self.vs = self.ks.copy()
        final = np.zeros(tr.num_sessions, np.int64)
        for tk in tr.ticks:
            np.maximum.at(final, tk.sessions, tk.ctx_len.astype(np.int64) + tk.incr_len)
        mk = lambda n: np.zeros((int(n), tr.Hkv, tr.d), np.float64)
        self.K = [mk(n) for n in final]                           # unquantised
        self.V = [mk(n) for n in final]
        self.Kd = [mk(n) for n in final]                          # dequantised cache contents
        self.Vd = [mk(n) for n in final]
        self.P = tr.P

    def append(self, tk, bt, k_bits, v_bits):
        oracle.fp8_append_reference(self.k, self.ks, bt, tk.ctx_len, tk.incr_len, k_bits, self.P, in_place=True)
        oracle.fp8_append_reference(self.v, self.vs, bt, tk.ctx_len, tk.incr_len, v_bits, self.P, in_place=True)
        off = np.concatenate([[0], np.cumsum(tk.incr_len)])
        P = self.P
        for i, s in enumerate(tk.sessions):
            C, L = int(tk.ctx_len[i]), int(tk.incr_len[i])
            self.K[s][C:C + L] = W.bf16_bits_to_f64(k_bits[off[i]:off[i + 1]])
            self.V[s][C:C + L] = W.bf16_bits_to_f64(v_bits[off[i]:off[i + 1]])
            lp0 = C // P                                          # first page this append touched
            t0, n = lp0 * P, C + L - lp0 * P
            self.Kd[s][t0:C + L] = oracle.fp8_dequant_request(self.k, self.ks, bt[i, lp0:], n, P)
            self.Vd[s][t0:C + L] = oracle.fp8_dequant_request(self.v, self.vs, bt[i, lp0:], n, P)


def replay_trace(tr, run_tick, fetch, *, decode_tick_fraction=0.05, prefill_rows=6, decode_rows_per_tick=3, seed=55,
                 progress_every=200, got_fn=None):
    """run_tick(t, tk, bt, q, k, v) enqueues the call of tick t and returns a handle; fetch(handle) -> bf16 bits
    [sum L, Hq, d] on the host.  All prefill ticks and a seeded fraction of the decode-only ticks are checked: every
    prefill row on sampled query positions, and a few sampled decode rows of the tick.  got_fn (CPU rehearsal of the
    bookkeeping only): stands in for the fetched output of the sampled rows.  Returns (mirror, report)."""
    Hq, Hkv, d, P = tr.Hq, tr.Hkv, tr.d, tr.P
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(d)
    mir = HostMirror(tr)
    rng = np.random.default_rng(seed)
    unq = Fp8UnquantisedCheck()
    deq_max, deq_sum, deq_n = 0.0, 0.0, 0
    checked_ticks = checked_rows = 0
    for t, tk in enumerate(tr.ticks):
        q, k, v = W.draw_tick_tensors(tr, t)
        bt = tr.tick_block_table(t)
        mir.append(tk, bt, k, v)
        handle = run_tick(t, tk, bt, q, k, v)
        is_prefill_tick = bool((tk.incr_len > 1).any())
        if is_prefill_tick or rng.random() < decode_tick_fraction:
            ob = fetch(handle) if got_fn is None else None
            off = np.concatenate([[0], np.cumsum(tk.incr_len)])
            dec = np.nonzero(tk.incr_len == 1)[0]
            pick = list(np.nonzero(tk.incr_len > 1)[0])
            if len(dec):
                pick += list(rng.choice(dec, size=min(decode_rows_per_tick, len(dec)), replace=False))
            for i in pick:
                s, C, L = int(tk.sessions[i]), int(tk.ctx_len[i]), int(tk.incr_len[i])
                rows = np.arange(L) if L <= prefill_rows + 2 else np.unique(np.concatenate([[0, L - 1], rng.integers(0, L, prefill_rows)]))
                rows = rows.astype(np.int32)
                qf = W.bf16_bits_to_f64(q[off[i]:off[i + 1]])
                ref_d = oracle.attn_oracle_request(qf, mir.Kd[s][:C + L], mir.Vd[s][:C + L], C, L, scale, rows=rows)
                got = W.bf16_bits_to_f64(ob[off[i]:off[i + 1]])[rows] if got_fn is None else got_fn(ref_d)
                ed = np.abs(got - ref_d)
                assert np.isfinite(ed).all(), f"tick {t} session {s}: non-finite output"
                assert ed.max() <= TOL_BF16[0], f"tick {t} session {s}: {ed.max():.3e} against the dequantised cache"
                deq_max = max(deq_max, float(ed.max())); deq_sum += float(ed.sum()); deq_n += ed.size
                ref_u = oracle.attn_oracle_request(qf, mir.K[s][:C + L], mir.V[s][:C + L], C, L, scale, rows=rows)
                unq.add(got, ref_u, mir.V[s][:C + L], C, rows, G, label=f"tick {t} session {s}")
                checked_rows += len(rows)
            checked_ticks += 1
        if progress_every and t % progress_every == 0:
            print(f"  tick {t} / {len(tr.ticks)}: {checked_ticks} ticks, {checked_rows} query positions checked", flush=True)
    deq_mean = deq_sum / max(deq_n, 1)
    assert deq_mean <= TOL_BF16[1], f"mean-abs {deq_mean:.3e} against the dequantised cache"
    report = (f"{len(tr.ticks)} ticks, {checked_ticks} checked ({checked_rows} query positions x {Hq} heads); "
              f"against the dequantised cache: max-abs {deq_max:.2e} mean-abs {deq_mean:.2e}; against unquantised inputs: "
              + unq.finish("trace replay"))
    return mir, report
