"""GPU parity of the 8-bit KV cache: append bit-exact against the E4M3 reference, attention
against the fp64 oracle on the dequantised cache contents (2e-2 / 2e-3 on every row: the kernel's own error) and
on the unquantised inputs (6e-2 / 6e-3 on rows that see at least 256 keys, a bound derived from the rounding of V
on the others: see gpu_util.fp8_row_bounds), and replays of a multi-round session trace through one persistent
pool, reduced and at the full size of benchmark configuration 5."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_14516_amd as A
import workloads as W
from fp8_replay import replay_trace
from gpu_util import to_dev_bits, from_dev_bits, fp8_row_bounds, Fp8UnquantisedCheck, TOL_BF16, TOL_FP8

pytestmark = pytest.mark.gpu


class Fp8Pool:
    """Device pool + host mirror maintained by the oracle's append reference."""

    def __init__(self, num_pages, Hq, Hkv, d, P, scale, poison=True):
        self.shape = (num_pages, Hkv, P, d)
        fill = 0x7F if poison else 0                      # 0x7F decodes to NaN
        self.h_k = np.full(self.shape, fill, np.uint8)
        self.h_v = np.full(self.shape, fill, np.uint8)
        self.h_ks = np.full((num_pages, Hkv), np.nan if poison else 1.0, np.float32)
        self.h_vs = self.h_ks.copy()
        self.d_k = torch.from_numpy(self.h_k.copy()).cuda()
        self.d_v = torch.from_numpy(self.h_v.copy()).cuda()
        self.d_ks = torch.from_numpy(self.h_ks.copy()).cuda()
        self.d_vs = torch.from_numpy(self.h_vs.copy()).cuda()
        self.cache = A.KVCache(Hq, Hkv, d, P, self.d_k, self.d_v, scale, self.d_ks, self.d_vs, kv_dtype=1)
        self.P = P

    def reference_append(self, bt, C, L, k_new, v_new):
        self.h_k, self.h_ks = oracle.fp8_append_reference(self.h_k, self.h_ks, bt, C, L, k_new, self.P)
        self.h_v, self.h_vs = oracle.fp8_append_reference(self.h_v, self.h_vs, bt, C, L, v_new, self.P)

    def assert_equal(self):
        """the whole device image (codes and scales of every page, used or not) equals the host mirror bit for bit"""
        dk, dv = self.d_k.cpu().numpy(), self.d_v.cpu().numpy()
        dks, dvs = self.d_ks.cpu().numpy(), self.d_vs.cpu().numpy()
        assert np.array_equal(dk, self.h_k), "K codes differ"
        assert np.array_equal(dv, self.h_v), "V codes differ"
        assert np.array_equal(dks.view(np.uint32), self.h_ks.view(np.uint32)), "K scales differ"
        assert np.array_equal(dvs.view(np.uint32), self.h_vs.view(np.uint32)), "V scales differ"


def errs(got_bits, ref_list, off):
    got = W.bf16_bits_to_f64(got_bits)
    parts = []
    for r in range(len(ref_list)):
        if ref_list[r] is None or not len(ref_list[r]):
            continue
        parts.append(np.abs(got[off[r]:off[r + 1]] - ref_list[r]).ravel())
    e = np.concatenate(parts) if parts else np.zeros(1)
    assert np.isfinite(e).all()
    return float(e.max()), float(e.mean())


@pytest.mark.parametrize("name,C0,L0,L1,Hq,Hkv,d,P", [
    ("fp8-ragged", [0, 0, 0, 0], [137, 5, 264, 330], [1, 70, 9, 33], 8, 2, 128, 16),
    ("fp8-d64-p32", [0, 0], [150, 3], [20, 140], 8, 2, 64, 32),
])
def test_fp8_append_bit_exact_and_attention_within_tolerance(name, C0, L0, L1, Hq, Hkv, d, P):
    print(f"case: {name}", flush=True)
    rng = np.random.default_rng(7)
    B = len(C0)
    tot = np.array(L0) + np.array(L1)
    pages = (tot + P - 1) // P
    num_pages = int(pages.sum()) + 5
    perm = rng.permutation(num_pages).astype(np.int32)
    bt = np.full((B, int(pages.max())), -1, np.int32)
    o = 0
    for r in range(B):
        bt[r, :pages[r]] = perm[o:o + pages[r]]; o += pages[r]
    scale = 1.0 / np.sqrt(d)
    pool = Fp8Pool(num_pages, Hq, Hkv, d, P, scale)
    d_bt = torch.from_numpy(bt).cuda()
    hist_k = [np.zeros((0, Hkv, d), np.uint16) for _ in range(B)]
    hist_v = [np.zeros((0, Hkv, d), np.uint16) for _ in range(B)]
    C = np.array(C0, np.int32)
    for step, Ls in enumerate((L0, L1)):
        L = np.array(Ls, np.int32)
        n = int(L.sum())
        # a wide dynamic range so that scales differ between pages and re-encoding of old slots happens
        # (V stays at or below unit variance: the tolerances are absolute)
        mag = np.exp2(rng.integers(-3, 1, size=(n, Hkv, 1))).astype(np.float32)
        q = W.f32_to_bf16_bits(rng.standard_normal((n, Hq, d), dtype=np.float32))
        k = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d), dtype=np.float32) * mag * (1.0 + 3 * step))
        v = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d), dtype=np.float32) * mag)
        out = A.mixed_batch_attn(pool.cache, C, L, d_bt, to_dev_bits(q), to_dev_bits(k), to_dev_bits(v), block_table_host=bt)
        torch.cuda.synchronize()
        pool.reference_append(bt, C, L, k, v)
        pool.assert_equal()
        off = np.concatenate([[0], np.cumsum(L)])
        ob = from_dev_bits(out)
        got = W.bf16_bits_to_f64(ob)
        ref_deq = []
        unq, vonly = Fp8UnquantisedCheck(), 0.0
        G = Hq // Hkv
        for r in range(B):
            hist_k[r] = np.concatenate([hist_k[r], k[off[r]:off[r + 1]]]); hist_v[r] = np.concatenate([hist_v[r], v[off[r]:off[r + 1]]])
            T = int(C[r] + L[r])
            qf = W.bf16_bits_to_f64(q[off[r]:off[r + 1]])
            Kd = oracle.fp8_dequant_request(pool.h_k, pool.h_ks, bt[r], T, P)
            Vd = oracle.fp8_dequant_request(pool.h_v, pool.h_vs, bt[r], T, P)
            ref_deq.append(oracle.attn_oracle_request(qf, Kd, Vd, int(C[r]), int(L[r]), scale))
            Vu = W.bf16_bits_to_f64(hist_v[r])
            rows = np.arange(int(L[r]))
            # (a) with the cache's K but the unquantised V the probabilities are the kernel's, so the difference is
            #     sum_j p_j dV_j: bounded on EVERY row, whatever the logits, by 2^-4 max|V| + the bf16 tolerance
            ref_kd = oracle.attn_oracle_request(qf, Kd, Vu, int(C[r]), int(L[r]), scale)
            _, bmax, _ = fp8_row_bounds(Vu, int(C[r]), rows, G)
            ratio = float((np.abs(got[off[r]:off[r + 1]] - ref_kd).max(axis=2) / bmax).max())
            assert ratio <= 1.0, f"step {step} request {r}: V rounding bound exceeded ({ratio:.2f} x)"
            vonly = max(vonly, ratio)
            # (b) against the oracle on the unquantised K and V.  The first round has keys of the configuration's
            #     magnitude (at most unit variance): the stated 6e-2 / 6e-3 where >= 256 keys are visible, the derived
            #     bound elsewhere.  The second round multiplies the keys by 4 on purpose (scale raises, re-encoding):
            #     logits four times as sharp carry four times the rounding of K, which no 3-bit mantissa can hold to
            #     6e-2; there (a) and the dequantised comparison are what is asserted.
            if step == 0:
                ref_u = oracle.attn_oracle_request(qf, W.bf16_bits_to_f64(hist_k[r]), Vu, int(C[r]), int(L[r]), scale)
                unq.add(got[off[r]:off[r + 1]], ref_u, Vu, int(C[r]), rows, G, label=f"step {step} request {r}")
        mx, mean = errs(ob, ref_deq, off)
        assert mx <= TOL_BF16[0] and mean <= TOL_BF16[1], f"vs dequantised cache: {mx:.2e} {mean:.2e}"
        print(f"  step {step}: vs dequantised {mx:.2e}/{mean:.2e}; V-rounding bound used to {vonly:.2f}; " + unq.finish(f"step {step}"), flush=True)
        # re-issuing the same call changes nothing (idempotent append incl. re-encoded old slots)
        out2 = A.mixed_batch_attn(pool.cache, C, L, d_bt, to_dev_bits(q), to_dev_bits(k), to_dev_bits(v), block_table_host=bt)
        torch.cuda.synchronize()
        pool.assert_equal()
        assert np.array_equal(from_dev_bits(out2), ob)
        C = (C + L).astype(np.int32)


@pytest.mark.timeout(900)
def test_seeded_random_fp8_rounds():
    """Ten seeded random shapes, three rounds each over one pool (a prefill, a second chunk that lands in partly
    filled pages with larger keys, a decode step), lengths biased towards page / block / stage boundaries, some with
    forced key splits: pools bit-exact against the E4M3 reference after every round, attention against the oracle on
    the dequantised cache at the bf16 tolerance."""
    rng = np.random.default_rng(20260215)
    edges = np.array([1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513])
    for case in range(10):
        Hkv = int(rng.choice([1, 2, 4])); G = int(rng.choice([1, 2, 4, 8])); d = int(rng.choice([64, 128])); P = int(rng.choice([16, 32]))
        Hq, B = Hkv * G, int(rng.integers(1, 5))
        pick = lambda hi: int(rng.choice(edges[edges <= hi])) if rng.random() < 0.6 else int(rng.integers(1, hi + 1))
        rounds = [[pick(600) for _ in range(B)], [pick(300) for _ in range(B)], [1] * B]
        splits = int(rng.choice([0, 0, 3]))
        print(f"case {case}: Hq={Hq} Hkv={Hkv} d={d} P={P} rounds={rounds} splits={splits}", flush=True)
        pages = (np.sum(np.array(rounds), axis=0) + P - 1) // P
        num_pages = int(pages.sum()) + 3
        perm = rng.permutation(num_pages).astype(np.int32)
        bt = np.full((B, int(pages.max())), -1, np.int32)
        o = 0
        for r in range(B):
            bt[r, :pages[r]] = perm[o:o + pages[r]]; o += pages[r]
        scale = 1.0 / np.sqrt(d)
        pool = Fp8Pool(num_pages, Hq, Hkv, d, P, scale)
        d_bt = torch.from_numpy(bt).cuda()
        C = np.zeros(B, np.int32)
        for step, L_ in enumerate(rounds):
            L = np.array(L_, np.int32); n = int(L.sum())
            mag = np.exp2(rng.integers(-2, 1, size=(n, Hkv, 1))).astype(np.float32)
            q = W.f32_to_bf16_bits(rng.standard_normal((n, Hq, d), dtype=np.float32))
            k = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d), dtype=np.float32) * mag * (1.0 + 2 * step))
            v = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d), dtype=np.float32) * mag)
            out = A.mixed_batch_attn(pool.cache, C, L, d_bt, to_dev_bits(q), to_dev_bits(k), to_dev_bits(v),
                                     block_table_host=bt, force_kv_splits=splits)
            torch.cuda.synchronize()
            pool.reference_append(bt, C, L, k, v)
            pool.assert_equal()
            off = np.concatenate([[0], np.cumsum(L)])
            ref = []
            for r in range(B):
                T = int(C[r] + L[r])
                Kd = oracle.fp8_dequant_request(pool.h_k, pool.h_ks, bt[r], T, P)
                Vd = oracle.fp8_dequant_request(pool.h_v, pool.h_vs, bt[r], T, P)
                ref.append(oracle.attn_oracle_request(W.bf16_bits_to_f64(q[off[r]:off[r + 1]]), Kd, Vd, int(C[r]), int(L[r]), scale))
            mx, mean = errs(from_dev_bits(out), ref, off)
            assert mx <= TOL_BF16[0] and mean <= TOL_BF16[1], f"case {case} round {step}: {mx:.2e} {mean:.2e}"
            C = (C + L).astype(np.int32)


@pytest.mark.timeout(900)
def test_seeded_fp8_batches_in_every_planner_regime():
    """Eighteen seeded batches over an 8-bit cache, three in each regime in which the planner shapes the launch differently
    (a lone prefill over history, a few long decode rows, a decode batch, decode rows next to prefill rows, a small ragged
    batch, many prefill rows: persistent workgroups); head geometry (odd group sizes included), head dim and page size
    drawn as well, some with forced splits.  The history is written by a first call (pools bit-exact after it), the
    batch itself by a second: pools bit-exact again, attention against the oracle on the dequantised cache at the bf16
    tolerance."""
    rng = np.random.default_rng(20260216)
    for case in range(18):
        regime = case % 6
        Hkv = int(rng.choice([1, 2, 8])); G = int(rng.choice([1, 3, 4, 5, 8, 16])); d = int(rng.choice([64, 128])); P = int(rng.choice([16, 32]))
        if regime == 0:
            C = [int(rng.integers(0, 9000))]; L = [int(rng.integers(33, 500))]
        elif regime == 1:
            n = int(rng.integers(1, 6)); C = [int(rng.integers(2000, 16000)) for _ in range(n)]; L = [1] * n
        elif regime == 2:
            n = int(rng.integers(20, 70)); C = [int(rng.integers(100, 3000)) for _ in range(n)]; L = [1] * n
        elif regime == 3:
            n = int(rng.integers(4, 30)); C = [int(rng.integers(100, 4000)) for _ in range(n)]; L = [1] * n
            for _ in range(int(rng.integers(1, 3))):
                C.append(int(rng.integers(0, 4000))); L.append(int(rng.integers(2, 400)))
        elif regime == 4:
            n = int(rng.integers(1, 8)); C = [int(rng.integers(0, 1200)) for _ in range(n)]; L = [int(rng.integers(0, 300)) for _ in range(n)]
            if sum(L) == 0:
                L[0] = 3
        else:
            n = int(rng.integers(6, 12)); C = [int(rng.integers(0, 2500)) for _ in range(n)]; L = [int(rng.integers(100, 500)) for _ in range(n)]
        if Hkv * G * d * sum(c + l for c, l in zip(C, L)) > 1.5e8:            # bound the host-side reference work
            Hkv = 1
        if Hkv * G * d * sum(c + l for c, l in zip(C, L)) > 1.5e8:
            G = min(G, 4)
        Hq, B = Hkv * G, len(C)
        splits = int(rng.choice([0, 0, 0, 2, 7]))
        print(f"case {case}: regime {regime} Hq={Hq} Hkv={Hkv} d={d} P={P} n={B} sum C={sum(C)} sum L={sum(L)} splits={splits}", flush=True)
        C, L = np.array(C, np.int32), np.array(L, np.int32)
        pages = (C.astype(np.int64) + L + P - 1) // P
        num_pages = int(pages.sum()) + 3
        perm = rng.permutation(num_pages).astype(np.int32)
        bt = np.full((B, max(1, int(pages.max()))), -1, np.int32)
        o = 0
        for r in range(B):
            bt[r, :pages[r]] = perm[o:o + pages[r]]; o += pages[r]
        scale = 1.0 / np.sqrt(d)
        pool = Fp8Pool(num_pages, Hq, Hkv, d, P, scale)
        d_bt = torch.from_numpy(bt).cuda()
        have = np.zeros(B, np.int32)
        for step, Ls in enumerate((C, L)):
            n = int(Ls.sum())
            if n > 0:
                mag = np.exp2(rng.integers(-2, 1, size=(n, Hkv, 1))).astype(np.float32)
                q = W.f32_to_bf16_bits(rng.standard_normal((n, Hq, d), dtype=np.float32))
                k = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d), dtype=np.float32) * mag * (0.5 + step))
                v = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d), dtype=np.float32) * mag)
                fn = A.mixed_batch_attn if case % 2 else A.incr_prefill_attn
                out = fn(pool.cache, have, Ls, d_bt, to_dev_bits(q), to_dev_bits(k), to_dev_bits(v), block_table_host=bt,
                         force_kv_splits=splits if step == 1 else 0)
                torch.cuda.synchronize()
                pool.reference_append(bt, have, Ls, k, v)
                pool.assert_equal()
                if step == 1:
                    off = np.concatenate([[0], np.cumsum(Ls)])
                    ref = []
                    for r in range(B):
                        if Ls[r] == 0:
                            ref.append(None)
                            continue
                        T = int(have[r] + Ls[r])
                        Kd = oracle.fp8_dequant_request(pool.h_k, pool.h_ks, bt[r], T, P)
                        Vd = oracle.fp8_dequant_request(pool.h_v, pool.h_vs, bt[r], T, P)
                        ref.append(oracle.attn_oracle_request(W.bf16_bits_to_f64(q[off[r]:off[r + 1]]), Kd, Vd, int(have[r]), int(Ls[r]), scale))
                    mx, mean = errs(from_dev_bits(out), ref, off)
                    assert mx <= TOL_BF16[0] and mean <= TOL_BF16[1], f"case {case}: {mx:.2e} {mean:.2e}"
            have = (have + Ls).astype(np.int32)
        del pool


def _replay_on_gpu(tr, **kw):
    Hq, Hkv, d, P = tr.Hq, tr.Hkv, tr.d, tr.P
    pool = Fp8Pool(tr.num_pages, Hq, Hkv, d, P, 1.0 / np.sqrt(d))
    d_bt_full = torch.from_numpy(tr.block_table).cuda()

    def run_tick(t, tk, bt, q, k, v):
        d_bt = d_bt_full[torch.from_numpy(tk.sessions.astype(np.int64)).cuda()].contiguous()
        return A.mixed_batch_attn(pool.cache, tk.ctx_len, tk.incr_len, d_bt, to_dev_bits(q), to_dev_bits(k), to_dev_bits(v),
                                  block_table_host=bt)

    def fetch(out):
        torch.cuda.synchronize()
        return from_dev_bits(out)

    mir, report = replay_trace(tr, run_tick, fetch, **kw)
    torch.cuda.synchronize()
    print("  " + report, flush=True)
    # the pool's final byte image equals the reference replay of all appends (codes and scales, every page)
    pool.h_k, pool.h_v, pool.h_ks, pool.h_vs = mir.k, mir.v, mir.ks, mir.vs
    pool.assert_equal()


def test_session_trace_replay_fp8_reduced():
    """Configuration 5 at reduced size (8 sessions x 4 rounds, L <= 2048, 16-48 decode steps): every append and attention
    call goes through one persistent 8-bit pool; all prefill ticks and a seeded 25 % of the decode ticks are checked."""
    print("case: session trace replay (reduced)", flush=True)
    tr = W.make_trace_schedule(W.BASE_SEED + 5, num_sessions=8, rounds=4, hi=2048, dec_lo=16, dec_hi=48)
    _replay_on_gpu(tr, decode_tick_fraction=0.25, progress_every=0)


@pytest.mark.timeout(900)
def test_config5_full_size_trace_replay_fp8():
    """Configuration 5 at its stated size: 32 sessions x 8 rounds, tool outputs ~ lognormal(median 512, sigma 1) clipped
    to [16, 8192], 64-256 decode steps per round, one ampd_mixed_batch_attn call per tick through ONE persistent 8-bit
    pool.  Checked: every prefill tick (each prefill row on its first, last and 6 random query positions, plus 3 sampled
    decode rows of the tick) and a seeded 5 % of the decode-only ticks, against the oracle on the dequantised cache
    (2e-2 / 2e-3) and on the unquantised inputs (6e-2 / 6e-3 where >= 256 keys are visible, the derived bound
    elsewhere); the pool's byte image (codes and scales of all pages) bit-exact at the end."""
    print("case: configuration 5, full-size session trace replay", flush=True)
    tr = W.make_trace_schedule(W.BASE_SEED + 5)
    assert tr.num_sessions == 32 and len(tr.ticks) > 1000
    _replay_on_gpu(tr)
