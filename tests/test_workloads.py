"""The seeded generators: determinism, shapes and length ranges of the benchmark configurations."""
import numpy as np

import workloads as W


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 0.0, 65504.0], np.float32)
    b = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f64(b)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625      # ties go to even
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


def test_config_lengths_follow_the_stated_ranges():
    C, L = W.config_lengths(2)
    assert len(C) == 16 and C.min() >= 1024 and C.max() <= 8192 and L.min() >= 64 and L.max() <= 1024
    C, L = W.config_lengths(3)
    dec = L == 1
    assert dec.sum() == 96 and (~dec).sum() == 8
    assert C[dec].min() >= 2048 and C[dec].max() <= 16384
    assert L[~dec].min() >= 256 and L[~dec].max() <= 2048 and C[~dec].min() >= 1024 and C[~dec].max() <= 8192
    Cd, Ld = W.config_lengths(3, part="decode")
    assert np.array_equal(np.sort(Cd), np.sort(C[dec])) and np.all(Ld == 1)
    C, L = W.config_lengths(4)
    assert len(C) == 4 and C.min() >= 32768 and C.max() <= 65536 and np.all(L == 4096)


def test_batches_are_deterministic_and_tables_disjoint():
    a = W.make_config(2, shrink=16)
    b = W.make_config(2, shrink=16)
    for f in ("k_pool", "v_pool", "q", "k_new", "v_new", "block_table"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    used = a.block_table[a.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < a.num_pages
    need = (a.ctx_len.astype(int) + a.incr_len + a.P - 1) // a.P
    assert np.array_equal((a.block_table >= 0).sum(axis=1), need)
    assert a.num_pages >= int(np.ceil(need.sum() * 1.1)) - 1


def test_trace_schedule_is_consistent():
    tr = W.make_trace_schedule(W.BASE_SEED + 5, num_sessions=6, rounds=3, hi=512, dec_lo=4, dec_hi=9)
    ctx = np.zeros(6, int)
    rounds = np.zeros(6, int)
    for t, tk in enumerate(tr.ticks):
        assert len(np.unique(tk.sessions)) == len(tk.sessions)
        for s, c, l in zip(tk.sessions, tk.ctx_len, tk.incr_len):
            assert c == ctx[s] and l >= 1
            ctx[s] += l
            rounds[s] += l > 1 or c == 0
        bt = tr.tick_block_table(t)
        need = (tk.ctx_len.astype(int) + tk.incr_len + tr.P - 1) // tr.P
        for i in range(len(need)):
            assert np.all(bt[i, :need[i]] >= 0)
    used = tr.block_table[tr.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < tr.num_pages
    q, k, v = W.draw_tick_tensors(tr, 3)
    q2, _, _ = W.draw_tick_tensors(tr, 3)
    assert np.array_equal(q, q2) and q.shape[0] == tr.ticks[3].incr_len.sum()
