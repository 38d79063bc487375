"""Pins of the fp64 oracle against things other than itself: closed forms, a pure-Python
brute force, library attention (torch SDPA with an explicit mask, numpy softmax(QK^T)V),
and the invariants the paper's setting fixes (Section 3: initial prefill is the
zero-history case of incremental prefill; after a prefill the decode worker holds all KV
and decodes one token at a time).  CPU only."""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as W

RNG = np.random.default_rng(1234)


def rand(*shape):
    return RNG.standard_normal(shape)


def numpy_attention(q, K, V, C, scale):
    """softmax(scale * Q K^T + causal mask) V written with numpy broadcasting (textbook form)."""
    L, Hq, d = q.shape
    Hkv = K.shape[1]
    Kr = np.repeat(K, Hq // Hkv, axis=1)
    Vr = np.repeat(V, Hq // Hkv, axis=1)
    S = scale * np.einsum("ihd,jhd->hij", q, Kr)
    j = np.arange(K.shape[0])[None, :]
    i = np.arange(L)[:, None]
    S = np.where(j <= C + i, S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    Pm = np.exp(S)
    Pm /= Pm.sum(axis=-1, keepdims=True)
    return np.einsum("hij,jhd->ihd", Pm, Vr)


# ---- P5 closed forms -------------------------------------------------------------------

def test_two_key_golden():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "two_key_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    q = np.array([[[2.0, 0.0]]])
    K = np.array([[[1.0, 3.0]], [[-1.0, 5.0]]])
    V = np.array([[[10.0, 0.0]], [[0.0, 20.0]]])
    out = oracle.attn_oracle_request(q, K, V, C=1, L=1, scale=0.5)
    assert out[0, 0, 0] == pytest.approx(vals["o0"], abs=1e-14)
    assert out[0, 0, 1] == pytest.approx(vals["o1"], abs=1e-14)
    p = oracle.attn_probs(q, K, 1, 1, 0.5, 0, 0)
    assert p[0] == pytest.approx(vals["p0"], abs=1e-15) and p[1] == pytest.approx(vals["p1"], abs=1e-15)
    # sigma(s0 - s1) form
    assert p[0] == pytest.approx(1.0 / (1.0 + math.exp(-2.0)), abs=1e-15)


def test_zero_query_gives_running_mean():
    C, L, Hq, Hkv, d = 5, 4, 4, 2, 8
    K, V = rand(C + L, Hkv, d), rand(C + L, Hkv, d)
    out = oracle.attn_oracle_request(np.zeros((L, Hq, d)), K, V, C, L, 0.3)
    for i in range(L):
        for h in range(Hq):
            np.testing.assert_allclose(out[i, h], V[:C + i + 1, h // 2].mean(axis=0), atol=1e-13)


def test_equal_keys_give_running_mean():
    C, L, Hq, Hkv, d = 3, 3, 2, 1, 4
    K = np.tile(rand(1, Hkv, d), (C + L, 1, 1))
    V = rand(C + L, Hkv, d)
    out = oracle.attn_oracle_request(rand(L, Hq, d), K, V, C, L, 1.7)
    for i in range(L):
        np.testing.assert_allclose(out[i, 0], V[:C + i + 1, 0].mean(axis=0), atol=1e-13)


def test_one_hot_values_return_probabilities():
    C, L, Hq, Hkv = 4, 3, 2, 2
    T = C + L
    d = T
    q, K = rand(L, Hq, d), rand(T, Hkv, d)
    V = np.zeros((T, Hkv, d))
    for j in range(T):
        V[j, :, j] = 1.0
    out = oracle.attn_oracle_request(q, K, V, C, L, 0.4)
    for i in range(L):
        for h in range(Hq):
            p = oracle.attn_probs(q, K, C, L, 0.4, i, h)
            np.testing.assert_allclose(out[i, h, :C + i + 1], p, atol=1e-15)
            assert np.all(out[i, h, C + i + 1:] == 0.0)      # causal: later keys carry no mass
            # independent closed form of the probabilities
            s = 0.4 * K[:C + i + 1, h] @ q[i, h]
            e = np.exp(s - s.max())
            np.testing.assert_allclose(p, e / e.sum(), atol=1e-15)


def test_dominant_key_selects_its_value():
    C, L, Hq, Hkv, d = 6, 1, 1, 1, 4
    q = np.zeros((L, Hq, d)); q[0, 0, 0] = 1.0
    K = np.zeros((C + L, Hkv, d)); K[2, 0, 0] = 50.0
    V = rand(C + L, Hkv, d)
    out = oracle.attn_oracle_request(q, K, V, C, L, 1.0)
    np.testing.assert_allclose(out[0, 0], V[2, 0], atol=1e-20 + 7 * np.abs(V).max() * math.exp(-50.0) * 2)


def test_single_token_no_history_returns_value():
    q, K, V = rand(1, 4, 8), rand(1, 2, 8), rand(1, 2, 8)
    out = oracle.attn_oracle_request(q, K, V, 0, 1, 0.35)
    for h in range(4):
        assert np.array_equal(out[0, h], V[0, h // 2])


def test_scale_enters_the_logits():
    # doubling scale == doubling q; and scale 0 == uniform weights
    C, L = 4, 2
    q, K, V = rand(L, 2, 8), rand(C + L, 1, 8), rand(C + L, 1, 8)
    a = oracle.attn_oracle_request(q, K, V, C, L, 0.6)
    b = oracle.attn_oracle_request(2 * q, K, V, C, L, 0.3)
    np.testing.assert_allclose(a, b, atol=1e-13)
    z = oracle.attn_oracle_request(q, K, V, C, L, 0.0)
    np.testing.assert_allclose(z[1, 0], V[:, 0].mean(axis=0), atol=1e-13)


# ---- brute force / library routines -----------------------------------------------------

@pytest.mark.parametrize("C,L,Hq,Hkv,d", [(0, 3, 2, 1, 4), (5, 1, 4, 2, 3), (7, 4, 6, 3, 5), (2, 5, 4, 4, 2)])
def test_against_pure_python_bruteforce(C, L, Hq, Hkv, d):
    q, K, V = rand(L, Hq, d), rand(C + L, Hkv, d), rand(C + L, Hkv, d)
    np.testing.assert_allclose(oracle.attn_oracle_request(q, K, V, C, L, 0.77),
                               oracle.attn_bruteforce(q, K, V, C, L, 0.77), atol=1e-13)


@pytest.mark.parametrize("C,L,Hq,Hkv,d", [(0, 17, 4, 2, 16), (33, 9, 8, 2, 64), (100, 1, 8, 1, 128), (64, 40, 6, 3, 32)])
def test_against_numpy_softmax_and_torch_sdpa(C, L, Hq, Hkv, d):
    import torch
    q, K, V = rand(L, Hq, d), rand(C + L, Hkv, d), rand(C + L, Hkv, d)
    scale = 1.0 / math.sqrt(d)
    out = oracle.attn_oracle_request(q, K, V, C, L, scale)
    np.testing.assert_allclose(out, numpy_attention(q, K, V, C, scale), atol=1e-12)
    G = Hq // Hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(K, G, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(V, G, axis=1)).permute(1, 0, 2)[None]
    mask = torch.arange(C + L)[None, :] <= (C + torch.arange(L))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


# ---- invariants ------------------------------------------------------------------------------

def test_incremental_equals_from_scratch_prefill():            # P1
    C, L, Hq, Hkv, d = 37, 11, 4, 2, 16
    T = C + L
    qall, K, V = rand(T, Hq, d), rand(T, Hkv, d), rand(T, Hkv, d)
    full = oracle.attn_oracle_request(qall, K, V, 0, T, 0.25)
    incr = oracle.attn_oracle_request(qall[C:], K, V, C, L, 0.25)
    np.testing.assert_allclose(incr, full[C:], atol=1e-13)


def test_chunked_prefill_composes():                           # P7
    C, L1, L2, Hq, Hkv, d = 9, 5, 7, 2, 1, 8
    T = C + L1 + L2
    q, K, V = rand(L1 + L2, Hq, d), rand(T, Hkv, d), rand(T, Hkv, d)
    one = oracle.attn_oracle_request(q, K, V, C, L1 + L2, 0.5)
    a = oracle.attn_oracle_request(q[:L1], K[:C + L1], V[:C + L1], C, L1, 0.5)
    b = oracle.attn_oracle_request(q[L1:], K, V, C + L1, L2, 0.5)
    np.testing.assert_allclose(one, np.concatenate([a, b]), atol=1e-13)


def test_decode_row_is_unmasked_attention_over_all_keys():    # P3
    C, Hq, Hkv, d = 50, 8, 2, 16
    q, K, V = rand(1, Hq, d), rand(C + 1, Hkv, d), rand(C + 1, Hkv, d)
    out = oracle.attn_oracle_request(q, K, V, C, 1, 0.2)
    for h in range(Hq):
        s = 0.2 * K[:, h // 4] @ q[0, h]
        p = np.exp(s - s.max()); p /= p.sum()
        np.testing.assert_allclose(out[0, h], p @ V[:, h // 4], atol=1e-13)


def test_probabilities_sum_to_one_and_output_in_hull():       # P4
    C, L, Hq, Hkv, d = 40, 6, 4, 2, 8
    q, K, V = 3 * rand(L, Hq, d), rand(C + L, Hkv, d), rand(C + L, Hkv, d)
    out, psum = oracle.attn_oracle_request(q, K, V, C, L, 1.0, want_psum=True)
    assert np.all(np.abs(psum - 1.0) < 1e-12)
    for i in range(L):
        for h in range(Hq):
            vis = V[:C + i + 1, h // 2]
            assert np.all(out[i, h] <= vis.max(axis=0) + 1e-12) and np.all(out[i, h] >= vis.min(axis=0) - 1e-12)
            assert np.all(oracle.attn_probs(q, K, C, L, 1.0, i, h) >= 0)


def test_gqa_equals_mha_with_repeated_kv_heads():             # P9
    C, L, Hq, Hkv, d = 12, 5, 6, 2, 8
    q, K, V = rand(L, Hq, d), rand(C + L, Hkv, d), rand(C + L, Hkv, d)
    a = oracle.attn_oracle_request(q, K, V, C, L, 0.4)
    b = oracle.attn_oracle_request(q, np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1), C, L, 0.4)
    np.testing.assert_allclose(a, b, atol=1e-14)
    # and the map is "consecutive query heads share a KV head", not interleaved
    c = oracle.attn_oracle_request(q, np.tile(K, (1, 3, 1)), np.tile(V, (1, 3, 1)), C, L, 0.4)
    assert np.abs(a - c).max() > 1e-3


def test_future_keys_do_not_leak():
    C, L, Hq, Hkv, d = 6, 4, 2, 1, 8
    q, K, V = rand(L, Hq, d), rand(C + L, Hkv, d), rand(C + L, Hkv, d)
    a = oracle.attn_oracle_request(q, K, V, C, L, 0.5)
    K2, V2 = K.copy(), V.copy()
    K2[C + 2:] = 1e3 * rand(L - 2, Hkv, d); V2[C + 2:] = np.nan
    b = oracle.attn_oracle_request(q, K2, V2, C, L, 0.5)
    np.testing.assert_array_equal(a[:2], b[:2])            # queries 0,1 never see keys C+2..
    # but query i does see its own key C+i
    K3 = K.copy(); K3[C + 1] += 5.0
    c = oracle.attn_oracle_request(q, K3, V, C, L, 0.5)
    assert np.array_equal(a[0], c[0]) and np.abs(a[1] - c[1]).max() > 1e-6


def test_split_kv_combine_is_associative():                   # P6
    C, d = 97, 16
    qv, K, V = rand(d), rand(C, d), rand(C, d)
    whole = oracle.combine_partials([oracle.partial_attention(qv, K, V, 0.3)])
    s = 0.3 * K @ qv; p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(whole, p @ V, atol=1e-13)
    for trial in range(20):
        cuts = np.sort(RNG.choice(np.arange(1, C), size=RNG.integers(1, 8), replace=False))
        bounds = [0, *cuts.tolist(), C]
        parts = [oracle.partial_attention(qv, K[a:b], V[a:b], 0.3) for a, b in zip(bounds[:-1], bounds[1:])]
        RNG.shuffle(parts)
        np.testing.assert_allclose(oracle.combine_partials(parts), whole, atol=1e-13)


# ---- paging ------------------------------------------------------------------------------

def test_page_permutation_and_pool_size_invariance():          # P2
    b1 = W.make_batch([37, 0, 16], [5, 9, 1], 4, 2, 8, 4, seed=7, poison=True)
    outs1 = oracle.attn_oracle(b1.k_pool, b1.v_pool, b1.block_table, b1.ctx_len, b1.incr_len,
                               b1.q, b1.k_new, b1.v_new, b1.P, b1.scale)
    # rebuild the same logical content in a larger pool with another permutation
    n2 = b1.num_pages + 13
    perm = np.random.default_rng(99).permutation(n2).astype(np.int32)
    k2 = np.full((n2,) + b1.k_pool.shape[1:], W.NAN_BF16, np.uint16)
    v2 = k2.copy()
    bt2 = np.full_like(b1.block_table, -1)
    o = 0
    for r in range(b1.num_reqs):
        for c in range(b1.block_table.shape[1]):
            if b1.block_table[r, c] >= 0:
                bt2[r, c] = perm[o]; o += 1
                k2[bt2[r, c]] = b1.k_pool[b1.block_table[r, c]]
                v2[bt2[r, c]] = b1.v_pool[b1.block_table[r, c]]
    outs2 = oracle.attn_oracle(k2, v2, bt2, b1.ctx_len, b1.incr_len, b1.q, b1.k_new, b1.v_new, b1.P, b1.scale)
    for a, b in zip(outs1, outs2):
        assert np.array_equal(a, b) and np.isfinite(a).all()


def test_poisoned_slots_are_never_read():                      # unused slots / pages / table tail
    b = W.make_batch([5, 12], [3, 1], 2, 1, 8, 4, seed=3, poison=True)
    outs = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                              b.q, b.k_new, b.v_new, b.P, b.scale)
    assert all(np.isfinite(o).all() for o in outs)


def test_append_reference_is_the_index_map():                  # P11 (append half)
    b = W.make_batch([5, 0, 8, 3], [6, 4, 1, 0], 2, 2, 4, 4, seed=11, poison=True)
    k2, v2 = oracle.kv_append_reference(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                                        b.k_new, b.v_new, b.P)
    off = b.row_offsets
    touched = np.zeros(b.k_pool.shape, bool)
    for r in range(b.num_reqs):
        C, L = int(b.ctx_len[r]), int(b.incr_len[r])
        # gather after append returns history followed by the new rows, bit for bit
        K = oracle.gather_request_kv(k2, b.block_table[r], C + L, b.P)
        V = oracle.gather_request_kv(v2, b.block_table[r], C + L, b.P)
        assert np.array_equal(K[:C], oracle.gather_request_kv(b.k_pool, b.block_table[r], C, b.P))
        assert np.array_equal(K[C:], b.k_new[off[r]:off[r + 1]])
        assert np.array_equal(V[C:], b.v_new[off[r]:off[r + 1]])
        for t in range(C, C + L):
            touched[b.block_table[r, t // b.P], :, t % b.P, :] = True
    assert np.array_equal(k2[~touched], b.k_pool[~touched])      # nothing else changes
    assert np.array_equal(v2[~touched], b.v_pool[~touched])
    # attention over (appended pool, no new tokens handed separately) == append-then-attend
    outs = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                              b.q, b.k_new, b.v_new, b.P, b.scale)
    for r in range(b.num_reqs):
        C, L = int(b.ctx_len[r]), int(b.incr_len[r])
        if L == 0:
            continue
        K = oracle.gather_request_kv(k2, b.block_table[r], C + L, b.P)
        V = oracle.gather_request_kv(v2, b.block_table[r], C + L, b.P)
        ref = oracle.attn_oracle_request(b.q[off[r]:off[r + 1]], K, V, C, L, b.scale)
        assert np.array_equal(ref, outs[r])


def test_sampled_rows_match_full_run():
    b = W.make_batch([20], [9], 4, 2, 8, 4, seed=5)
    full = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                              b.q, b.k_new, b.v_new, b.P, b.scale)[0]
    rows = np.array([0, 3, 8], np.int32)
    part = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                              b.q, b.k_new, b.v_new, b.P, b.scale, rows={0: rows})[0]
    assert np.array_equal(part, full[rows])


def test_config1_shape_runs_and_is_finite():
    b = W.make_config(1, poison=True)
    assert b.num_pages == 32 and b.block_table.shape == (1, 18) and b.flops() == 17858560
    out = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                             b.q, b.k_new, b.v_new, b.P, b.scale)[0]
    assert out.shape == (32, 8, 64) and np.isfinite(out).all()
    assert b.scale == pytest.approx(0.125)
