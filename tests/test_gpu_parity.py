"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element by element."""
import zlib

import numpy as np
import pytest
import torch

import oracle
import paper_2602_14516_amd as A
import workloads as W
from gpu_util import DevBatch, compare, from_dev_bits, sample_rows, TOL_BF16

pytestmark = pytest.mark.gpu


def run_attn(db, fn=A.incr_prefill_attn, **kw):
    b = db.b
    out = fn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q, db.k_new, db.v_new,
             block_table_host=b.block_table, **kw)
    torch.cuda.synchronize()
    return from_dev_bits(out)


def check_append(db):
    b = db.b
    k_ref, v_ref = oracle.kv_append_reference(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                                              b.k_new, b.v_new, b.P)
    assert np.array_equal(from_dev_bits(db.k_pool), k_ref), "K pool differs from the append reference"
    assert np.array_equal(from_dev_bits(db.v_pool), v_ref), "V pool differs from the append reference"


def test_config1_full():
    print("case: config 1", flush=True)
    db = DevBatch(W.make_config(1, poison=True))
    out = run_attn(db)
    check_append(db)
    mx, mean = compare(db.b, out, label="cfg1")
    print(f"cfg1 max-abs {mx:.2e} mean-abs {mean:.2e}")


@pytest.mark.parametrize("name,C,L,Hq,Hkv,d,P", [
    ("ragged-d128", [0, 1, 15, 16, 17, 100, 257, 64], [1, 7, 33, 64, 129, 5, 70, 200], 8, 2, 128, 16),
    ("ragged-d64", [0, 3, 31, 200], [65, 1, 40, 130], 8, 2, 64, 16),
    ("gqa8-p32", [300, 0, 77], [150, 31, 1], 16, 2, 128, 32),
    ("mha", [50, 129], [140, 9], 4, 4, 128, 16),
    ("gqa16-p64", [130, 5], [3, 70], 32, 2, 64, 64),
    ("decode-only", [1, 15, 16, 63, 64, 65, 1000, 2500], [1] * 8, 16, 2, 128, 16),
    ("empty-rows", [10, 0, 20], [0, 5, 0], 8, 2, 128, 16),
])
def test_small_shapes_elementwise(name, C, L, Hq, Hkv, d, P):
    print(f"case: {name}", flush=True)
    db = DevBatch(W.make_batch(C, L, Hq, Hkv, d, P, seed=zlib.crc32(name.encode()) % 10000, poison=True, name=name))
    out = run_attn(db)
    check_append(db)
    compare(db.b, out, label=name)


def test_narrow_items_of_every_row_count():
    """Items of at most 32 query rows (tokens x grouped heads) take the streaming path, in two shapes: up to 16 rows on
    16-row matrix tiles, 17 to 32 rows on 32-row tiles.  Every row count that group sizes 1, 2, 3, 4, 5, 8, 16 and
    1 to 6 new tokens give is run, with several requests per batch (chunks of more than one token cross the causal
    diagonal inside a 32-key block; context lengths around block and page boundaries; one batch with forced key splits),
    for both head dims."""
    seen = set()
    case = 0
    for d in (128, 64):
        for G in (1, 2, 3, 4, 5, 8, 16):
            Ls = [l for l in (1, 2, 3, 4, 5, 6) if l * G <= 32]
            for splits in (0, 3):
                C = [0, 1, 31, 32, 33, 100, 257, 1000][:len(Ls) + 2]
                L = (Ls + Ls)[:len(C)]
                print(f"case {case}: d={d} G={G} C={C} L={L} splits={splits}", flush=True)
                db = DevBatch(W.make_batch(C, L, 2 * G, 2, d, 16, seed=300 + case, poison=True))
                out = run_attn(db, fn=A.mixed_batch_attn, force_kv_splits=splits)
                check_append(db)
                compare(db.b, out, label=f"narrow rows case {case}")
                items = A.plan_items(db.cache, db.b.ctx_len, db.b.incr_len, db.b.block_table.shape[1], force_kv_splits=splits)
                assert (items[items[:, 1] != 3][:, 1] == 1).all()             # every attention item is a narrow one
                seen |= {int(t * g) for t, g in items[items[:, 1] == 1][:, [6, 4]]}
                case += 1
    assert {1, 2, 3, 4, 5, 6, 8, 9, 10, 12, 15, 16, 18, 20, 24, 25, 30, 32} <= seen, sorted(seen)


def test_seeded_random_shapes_elementwise():
    """Sixteen seeded random batches: head geometry, page size, head dim, request count and lengths drawn at random,
    with lengths biased towards the boundaries of pages (16 / 32), 32-key blocks, 64-key units and 128-key stages.
    Append bit-exact, attention element-wise against the oracle (sampled rows when a batch is large)."""
    rng = np.random.default_rng(20260214)
    edges = np.array([0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513])
    for case in range(16):
        Hkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 3, 4, 8, 16]))
        d = int(rng.choice([64, 128]))
        P = int(rng.choice([16, 32]))
        n = int(rng.integers(1, 7))
        pick = lambda hi: int(rng.choice(edges[edges <= hi])) if rng.random() < 0.6 else int(rng.integers(0, hi + 1))
        C = [pick(700) for _ in range(n)]
        L = [pick(300) for _ in range(n)]
        if sum(L) == 0:
            L[0] = 1
        print(f"case {case}: Hq={Hkv * G} Hkv={Hkv} d={d} P={P} C={C} L={L}", flush=True)
        db = DevBatch(W.make_batch(C, L, Hkv * G, Hkv, d, P, seed=1000 + case, poison=True))
        fn = A.mixed_batch_attn if case % 2 else A.incr_prefill_attn
        out = run_attn(db, fn=fn, force_kv_splits=int(rng.choice([0, 0, 2, 5])))
        check_append(db)
        rows = sample_rows(db.b, 12, seed=case) if sum(L) * Hkv * G > 6000 else None
        compare(db.b, out, rows=rows, label=f"random case {case}")


@pytest.mark.parametrize("splits", [2, 3, 7])
def test_forced_kv_splits_match(splits):
    print(f"case: forced splits {splits}", flush=True)
    b = W.make_batch([0, 500, 1025, 64, 3000], [300, 1, 77, 2, 1], 8, 2, 128, 16, seed=21, poison=True)
    db = DevBatch(b)
    out = run_attn(db, force_kv_splits=splits)
    compare(b, out, label=f"splits{splits}")


@pytest.mark.parametrize("splits", [9, 17, 33])
def test_many_kv_splits_take_the_wide_combine_groups(splits):
    """More than 8 splits per row (long decode contexts): the combine pass then walks them 16 at a time, with a
    ragged last group (9 -> 9, 17 -> 16 + 1 or 16, 33 -> 29 splits on the longest row)."""
    print(f"case: many splits {splits}", flush=True)
    b = W.make_batch([9000, 4100, 2500], [1, 1, 40], 8, 2, 128, 16, seed=23, poison=True)
    out = run_attn(DevBatch(b), force_kv_splits=splits)
    compare(b, out, label=f"splits{splits}")


@pytest.mark.parametrize("d,G", [(64, 3), (128, 5)])
def test_many_kv_splits_odd_row_counts(d, G):
    """Few tiles with many splits are combined by thread slices that share a tile's splits (two rows per workgroup):
    odd row counts (3 or 5 heads per KV head) leave the last workgroup of a tile one row, and d = 64 doubles the slices."""
    print(f"case: many splits, odd rows, d={d} G={G}", flush=True)
    b = W.make_batch([9000, 4100, 700], [1, 5, 1], 2 * G, 2, d, 16, seed=29, poison=True)
    out = run_attn(DevBatch(b), force_kv_splits=40)
    compare(b, out, label=f"splits40 d{d} G{G}")


@pytest.mark.parametrize("C,L", [(4096, 512), (16384, 64), (1024, 2048), (700, 1024)])
def test_lone_prefill_whose_tiles_the_planner_cuts_for_one_round(C, L):
    """A single request with fewer query tiles than CUs: the planner cuts the key ranges of its tiles (4 and 16 pieces
    in the first two cases, none in the third, two for the longer tiles of the fourth); sampled rows against the oracle."""
    print(f"case: lone prefill C={C} L={L}", flush=True)
    b = W.make_batch([C], [L], 32, 8, 128, 16, seed=C + L, poison=True)
    db = DevBatch(b)
    out = run_attn(db)
    check_append(db)
    compare(b, out, rows=sample_rows(b, 24, seed=5), label=f"lone prefill {C}+{L}")


def test_seeded_batches_in_the_regimes_of_the_split_policy():
    """Forty-eight seeded random batches, six in each regime in which the planner cuts key ranges or shapes the launch
    differently: a lone prefill (tiles cut for one round), a few long decode rows (one round of key ranges), a decode batch
    with one to three blocks per workgroup slot, decode rows next to a prefill row, a small ragged batch, several prefill
    rows, many prefill rows and large mixed batches (long work lists with tiles: persistent workgroups that take items
    from their die's queue and from other dies'); head geometry (odd group sizes included), head dim and page size drawn
    as well, some with forced splits."""
    rng = np.random.default_rng(20260215)
    for case in range(48):
        regime = case % 8
        Hkv = int(rng.choice([1, 2, 8])); G = int(rng.choice([1, 3, 4, 5, 8, 16])); d = int(rng.choice([64, 128])); P = int(rng.choice([16, 32]))
        if regime == 0:
            C = [int(rng.integers(0, 20000))]; L = [int(rng.integers(33, 1500))]
        elif regime == 1:
            n = int(rng.integers(1, 6)); C = [int(rng.integers(2000, 40000)) for _ in range(n)]; L = [1] * n
        elif regime == 2:
            n = int(rng.integers(20, 90)); C = [int(rng.integers(100, 6000)) for _ in range(n)]; L = [1] * n
        elif regime == 3:
            n = int(rng.integers(4, 30)); C = [int(rng.integers(100, 8000)) for _ in range(n)]; L = [1] * n
            for _ in range(int(rng.integers(1, 3))):
                C.append(int(rng.integers(0, 6000))); L.append(int(rng.integers(2, 900)))
        elif regime == 4:
            n = int(rng.integers(1, 8)); C = [int(rng.integers(0, 1200)) for _ in range(n)]; L = [int(rng.integers(0, 300)) for _ in range(n)]
            if sum(L) == 0:
                L[0] = 3
        elif regime == 5:
            n = int(rng.integers(2, 6)); C = [int(rng.integers(0, 5000)) for _ in range(n)]; L = [int(rng.integers(40, 700)) for _ in range(n)]
        elif regime == 6:
            n = int(rng.integers(6, 15)); C = [int(rng.integers(0, 4000)) for _ in range(n)]; L = [int(rng.integers(100, 900)) for _ in range(n)]
        else:
            n = int(rng.integers(30, 80)); C = [int(rng.integers(100, 3000)) for _ in range(n)]; L = [1] * n
            for _ in range(int(rng.integers(3, 8))):
                C.append(int(rng.integers(0, 3000))); L.append(int(rng.integers(64, 700)))
        if Hkv * G * d * sum(c + l for c, l in zip(C, L)) > 6e8:          # bound the host-side pool
            Hkv = 1
        splits = int(rng.choice([0, 0, 0, 2, 7]))
        print(f"case {case}: regime {regime} Hq={Hkv * G} Hkv={Hkv} d={d} P={P} n={len(C)} sum C={sum(C)} sum L={sum(L)} splits={splits}", flush=True)
        db = DevBatch(W.make_batch(C, L, Hkv * G, Hkv, d, P, seed=10000 + case, poison=True))
        out = run_attn(db, fn=A.mixed_batch_attn if case % 2 else A.incr_prefill_attn, force_kv_splits=splits)
        check_append(db)
        compare(db.b, out, rows=sample_rows(db.b, 6, seed=case) if sum(L) > 12 else None, label=f"regime {regime} case {case}")


def test_mixed_equals_separate_sub_batches():
    print("case: mixed vs separate", flush=True)
    C = [700, 90, 2048, 5, 300, 1500]
    L = [1, 260, 1, 1, 40, 1]
    b = W.make_batch(C, L, 16, 2, 128, 16, seed=31, poison=True)
    db = DevBatch(b)
    mixed = run_attn(db, fn=A.mixed_batch_attn)
    check_append(db)
    compare(b, mixed, label="mixed")
    # the rows of a mixed batch equal the rows of running each row alone
    off = b.row_offsets
    for r in range(len(C)):
        sub = W.Batch(b.Hq, b.Hkv, b.d, b.P, b.scale, b.ctx_len[r:r + 1], b.incr_len[r:r + 1],
                      b.block_table[r:r + 1], b.num_pages, b.k_pool, b.v_pool,
                      b.q[off[r]:off[r + 1]], b.k_new[off[r]:off[r + 1]], b.v_new[off[r]:off[r + 1]])
        o = run_attn(DevBatch(sub), fn=A.mixed_batch_attn)
        assert np.array_equal(o, mixed[off[r]:off[r + 1]]), f"row {r} differs between mixed and single-row launch"


def test_page_permutation_is_bitwise_invariant_and_relaunch_idempotent():
    print("case: permutation", flush=True)
    C, L = [333, 40, 1200], [70, 1, 5]
    b1 = W.make_batch(C, L, 8, 2, 128, 16, seed=41, poison=True)
    db1 = DevBatch(b1)
    o1 = run_attn(db1)
    o1b = run_attn(db1)                       # same call again: append and attention are idempotent
    assert np.array_equal(o1, o1b)
    # same logical content, other physical pages, bigger pool
    n2 = b1.num_pages + 37
    perm = np.random.default_rng(5).permutation(n2).astype(np.int32)
    k2 = np.full((n2,) + b1.k_pool.shape[1:], W.NAN_BF16, np.uint16)
    v2 = k2.copy()
    bt2 = np.full_like(b1.block_table, -1)
    i = 0
    for r in range(b1.num_reqs):
        for c in range(b1.block_table.shape[1]):
            if b1.block_table[r, c] >= 0:
                bt2[r, c] = perm[i]; i += 1
                k2[bt2[r, c]] = b1.k_pool[b1.block_table[r, c]]
                v2[bt2[r, c]] = b1.v_pool[b1.block_table[r, c]]
    b2 = W.Batch(b1.Hq, b1.Hkv, b1.d, b1.P, b1.scale, b1.ctx_len, b1.incr_len, bt2, n2, k2, v2, b1.q, b1.k_new, b1.v_new)
    o2 = run_attn(DevBatch(b2))
    assert np.array_equal(o1, o2)


def test_append_alone_is_bit_exact_and_touches_nothing_else():
    print("case: append alone", flush=True)
    b = W.make_batch([0, 5, 16, 100, 31], [40, 1, 16, 3, 0], 8, 4, 128, 16, seed=51, poison=True)
    db = DevBatch(b)
    A.kv_append(db.cache, b.ctx_len, b.incr_len, db.bt, db.k_new, db.v_new, block_table_host=b.block_table)
    torch.cuda.synchronize()
    check_append(db)
    # attention-only over the appended pool equals append-then-attend
    o = A.paged_attn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q)
    torch.cuda.synchronize()
    compare(b, from_dev_bits(o), label="append+paged_attn")


def test_shrunk_config_shapes():
    for k, s in ((2, 8), (3, 16), (4, 32)):
        print(f"case: cfg{k}/s{s}", flush=True)
        b = W.make_config(k, shrink=s, poison=True)
        db = DevBatch(b)
        out = run_attn(db, fn=A.mixed_batch_attn if k == 3 else A.incr_prefill_attn)
        rows = sample_rows(b, 6, seed=k)
        mx, mean = compare(b, out, rows=rows, label=b.name)
        print(f"{b.name} max-abs {mx:.2e} mean-abs {mean:.2e}")


# ---- full-size configurations, in the launch configuration bench.py times --------------------

def _full_config(k, part="all", fn=None, per_req=6, **kw):
    b = W.make_config(k, part=part)
    db = DevBatch(b)
    out = run_attn(db, fn=fn or A.incr_prefill_attn, **kw)
    rows = sample_rows(b, per_req, seed=k)
    mx, mean = compare(b, out, rows=rows, label=b.name)
    print(f"{b.name}: sampled max-abs {mx:.2e} mean-abs {mean:.2e}", flush=True)
    return b, db, out


@pytest.mark.timeout(600)
def test_config2_full_size_sampled_rows_and_append():
    print("case: config 2 full size", flush=True)
    b, db, out = _full_config(2)
    check_append(db)
    # property that holds at any size: with the same key-range cutting (here: none), the output of a row
    # is bitwise independent of the rest of the batch
    assert A.plan_describe(db.cache, b.ctx_len, b.incr_len, b.block_table.shape[1])["num_combine_items"] == 0
    r = int(np.argmin(b.incr_len))
    off = b.row_offsets
    sub = W.Batch(b.Hq, b.Hkv, b.d, b.P, b.scale, b.ctx_len[r:r + 1], b.incr_len[r:r + 1],
                  b.block_table[r:r + 1], b.num_pages, b.k_pool, b.v_pool,
                  b.q[off[r]:off[r + 1]], b.k_new[off[r]:off[r + 1]], b.v_new[off[r]:off[r + 1]])
    o = run_attn(DevBatch(sub), force_kv_splits=1)
    assert np.array_equal(o, out[off[r]:off[r + 1]])
    # and with the automatic cutting of the small batch it stays within tolerance
    o2 = run_attn(DevBatch(sub))
    assert np.abs(W.bf16_bits_to_f64(o2) - W.bf16_bits_to_f64(o)).max() <= 2e-2


@pytest.mark.timeout(900)
def test_config2_full_size_every_row():
    """Configuration 2 at full size, in the launch configuration bench.py times, compared with the oracle on EVERY
    query position and head (about 0.67 TFLOP of fp64 oracle work: minutes on the host cores)."""
    print("case: config 2 full size, every row", flush=True)
    b = W.make_config(2)
    out = run_attn(DevBatch(b))
    got = W.bf16_bits_to_f64(out)
    off = b.row_offsets
    worst, total, count = 0.0, 0.0, 0
    for r in range(b.num_reqs):                        # one request at a time keeps the fp64 copies small
        ref = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len, b.q, b.k_new, b.v_new, b.P, b.scale,
                                 rows={r: np.arange(int(b.incr_len[r]), dtype=np.int32)})[r]
        g = got[off[r]:off[r + 1]]
        assert np.isfinite(g).all()
        e = np.abs(g - ref)
        assert e.max() <= TOL_BF16[0], f"request {r}: max-abs {e.max():.3e}"
        worst, total, count = max(worst, float(e.max())), total + float(e.sum()), count + e.size
        print(f"  request {r} (C={int(b.ctx_len[r])}, L={int(b.incr_len[r])}): max-abs {e.max():.2e}", flush=True)
    assert total / count <= TOL_BF16[1]
    print(f"cfg2, all {off[-1]} query positions x {b.Hq} heads: max-abs {worst:.2e} mean-abs {total / count:.2e}", flush=True)


@pytest.mark.timeout(900)
def test_config3_full_size_mixed_batch():
    print("case: config 3 full size (mixed, one fused launch)", flush=True)
    b, db, out = _full_config(3, fn=A.mixed_batch_attn, per_req=4)
    info = A.plan_describe(db.cache, b.ctx_len, b.incr_len, b.block_table.shape[1])
    # 768 decode blocks on 256 workgroup slots: the planner cuts none of them, and the prefill rows are not cut either
    assert info["num_wide_items"] > 0 and info["num_narrow_items"] == 96 * 8 and info["num_combine_items"] == 0
    # the same launch with every key range cut in three (split-KV items of both kinds and the combine pass, full size)
    print("case: config 3 full size, forced splits", flush=True)
    out3 = run_attn(db, fn=A.mixed_batch_attn, force_kv_splits=3)       # (the append is idempotent)
    compare(b, out3, rows=sample_rows(b, 4, seed=33), label="cfg3 forced splits")
    assert np.abs(W.bf16_bits_to_f64(out) - W.bf16_bits_to_f64(out3)).max() <= 2e-2


@pytest.mark.timeout(900)
def test_config3_decode_rows_only():
    print("case: config 3 decode rows", flush=True)
    _full_config(3, part="decode", fn=A.mixed_batch_attn, per_req=1)


@pytest.mark.timeout(900)
def test_config4_long_context_prefill_then_decode_with_and_without_forced_splits():
    print("case: config 4 full size", flush=True)
    b, db, out = _full_config(4, per_req=5)
    check_append(db)
    # split-KV forced on the prefill rows: same rows within tolerance of the oracle and close to the unsplit run
    out2 = run_attn(db, force_kv_splits=3)
    rows = sample_rows(b, 5, seed=4)
    compare(b, out2, rows=rows, label="cfg4 forced splits")
    d = np.abs(W.bf16_bits_to_f64(out) - W.bf16_bits_to_f64(out2))
    assert d.max() <= 2e-2
    # the decode step that follows: L = 1 over C + 4096 keys, split-KV path
    print("case: config 4 decode step", flush=True)
    C2 = (b.ctx_len + b.incr_len).astype(np.int32)
    g = np.random.default_rng(44)
    q1 = W.f32_to_bf16_bits(g.standard_normal((4, b.Hq, b.d), dtype=np.float32))
    k1 = W.f32_to_bf16_bits(g.standard_normal((4, b.Hkv, b.d), dtype=np.float32))
    v1 = W.f32_to_bf16_bits(g.standard_normal((4, b.Hkv, b.d), dtype=np.float32))
    need = (C2.astype(np.int64) + 1 + b.P - 1) // b.P
    k_after, v_after = from_dev_bits(db.k_pool), from_dev_bits(db.v_pool)
    bt = b.block_table
    if need.max() > bt.shape[1]:                 # a row whose T was a multiple of P needs one more page
        used = set(bt[bt >= 0].tolist())
        free = [x for x in range(b.num_pages) if x not in used]
        bt = np.concatenate([bt, np.full((4, 1), -1, np.int32)], axis=1)
        for r in range(4):
            if need[r] > (bt[r] >= 0).sum():
                bt[r, need[r] - 1] = free.pop()
    b2 = W.Batch(b.Hq, b.Hkv, b.d, b.P, b.scale, C2, np.ones(4, np.int32), bt, b.num_pages, k_after, v_after, q1, k1, v1)
    db2 = DevBatch(b2)
    o2 = run_attn(db2, fn=A.mixed_batch_attn)
    info = A.plan_describe(db2.cache, b2.ctx_len, b2.incr_len, bt.shape[1])
    assert info["num_narrow_items"] > 4 and info["num_combine_items"] == 4
    compare(b2, o2, label="cfg4 decode step")
