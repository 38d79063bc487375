"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, validates
arguments on the host, and its work planner covers every causal (query, key) pair exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2602_14516_amd as A
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_declared_in_the_header():
    hdr = open(os.path.join(ROOT, "include", "ampd.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ampd_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(A.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(A.lib, name), name
    assert "gfx950" in A.version()
    assert A.status_string(0) == "ok" and "range" in A.status_string(-4)


def shape_cache(Hq=8, Hkv=2, d=128, P=16, scale=0.1, pages=1000):
    c = A.KVCache(Hq, Hkv, d, P, None, None, scale)
    c.num_pages_hint = pages
    return c


def test_host_validation_rejects_bad_arguments_without_a_gpu():
    ok = A.workspace_bytes(shape_cache(), [10], [5], 1)
    assert ok >= 256
    assert A.workspace_bytes(shape_cache(Hq=7), [10], [5], 1) == 0          # Hq % Hkv
    assert A.workspace_bytes(shape_cache(d=96), [10], [5], 1) == 0          # head_dim
    assert A.workspace_bytes(shape_cache(P=8), [10], [5], 1) == 0           # page size
    assert A.workspace_bytes(shape_cache(scale=0.0), [10], [5], 1) == 0     # scale
    assert A.workspace_bytes(shape_cache(), [-1], [5], 1) == 0              # negative length
    assert A.workspace_bytes(shape_cache(), [10], [7], 1) == 0              # table too narrow: 17 tokens
    assert A.workspace_bytes(shape_cache(), [10], [0], 0) >= 256            # L = 0 rows need no pages
    with pytest.raises(A.AmpdError) as e:
        A.plan_describe(shape_cache(d=96), [10], [5], 1)
    assert e.value.status == -2
    # entry points refuse NULL pools / tables before touching the GPU
    c = shape_cache()
    with pytest.raises(A.AmpdError) as e:
        A.kv_append(c, [10], [5], None, None, None, stream=0)
    assert e.value.status == -1


def test_page_range_check_uses_the_host_mirror():
    # host-only call path: ampd_kv_append validates the mirror before anything else that needs a GPU
    c = shape_cache(pages=4)
    b = A.binding
    batch, keep = b._batch([0], [20], None, np.array([[0, 9]], np.int32), max_pages=2)
    batch.d_block_table = 8          # any non-NULL address: validation must fail before it is used
    cs = c.c_struct()
    cs.k_pool = cs.v_pool = 8
    st = A.lib.ampd_kv_append(ctypes.byref(cs), ctypes.byref(batch), 8, 8, None)
    assert st == -4


def coverage_check(Hq, Hkv, d, P, C, L, splits=0):
    c = shape_cache(Hq, Hkv, d, P)
    mp = int(max(1, ((np.array(C) + np.array(L) + P - 1) // P).max()))
    items = A.plan_items(c, C, L, mp, force_kv_splits=splits)
    G = Hq // Hkv
    ranges = {}
    off = np.concatenate([[0], np.cumsum(L)])
    copied = np.zeros(int(off[-1]), np.int32)          # packed rows moved to their pages by append items
    seen_append = False
    slots = []                                         # partial-result slots [begin, end) in floats
    for req, kind, kvh, g0, gn, q0, nq, kb, ke, po in items.tolist():
        if kind == 2:                                  # null item: pads a die's queue, does no work
            assert req == -1 and nq == 0 and po == -1
            continue
        if kind == 3:                                  # append item: nq packed rows from token q0 of request req on
            assert 0 < nq <= 64 and 0 <= q0 < L[req] and po == -1
            copied[off[req] + q0:off[req] + q0 + nq] += 1
            seen_append = True
            continue
        assert not seen_append, "append items close the work list"
        assert 0 < gn <= 32 and g0 + gn <= G and nq > 0 and kb < ke and kb % 64 == 0
        assert nq * gn <= (256 if kind == 0 else 32)
        if po >= 0:
            slots.append((po, po + nq * gn * (d + 2)))
        for g in range(g0, g0 + gn):
            for i in range(q0, q0 + nq):
                ranges.setdefault((req, kvh * G + g, i), []).append((kb, ke))
    for r in range(len(C)):
        for h in range(Hq):
            for i in range(L[r]):
                rs = sorted(ranges.pop((r, h, i)))
                vis = C[r] + i + 1
                pos = 0
                for kb, ke in rs:
                    assert kb == pos, f"gap/overlap at request {r} head {h} query {i}: {rs}"
                    pos = ke
                assert pos >= vis and rs[-1][0] < vis or len(rs) == 1 or rs[-1][0] < C[r] + L[r]
                assert pos >= vis
    slots.sort()
    for (b0, e0), (b1, e1) in zip(slots, slots[1:]):
        assert e0 <= b1, "partial-result slots overlap"
    assert not ranges, "items refer to queries that do not exist"
    assert np.all(copied == 1), "every new token is written to its page exactly once"
    return items


@pytest.mark.parametrize("splits", [0, 2, 5])
def test_planner_covers_every_causal_pair_exactly_once(splits):
    rng = np.random.default_rng(splits)
    for Hq, Hkv, d, P in [(8, 2, 128, 16), (4, 4, 64, 32), (6, 2, 128, 16), (64, 1, 128, 16), (8, 1, 128, 32)]:
        C = rng.integers(0, 700, size=5).tolist()
        L = rng.integers(0, 90, size=5).tolist()
        L[0] = 1
        C[1] = 0
        coverage_check(Hq, Hkv, d, P, C, L, splits)


@pytest.mark.parametrize("geom,C,L", [
    ((32, 8, 128, 16), [4096], [512]),                 # a lone prefill whose tiles are cut for one round
    ((32, 8, 128, 16), [16384], [64]),
    ((32, 8, 128, 16), [1024], [2048]),                # tiles that fill the slots uncut
    ((8, 1, 128, 32), [57000, 60000, 50000, 61000], [1, 1, 1, 1]),     # long decode rows, one round of key ranges
    ((32, 8, 128, 16), [6000] * 26 + [3000], [1] * 26 + [300]),        # decode rows next to a prefill row
    ((32, 8, 128, 16), [9000] * 40, [1] * 40),         # 320 decode blocks on 256 slots
])
def test_planner_coverage_where_the_split_policy_cuts(geom, C, L):
    Hq, Hkv, d, P = geom
    coverage_check(Hq, Hkv, d, P, C, L)


def test_planner_coverage_on_drawn_shapes():
    """The same exact-cover property on shapes and lengths drawn by hypothesis (head geometry, page size, a few rows
    with anything from empty to several query tiles, automatic and forced key splits)."""
    from hypothesis import given, settings, strategies as st

    geoms = st.sampled_from([(8, 2, 128, 16), (32, 8, 128, 16), (4, 4, 64, 32), (10, 2, 64, 16), (64, 1, 128, 16), (48, 1, 128, 32)])
    rows = st.lists(st.tuples(st.integers(0, 1500), st.integers(0, 300)), min_size=1, max_size=4)

    @settings(max_examples=25, deadline=None, derandomize=True)
    @given(geoms, rows, st.sampled_from([0, 0, 3]))
    def check(geom, cl, splits):
        Hq, Hkv, d, P = geom
        coverage_check(Hq, Hkv, d, P, [c for c, _ in cl], [l for _, l in cl], splits)

    check()


def test_planner_kinds_and_split_policy():
    c = shape_cache(64, 8, 128, 16)
    C, L = W.config_lengths(3)
    mp = int(((C.astype(int) + L + 15) // 16).max())
    info = A.plan_describe(c, C, L, mp)
    # decode rows x 8 KV heads are narrow: 768 blocks for 256 workgroup slots, so none is cut; prefill rows are wide and unsplit
    assert info["num_combine_items"] == 0
    assert info["num_narrow_items"] == 96 * 8
    assert info["num_wide_items"] == sum(8 * -(-int(l) // 32) for l in L if l > 1)
    assert A.workspace_bytes(c, C, L, mp) == info["plan_bytes"] + -(-info["partial_bytes"] // 256) * 256
    # the order of the work list depends on lengths only (needed for bitwise page-permutation invariance)
    a = A.plan_items(c, C, L, mp)
    b = A.plan_items(c, C, L, mp)
    assert np.array_equal(a, b)
    assert info["num_append_items"] == int((a[:, 1] == 3).sum()) == -(-int(L.sum()) // 64) and np.all(a[-info["num_append_items"]:, 1] == 3)
    a = a[a[:, 1] != 3]
    keys = (a[:, 8] - a[:, 7]).astype(np.int64)
    wide, narrow = a[:, 1] == 0, a[:, 1] == 1
    assert np.all(np.diff(keys[narrow]) <= 0)          # decode items: longest first
    # the two kinds are interleaved: both appear in every quarter of the launch order
    for part_w, part_n in zip(np.array_split(wide, 4), np.array_split(narrow, 4)):
        assert part_w.any() and part_n.any()
    check_xcd_queues(a, 0.98)


def test_planner_narrow_chunks_follow_the_number_of_workgroup_slots():
    """Decode rows are cut along the keys into few, long items: one round of items on the 256 workgroup slots when the
    rows are few and long, and several pieces per row when whole rows would fill the slots
    unevenly (320 rows on 256 slots would take two rounds of whole rows; three pieces each take four rounds of thirds)."""
    c4 = shape_cache(8, 1, 128, 32)
    C = np.array([57000, 60000, 50000, 61000], np.int32)
    L = np.ones(4, np.int32)
    info = A.plan_describe(c4, C, L, 2000)
    assert 200 <= info["num_narrow_items"] <= 256 and info["num_combine_items"] == 4
    a = A.plan_items(c4, C, L, 2000)
    a = a[a[:, 1] == 1]
    keys = (a[:, 8] - a[:, 7]).astype(np.int64)
    for r in range(4):
        k = keys[a[:, 0] == r]
        assert k.sum() == C[r] + 1 and (np.sort(k)[1:] == k.max()).all()    # chunk-sized pieces and one remainder
    c2 = shape_cache(32, 8, 128, 16)
    C = np.full(40, 10000, np.int32)
    L = np.ones(40, np.int32)
    info = A.plan_describe(c2, C, L, 700)
    assert info["num_combine_items"] == 320 and info["num_narrow_items"] in (3 * 320, 4 * 320)
    # a small decode batch of uneven rows (208 on 256 slots): one round would last as long as its longest rows, so
    # the rows are cut for two to three items per slot
    C = np.random.default_rng(0).integers(500, 8000, 26).astype(np.int32)
    info = A.plan_describe(c2, C, np.ones(26, np.int32), 700)
    assert 2 * 256 <= info["num_narrow_items"] <= 3 * 256
    # ... and of few rows: one round
    info = A.plan_describe(c2, C[:6], np.ones(6, np.int32), 700)
    assert 200 <= info["num_narrow_items"] <= 256
    # a tiny launch never goes below 256-key chunks
    a1 = A.plan_items(c2, np.full(4, 700, np.int32), np.ones(4, np.int32), 701 // 16 + 1)
    a1 = a1[a1[:, 1] != 3]
    k1 = (a1[:, 8] - a1[:, 7]).astype(np.int64)
    assert k1.max() == 256 and len(a1) == 4 * 8 * 3


def test_planner_launch_shape_persistent_workgroups_only_for_long_lists_with_tiles():
    """A launch with tiles and more items than CUs is run by 256 persistent workgroups; decode rows alone, and everything
    that fits one round, get one workgroup per item."""
    c2 = shape_cache(32, 8, 128, 16)
    C, L = W.config_lengths(2)
    info = A.plan_describe(c2, C, L, int(((C.astype(int) + L + 15) // 16).max()))
    assert info["num_items"] > 256 and info["num_wide_items"] > 0 and info["num_workgroups"] == 256
    c3 = shape_cache(64, 8, 128, 16)
    C, L = W.config_lengths(3, part="decode")
    info = A.plan_describe(c3, C, L, int(((C.astype(int) + L + 15) // 16).max()))
    assert info["num_wide_items"] == 0 and info["num_workgroups"] == info["num_items"] == 770
    C, L = W.config_lengths(3)
    info = A.plan_describe(c3, C, L, int(((C.astype(int) + L + 15) // 16).max()))
    assert info["num_workgroups"] == 256
    info = A.plan_describe(c2, np.array([700], np.int32), np.array([100], np.int32), 60)
    assert info["num_workgroups"] == info["num_items"] <= 256


def test_planner_cuts_the_tiles_of_a_small_prefill_for_one_round():
    """A single incremental prefill (the paper's T_pre(l_hist, l_incr) case) has fewer tiles than workgroup slots: the key
    ranges of its tiles are cut so that the pieces fit one round on the 256 slots (all, half or a quarter of them), in
    whole 128-key stages, and not at all when the tiles already fill the slots or a cut would cost more than it saves."""
    c = shape_cache(32, 8, 128, 16)
    def plan(h, l):
        C, L = np.array([h], np.int32), np.array([l], np.int32)
        info = A.plan_describe(c, C, L, (h + l) // 16 + 1)
        a = A.plan_items(c, C, L, (h + l) // 16 + 1)
        a = a[a[:, 1] == 0]
        return info, (a[:, 8] - a[:, 7]).astype(np.int64), a
    info, keys, a = plan(4096, 512)                      # 64 tiles of 4 160 .. 4 608 keys -> 4 pieces each
    assert info["num_wide_items"] == 256 and info["num_combine_items"] == 64 and keys.max() == 1152
    info, keys, a = plan(16384, 64)                      # 8 tiles of 16 448 keys -> 16 pieces each on half the slots
    assert info["num_combine_items"] == 8 and info["num_wide_items"] <= 256 and keys.max() % 128 == 0
    info, keys, a = plan(1024, 2048)                     # 256 tiles: one round as they are
    assert info["num_wide_items"] == 256 and info["num_combine_items"] == 0
    info, keys, a = plan(0, 512)                         # short rows: nothing worth cutting
    assert info["num_combine_items"] == 0
    for h, l in ((4096, 512), (16384, 64), (1024, 512)): # pieces of a tile are contiguous and cover [0, C + q0 + nq)
        info, keys, a = plan(h, l)
        for kvh in (0, 7):
            for q0 in np.unique(a[:, 5]):
                m = a[(a[:, 2] == kvh) & (a[:, 5] == q0)]
                m = m[np.argsort(m[:, 7])]
                assert m[0, 7] == 0 and np.all(m[1:, 7] == m[:-1, 8]) and m[-1, 8] == h + q0 + m[0, 6]


def check_xcd_queues(a, min_balance):
    """Workgroup i runs on die i % 8: the tiles of one K/V stream (request, KV head) share a die, next to each
    other and longest first, and the dies carry equal wide work."""
    die = np.arange(len(a)) % 8
    wide = a[:, 1] == 0
    keys = (a[:, 8] - a[:, 7]).astype(np.int64)
    stream = a[:, 0].astype(np.int64) * 256 + a[:, 2]
    one_die = 0
    for s in np.unique(stream[wide]):
        m = np.nonzero(wide & (stream == s))[0]
        dies = np.unique(die[m])
        if len(dies) == 1:
            one_die += 1
            rises = int((np.diff(keys[m]) > 0).sum())      # a heavy stream is cut into up to 8 pieces
            assert rises <= 7
            if rises == 0:
                # adjacent in the die's queue: no wide item of another stream between the first and the last tile
                between = (die == dies[0]) & wide & (np.arange(len(a)) >= m[0]) & (np.arange(len(a)) <= m[-1])
                assert np.all(stream[between] == s)
    assert one_die >= 0.9 * len(np.unique(stream[wide]))
    load = np.array([keys[wide & (die == x)].sum() for x in range(8)])
    assert load.min() >= min_balance * load.max()


def test_planner_spreads_few_streams_over_all_dies():
    # 4 long requests with one KV head: 4 streams for 8 dies; each is cut in pieces and the dies still level out
    c = shape_cache(8, 1, 128, 32)
    C, L = W.config_lengths(4)
    mp = int(((C.astype(int) + L + 31) // 32).max())
    a = A.plan_items(c, C, L, mp)
    die = np.arange(len(a)) % 8
    wide = a[:, 1] == 0
    keys = (a[:, 8] - a[:, 7]).astype(np.int64)
    load = np.array([keys[wide & (die == x)].sum() for x in range(8)])
    assert load.min() >= 0.97 * load.max()
    assert int((a[:, 1] == 2).sum()) < 0.1 * len(a)    # null items
    for x in range(8):                                  # every die keeps at least 8 tiles of a stream it touches
        reqs, counts = np.unique(a[wide & (die == x), 0], return_counts=True)
        assert counts.min() >= 8


