"""GPU parity of the KV pack / unpack kernels (the GPU side of a KV transfer between workers with
different tensor-parallel degrees): bit-exact against a numpy gather / scatter."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_14516_amd as A
import workloads as W
from gpu_util import DevBatch, from_dev_bits, to_dev_bits

pytestmark = pytest.mark.gpu


def test_pack_equals_gather_for_every_head_share():
    print("case: pack", flush=True)
    b = W.make_batch([300, 17, 64, 0], [0, 0, 0, 0], 16, 8, 128, 16, seed=3, poison=False)
    # tokens [first, first+count) of each request; request 3 contributes nothing
    first = np.array([37, 0, 16, 0], np.int32)
    count = np.array([200, 17, 48, 0], np.int32)
    pages = (first + count + b.P - 1) // b.P
    assert (pages <= b.block_table.shape[1]).all()
    db = DevBatch(b)
    n = int(count.sum())
    for h0, hn in [(0, 8), (0, 2), (2, 2), (4, 4), (7, 1)]:       # e.g. source TP=1 serving destination TP=4, 4, 2, 8
        ko = torch.zeros(n, hn, b.d, dtype=torch.bfloat16, device="cuda")
        vo = torch.zeros_like(ko)
        A.kv_pack(db.cache, first, count, db.bt, h0, hn, ko, vo, block_table_host=b.block_table)
        torch.cuda.synchronize()
        off = 0
        for r in range(4):
            if count[r] == 0:
                continue
            Kr = oracle.gather_request_kv(b.k_pool, b.block_table[r], int(first[r] + count[r]), b.P)[first[r]:, h0:h0 + hn]
            Vr = oracle.gather_request_kv(b.v_pool, b.block_table[r], int(first[r] + count[r]), b.P)[first[r]:, h0:h0 + hn]
            assert np.array_equal(from_dev_bits(ko[off:off + count[r]]), Kr)
            assert np.array_equal(from_dev_bits(vo[off:off + count[r]]), Vr)
            off += int(count[r])


def test_reshard_round_trip_between_tp_degrees():
    """A decode worker at TP=2 (4 KV heads per rank) sends history KV to a prefill worker at TP=4 (2 heads per rank):
    each source rank packs one buffer per destination rank; each destination rank unpacks what it receives.  The
    destination pools must end up holding exactly the source tokens of their heads."""
    print("case: reshard 2 -> 4", flush=True)
    Hkv, d, P = 8, 128, 16
    C = np.array([150, 33], np.int32)
    zero = np.zeros(2, np.int32)
    src = W.make_batch(C.tolist(), [0, 0], 16, Hkv, d, P, seed=8)
    # source rank s holds heads [4s, 4s+4) in a pool with 4 heads; destination rank t holds heads [2t, 2t+2)
    n = int(C.sum())
    dst_pages = src.num_pages + 7
    perm = np.random.default_rng(1).permutation(dst_pages).astype(np.int32)
    need = (C + P - 1) // P
    bt_dst = np.full((2, int(need.max())), -1, np.int32)
    o = 0
    for r in range(2):
        bt_dst[r, :need[r]] = perm[o:o + need[r]]; o += need[r]
    d_bt_src = torch.from_numpy(src.block_table).cuda()
    d_bt_dst = torch.from_numpy(bt_dst).cuda()
    dst_pools = []
    for t in range(4):
        kp = torch.zeros(dst_pages, 2, P, d, dtype=torch.bfloat16, device="cuda")
        dst_pools.append((kp, torch.zeros_like(kp)))
    for s in range(2):
        kp = to_dev_bits(src.k_pool[:, 4 * s:4 * s + 4].copy())
        vp = to_dev_bits(src.v_pool[:, 4 * s:4 * s + 4].copy())
        cache_s = A.KVCache(8, 4, d, P, kp, vp, 0.1)
        for t in (2 * s, 2 * s + 1):                             # destination ranks whose heads live on source rank s
            local_h0 = 2 * t - 4 * s
            kb = torch.empty(n, 2, d, dtype=torch.bfloat16, device="cuda")
            vb = torch.empty_like(kb)
            A.kv_pack(cache_s, zero, C, d_bt_src, local_h0, 2, kb, vb, block_table_host=src.block_table)
            cache_t = A.KVCache(4, 2, d, P, dst_pools[t][0], dst_pools[t][1], 0.1)
            A.kv_unpack(cache_t, zero, C, d_bt_dst, 0, 2, kb, vb, block_table_host=bt_dst)
    torch.cuda.synchronize()
    for t in range(4):
        for r in range(2):
            got_k = oracle.gather_request_kv(from_dev_bits(dst_pools[t][0]), bt_dst[r], int(C[r]), P)
            got_v = oracle.gather_request_kv(from_dev_bits(dst_pools[t][1]), bt_dst[r], int(C[r]), P)
            want_k = oracle.gather_request_kv(src.k_pool, src.block_table[r], int(C[r]), P)[:, 2 * t:2 * t + 2]
            want_v = oracle.gather_request_kv(src.v_pool, src.block_table[r], int(C[r]), P)[:, 2 * t:2 * t + 2]
            assert np.array_equal(got_k, want_k) and np.array_equal(got_v, want_v)


def test_unpack_over_all_heads_equals_append_and_errors():
    print("case: unpack == append", flush=True)
    b = W.make_batch([40, 5], [30, 1], 8, 4, 64, 32, seed=2, poison=True)
    db1, db2 = DevBatch(b), DevBatch(b)
    A.kv_append(db1.cache, b.ctx_len, b.incr_len, db1.bt, db1.k_new, db1.v_new)
    A.kv_unpack(db2.cache, b.ctx_len, b.incr_len, db2.bt, 0, 4, db2.k_new, db2.v_new)
    torch.cuda.synchronize()
    assert np.array_equal(from_dev_bits(db1.k_pool), from_dev_bits(db2.k_pool))
    assert np.array_equal(from_dev_bits(db1.v_pool), from_dev_bits(db2.v_pool))
    with pytest.raises(A.AmpdError) as e:
        A.kv_pack(db1.cache, b.ctx_len, b.incr_len, db1.bt, 3, 2, db1.k_new, db1.v_new)      # heads 3..4 of 4
    assert e.value.status == -1
