"""The entry point that allocates nothing: ampd_mixed_batch_attn_static keeps the work list and the split-KV partial
results in the library's static device array instead of a caller workspace.  Called through the C ABI twice in a row,
the second time with a smaller batch (whose work list and partials then sit in memory the first call left dirty),
and compared bit for bit with ampd_mixed_batch_attn on the same inputs, and with the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_14516_amd as A
import workloads as W
from gpu_util import DevBatch, compare, from_dev_bits

pytestmark = pytest.mark.gpu


def _both(b, **kw):
    ref_db, st_db = DevBatch(b), DevBatch(b)
    ref = A.mixed_batch_attn(ref_db.cache, b.ctx_len, b.incr_len, ref_db.bt, ref_db.q, ref_db.k_new, ref_db.v_new,
                             block_table_host=b.block_table)
    out = torch.full_like(st_db.q, float("nan"))
    A.mixed_batch_attn_static(st_db.cache, b.ctx_len, b.incr_len, st_db.bt, st_db.q, st_db.k_new, st_db.v_new, out,
                              block_table_host=b.block_table)
    return ref_db, st_db, ref, out


def test_static_workspace_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    print("case: static workspace, two calls", flush=True)
    A.init()
    assert A.static_workspace_limit() == 32 << 20
    # call 1: decode rows over long contexts (many key splits: partial results and a combine pass), a prefill row whose
    # key range is split too (few wide tiles), and a short row; call 2: a smaller batch of the same kinds
    big = W.make_batch([9000, 4100, 300, 2500, 0], [1, 1, 700, 40, 9], 16, 2, 128, 16, seed=71, poison=True)
    small = W.make_batch([1200, 64, 5], [1, 130, 3], 16, 2, 128, 16, seed=72, poison=True)
    for b in (big, small):
        info = A.plan_describe(DevBatch(b).cache, b.ctx_len, b.incr_len, b.block_table.shape[1])
        assert info["num_combine_items"] > 0 and info["partial_bytes"] > 0, "the case is meant to use the partial results"
    pending = [_both(big), _both(small)]              # both calls enqueued back to back before anything is read
    torch.cuda.synchronize()
    for b, (ref_db, st_db, ref, out) in zip((big, small), pending):
        o = from_dev_bits(out)
        assert np.array_equal(o, from_dev_bits(ref)), "static-workspace output differs from the workspace entry point"
        assert np.array_equal(from_dev_bits(st_db.k_pool), from_dev_bits(ref_db.k_pool))
        assert np.array_equal(from_dev_bits(st_db.v_pool), from_dev_bits(ref_db.v_pool))
        compare(b, o, label="static workspace")


@pytest.mark.parametrize("name,n,c,l,Hq,Hkv", [
    ("work list beyond one staging buffer", 1500, 40000, 1, 64, 8),       # 12 000 work items = 600 KB of work list
    ("partial results beyond the static array", 300, 20000, 32, 8, 1),    # 300 256-row tiles cut into 3 key pieces each = 114 MiB
])
def test_static_workspace_entry_point_rejects_what_does_not_fit(name, n, c, l, Hq, Hkv):
    """Both limits are checked on the host before anything is enqueued.  (The inputs are harmless even if they were
    not: every block-table entry names page 0 of a 16-page pool.)"""
    print(f"case: static workspace, {name}", flush=True)
    A.init()
    d, P = 128, 16
    C = np.full(n, c, np.int32)
    L = np.full(n, l, np.int32)
    max_pages = (c + l) // P + 1
    pool = torch.zeros(16, Hkv, P, d, dtype=torch.bfloat16, device="cuda")
    cache = A.KVCache(Hq, Hkv, d, P, pool, pool.clone(), 1.0 / np.sqrt(d))
    info = A.plan_describe(cache, C, L, max_pages)
    need = A.workspace_bytes(cache, C, L, max_pages)
    assert need > A.static_workspace_limit() or info["plan_bytes"] > (256 << 10), (need, info)
    bt = torch.zeros(n, max_pages, dtype=torch.int32, device="cuda")
    q = torch.ones(n * l, Hq, d, dtype=torch.bfloat16, device="cuda")
    kv = torch.ones(n * l, Hkv, d, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(A.AmpdError) as ei:
        A.mixed_batch_attn_static(cache, C, L, bt, q, kv, kv, torch.empty_like(q))
    assert ei.value.status == -3                      # AMPD_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not pool.any(), "a rejected call must not have enqueued the append"


def test_static_entry_point_waits_for_the_oldest_staging_buffer_when_all_are_in_flight():
    """The entry point may not pin another staging buffer, so with all buffers of the ring in flight it waits until the
    attention launch of the oldest call has started.  Far more calls than buffers are enqueued back to back, each long
    enough on the GPU for the host to run ahead; every call must come back (in bounded time), and the last output must
    equal that of the workspace entry point bit for bit."""
    import time
    print("case: static workspace, calls in flight beyond the ring", flush=True)
    A.init()
    b = W.make_batch([3000, 2500, 3500, 2800], [400, 380, 420, 390], 32, 8, 128, 16, seed=73, poison=True)
    ref_db, st_db = DevBatch(b), DevBatch(b)
    ref = A.mixed_batch_attn(ref_db.cache, b.ctx_len, b.incr_len, ref_db.bt, ref_db.q, ref_db.k_new, ref_db.v_new,
                             block_table_host=b.block_table)
    outs = [torch.full_like(st_db.q, float("nan")) for _ in range(4)]
    torch.cuda.synchronize()
    calls = 400
    t0 = time.perf_counter()
    for i in range(calls):
        A.mixed_batch_attn_static(st_db.cache, b.ctx_len, b.incr_len, st_db.bt, st_db.q, st_db.k_new, st_db.v_new,
                                  outs[i % 4], block_table_host=b.block_table)
    host_s = time.perf_counter() - t0
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    print(f"{calls} calls: host {host_s * 1e3:.1f} ms, with the GPU {total_s * 1e3:.1f} ms", flush=True)
    assert total_s < 2.0, "a call waited for its staging buffer far longer than the GPU work takes"
    for o in outs:
        assert np.array_equal(from_dev_bits(o), from_dev_bits(ref))
