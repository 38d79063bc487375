"""GPU edge cases of the C ABI: head-group shapes, many requests, chunked prefill, determinism,
error paths that must not enqueue anything, non-default streams."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_14516_amd as A
import workloads as W
from gpu_util import DevBatch, compare, from_dev_bits, sample_rows, to_dev_bits

pytestmark = pytest.mark.gpu


def run(db, fn=A.mixed_batch_attn, **kw):
    b = db.b
    out = fn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q, db.k_new, db.v_new, block_table_host=b.block_table, **kw)
    torch.cuda.synchronize()
    return from_dev_bits(out)


@pytest.mark.parametrize("name,C,L,Hq,Hkv,d,P", [
    ("mqa-64-heads", [40, 300], [3, 1], 64, 1, 128, 16),          # G = 64: two head blocks of 32
    ("g3", [77, 0, 500], [50, 11, 1], 6, 2, 128, 16),             # G = 3: 10 tokens per wave, 2 idle rows
    ("g5-d64", [10, 200], [70, 1], 10, 2, 64, 32),
    ("g48", [65], [2], 48, 1, 128, 16),                           # head blocks of 32 + 16
    ("initial-prefill-long", [0], [3000], 8, 2, 64, 16),          # C = 0, many tiles, diagonal everywhere
    ("one-token-no-history", [0, 0], [1, 1], 8, 8, 128, 16),      # output = v_new exactly
])
def test_head_group_shapes(name, C, L, Hq, Hkv, d, P):
    print(f"case: {name}", flush=True)
    b = W.make_batch(C, L, Hq, Hkv, d, P, seed=len(name) * 7 + 1, poison=True)
    db = DevBatch(b)
    out = run(db)
    rows = sample_rows(b, 8, seed=1) if sum(L) > 400 else None
    compare(b, out, rows=rows, label=name)
    if name == "one-token-no-history":
        G = Hq // Hkv
        assert np.array_equal(out.reshape(2, Hq, d), np.repeat(b.v_new, G, axis=1))


@pytest.mark.parametrize("C,L,Hq,Hkv", [
    ([897], [287], 16, 2),                           # 2 K/V streams for 8 dies: pieces, levelling, null items
    ([1355, 407, 542], [618, 147, 63], 8, 1),        # 3 streams of very different weight
    ([1325, 1308, 459, 27], [549, 501, 544, 20], 8, 1),
])
def test_launch_order_with_null_items(C, L, Hq, Hkv):
    """Few K/V streams: the per-die queues differ in length and are padded with null items, which must do nothing."""
    print(f"case: null items C={C} L={L}", flush=True)
    b = W.make_batch(C, L, Hq, Hkv, 128, 16, seed=sum(C) + Hq, poison=True)
    db = DevBatch(b)
    items = A.plan_items(db.cache, b.ctx_len, b.incr_len, b.block_table.shape[1])
    assert (items[:, 1] == 2).any(), "this case is meant to produce null items"
    out = run(db)
    compare(b, out, rows=sample_rows(b, 12, seed=2), label="null items")


@pytest.mark.parametrize("k_mult", [6.0, 16.0])
def test_sharp_logits_exercise_the_reference_maximum(k_mult):
    """Logits with a standard deviation of 6 and 16 (scale 1/sqrt(d) on keys 6x / 16x too large): the row maximum
    keeps rising by more than the slack of the lazily raised reference, in wide tiles, narrow items and across
    key splits, and the softmax is nearly one-hot."""
    print(f"case: sharp logits x{k_mult}", flush=True)
    b = W.make_batch([900, 3000, 0, 517], [300, 1, 130, 9], 16, 4, 128, 16, seed=int(k_mult) + 40, k_mult=k_mult, poison=True)
    db = DevBatch(b)
    out = run(db)
    compare(b, out, rows=sample_rows(b, 24, seed=3), label=f"sharp x{k_mult}")
    out2 = run(DevBatch(b), force_kv_splits=3)
    compare(b, out2, rows=sample_rows(b, 24, seed=3), label=f"sharp x{k_mult}, 3 key splits")


@pytest.mark.parametrize("per_key,jump_every,jump", [(4.0, 0, 0.0), (0.0, 100, 3000.0), (1.0, 37, 400.0)])
def test_logits_rising_along_the_keys_keep_raising_the_reference(per_key, jump_every, jump):
    """Logits that grow with the key position (about +3 per key; steps of ~+2000 every 100 keys, far past the range of
    exp2 in fp32; both): every block needs a new reference, in the step cases the exponentials taken against the old
    one overflow first.  Wide tiles, narrow items and key splits."""
    print(f"case: rising logits {per_key} {jump_every} {jump}", flush=True)
    b = W.make_batch([900, 3000, 0, 517], [300, 1, 130, 9], 16, 4, 128, 16, seed=71, poison=True)
    W.impose_key_ramp(b, per_key, jump_every, jump)
    out = run(DevBatch(b))
    compare(b, out, rows=sample_rows(b, 24, seed=4), label="rising logits")
    out2 = run(DevBatch(b), force_kv_splits=3)
    compare(b, out2, rows=sample_rows(b, 24, seed=4), label="rising logits, 3 key splits")


@pytest.mark.parametrize("Hq,Hkv,d,P", [(8, 2, 64, 32), (6, 2, 64, 16), (32, 1, 128, 32)])
def test_rising_logits_other_geometries(Hq, Hkv, d, P):
    """The same ramp + steps with head dimension 64 (four steps per pipeline iteration instead of eight), G = 3 (idle
    rows in every wave) and G = 32 (one token per wave)."""
    print(f"case: rising logits Hq={Hq} Hkv={Hkv} d={d} P={P}", flush=True)
    b = W.make_batch([700, 1500, 0, 333], [260, 1, 150, 40], Hq, Hkv, d, P, seed=72, poison=True)
    W.impose_key_ramp(b, 1.0, 37, 400.0)
    out = run(DevBatch(b))
    compare(b, out, rows=sample_rows(b, 24, seed=5), label="rising logits, geometry")


def test_more_requests_than_one_append_launch_carries():
    print("case: 300 decode rows + 3 prefill rows", flush=True)
    rng = np.random.default_rng(3)
    C = rng.integers(1, 400, size=303).tolist()
    L = [1] * 300 + [40, 130, 7]
    b = W.make_batch(C, L, 8, 2, 128, 16, seed=77, poison=True)
    db = DevBatch(b)
    out = run(db)
    k_ref, v_ref = oracle.kv_append_reference(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len, b.k_new, b.v_new, b.P)
    assert np.array_equal(from_dev_bits(db.k_pool), k_ref) and np.array_equal(from_dev_bits(db.v_pool), v_ref)
    compare(b, out, label="303 rows")


def test_chunked_prefill_composes_on_the_gpu():
    """One call with L new tokens == a call with L1 followed by a call with L2 over C + L1 (the paper's
    future-work chunked local prefill needs no new kernel)."""
    print("case: chunked prefill", flush=True)
    C, L1, L2 = 700, 190, 333
    b = W.make_batch([C], [L1 + L2], 8, 2, 128, 16, seed=9, poison=True)
    db = DevBatch(b)
    whole = run(db, fn=A.incr_prefill_attn)
    db2 = DevBatch(b)                                            # fresh pools
    o1 = A.incr_prefill_attn(db2.cache, [C], [L1], db2.bt, db2.q[:L1].contiguous(), db2.k_new[:L1].contiguous(),
                             db2.v_new[:L1].contiguous(), block_table_host=b.block_table)
    o2 = A.incr_prefill_attn(db2.cache, [C + L1], [L2], db2.bt, db2.q[L1:].contiguous(), db2.k_new[L1:].contiguous(),
                             db2.v_new[L1:].contiguous(), block_table_host=b.block_table)
    torch.cuda.synchronize()
    parts = np.concatenate([from_dev_bits(o1), from_dev_bits(o2)])
    assert np.array_equal(from_dev_bits(db.k_pool), from_dev_bits(db2.k_pool))      # same final cache image
    assert np.array_equal(from_dev_bits(db.v_pool), from_dev_bits(db2.v_pool))
    compare(b, parts, label="chunked")
    assert np.abs(W.bf16_bits_to_f64(parts) - W.bf16_bits_to_f64(whole)).max() <= 1e-2


def test_three_identical_launches_are_bitwise_equal():
    print("case: determinism", flush=True)
    b = W.make_batch([900, 30, 4000, 0], [1, 200, 1, 64], 16, 2, 128, 16, seed=12, poison=True)
    db = DevBatch(b)
    outs = [run(db) for _ in range(3)]
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[1], outs[2])
    outs = [run(db, force_kv_splits=4) for _ in range(2)]
    assert np.array_equal(outs[0], outs[1])


def test_error_paths_enqueue_nothing():
    print("case: error paths", flush=True)
    b = W.make_batch([100, 50], [20, 1], 8, 2, 128, 16, seed=5)
    db = DevBatch(b)
    k_before = from_dev_bits(db.k_pool).copy()
    out = torch.full_like(db.q, 7.0)
    need = A.workspace_bytes(db.cache, b.ctx_len, b.incr_len, b.block_table.shape[1])
    small = torch.empty(max(need - 256, 16), dtype=torch.uint8, device="cuda")
    with pytest.raises(A.AmpdError) as e:
        A.mixed_batch_attn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q, db.k_new, db.v_new, out=out, workspace=small)
    assert e.value.status == -3
    big = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    with pytest.raises(A.AmpdError) as e:                         # misaligned workspace
        A.mixed_batch_attn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q, db.k_new, db.v_new, out=out, workspace=big[16:])
    assert e.value.status == -3
    bad = b.block_table.copy()
    bad[0, 1] = b.num_pages + 3
    with pytest.raises(A.AmpdError) as e:                         # host mirror catches an out-of-range page
        A.mixed_batch_attn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q, db.k_new, db.v_new, out=out, block_table_host=bad)
    assert e.value.status == -4
    with pytest.raises(A.AmpdError) as e:                         # block table too narrow for C + L
        A.mixed_batch_attn(db.cache, [100, 50], [200, 1], db.bt, db.q, db.k_new, db.v_new, out=out)
    assert e.value.status == -1
    torch.cuda.synchronize()
    assert np.array_equal(from_dev_bits(db.k_pool), k_before), "a rejected call wrote to the cache"
    assert bool((out == 7.0).all()), "a rejected call wrote to the output"
    # all-empty batch is a legal no-op
    A.mixed_batch_attn(db.cache, [5, 6], [0, 0], db.bt, db.q[:0], db.k_new[:0], db.v_new[:0], out=out[:0])
    torch.cuda.synchronize()


def test_runs_on_a_non_default_stream():
    print("case: side stream", flush=True)
    b = W.make_batch([300, 10], [90, 1], 8, 2, 128, 16, seed=15, poison=True)
    db = DevBatch(b)
    ref = run(db)
    db2 = DevBatch(b)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = A.mixed_batch_attn(db2.cache, b.ctx_len, b.incr_len, db2.bt, db2.q, db2.k_new, db2.v_new, stream=s)
    s.synchronize()
    assert np.array_equal(from_dev_bits(out), ref)


def test_many_calls_in_flight_never_wait_for_the_gpu():
    """64 calls enqueued back to back without a synchronisation (more than the staging ring holds at first): every call
    returns in bounded host time, the host stays ahead of the GPU for the whole sequence, and all outputs are equal."""
    import time
    print("case: 64 calls in flight", flush=True)
    A.init()
    Hq, Hkv, d, P, B, Cx, Lx = 32, 8, 128, 16, 8, 8000, 1024
    pages_per = (Cx + Lx + P - 1) // P
    gen = torch.Generator(device="cuda").manual_seed(3)
    rnd = lambda *s: torch.randn(*s, device="cuda", generator=gen).to(torch.bfloat16)
    k_pool, v_pool = rnd(B * pages_per, Hkv, P, d), rnd(B * pages_per, Hkv, P, d)
    bt = torch.randperm(B * pages_per, device="cuda", generator=gen).to(torch.int32).view(B, pages_per).contiguous()
    q, k_new, v_new = rnd(B * Lx, Hq, d), rnd(B * Lx, Hkv, d), rnd(B * Lx, Hkv, d)
    cache = A.KVCache(Hq, Hkv, d, P, k_pool, v_pool, 1.0 / np.sqrt(d))
    C, L = np.full(B, Cx, np.int32), np.full(B, Lx, np.int32)
    ncalls = 64
    ws = [torch.empty(A.workspace_bytes(cache, C, L, pages_per), dtype=torch.uint8, device="cuda") for _ in range(ncalls)]
    outs = [torch.empty_like(q) for _ in range(ncalls)]
    call = lambda i: A.mixed_batch_attn(cache, C, L, bt, q, k_new, v_new, out=outs[i], workspace=ws[i])
    for i in range(3):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    host = []
    e0.record()
    t_begin = time.perf_counter()
    for i in range(ncalls):
        t0 = time.perf_counter()
        call(i)
        host.append(time.perf_counter() - t0)
    t_host = time.perf_counter() - t_begin
    e1.record()
    torch.cuda.synchronize()
    t_gpu = e0.elapsed_time(e1) * 1e-3
    print(f"  host {t_host * 1e3:.1f} ms for {ncalls} calls (slowest {max(host) * 1e3:.2f} ms), GPU {t_gpu * 1e3:.1f} ms", flush=True)
    assert t_gpu > 0.03, "the case is meant to keep the GPU busy for tens of milliseconds"
    assert t_host < 0.5 * t_gpu, "the host did not stay ahead of the GPU: some call waited"
    assert max(host) < 0.25 * t_gpu, "one call took a large part of the whole sequence"
    for i in range(1, ncalls):
        assert torch.equal(outs[i], outs[0])


def test_two_host_threads_on_two_streams_share_the_library():
    """Two host threads, each with its own stream, workspace and batch, call the library at the same time (ctypes releases
    the interpreter lock during a call): the staging ring and its sequence numbers are shared under a mutex, the last
    plan is kept per thread.  Every output must equal the single-threaded result of its batch bit for bit."""
    import threading
    print("case: two host threads", flush=True)
    batches = [W.make_batch([900, 40, 2000], [130, 1, 260], 16, 4, 128, 16, seed=91, poison=True),
               W.make_batch([3000, 3100, 2900, 5], [1, 1, 1, 70], 16, 4, 128, 16, seed=92, poison=True)]
    refs = [run(DevBatch(b)) for b in batches]
    dbs = [DevBatch(b) for b in batches]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ncalls = 60
    outs = [[torch.empty_like(db.q) for _ in range(ncalls)] for db in dbs]
    wss = [torch.empty(A.workspace_bytes(db.cache, b.ctx_len, b.incr_len, db.bt.shape[1]), dtype=torch.uint8, device="cuda")
           for db, b in zip(dbs, batches)]
    errors = []
    torch.cuda.synchronize()

    def worker(t):
        try:
            b, db = batches[t], dbs[t]
            for i in range(ncalls):
                A.mixed_batch_attn(db.cache, b.ctx_len, b.incr_len, db.bt, db.q, db.k_new, db.v_new, out=outs[t][i],
                                   workspace=wss[t], stream=streams[t])
            streams[t].synchronize()
        except Exception as e:            # noqa: BLE001 (reported by the main thread)
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for t in range(2):
        for i in range(ncalls):
            assert np.array_equal(from_dev_bits(outs[t][i]), refs[t]), f"thread {t} call {i}"
