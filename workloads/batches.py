"""Batch generators: lengths, block tables and bf16 tensors for the benchmark configurations."""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 260214516
NAN_BF16 = np.uint16(0x7FC1)          # a quiet-NaN bf16 pattern used to poison unused memory
_CHUNK = 1 << 22                      # elements per independently seeded chunk


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to float64."""
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _normal_bf16(shape, seed: int, stream: int, mult: float = 1.0) -> np.ndarray:
    """N(0,1)*mult as bf16 bits.  Chunked so that the result does not depend on thread count."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def work(c):
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, c])))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if mult != 1.0:
            x *= np.float32(mult)
        out[lo:hi] = f32_to_bf16_bits(x)

    if nchunks <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(work, range(nchunks)))
    return out.reshape(shape)


@dataclass
class Batch:
    """One batch of rows (C_r cached tokens, L_r new tokens) over a paged bf16 KV pool.

    k_pool / v_pool hold bf16 bit patterns laid out [num_pages, Hkv, P, d]; the history of
    request r occupies logical positions 0..C_r-1 reached through block_table[r].  Pages and
    slots that hold no history are poisoned with NaN patterns when ``poison`` was requested,
    else hold arbitrary finite values.
    """
    Hq: int
    Hkv: int
    d: int
    P: int
    scale: float
    ctx_len: np.ndarray
    incr_len: np.ndarray
    block_table: np.ndarray
    num_pages: int
    k_pool: np.ndarray
    v_pool: np.ndarray
    q: np.ndarray
    k_new: np.ndarray
    v_new: np.ndarray
    name: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def num_reqs(self) -> int:
        return int(self.ctx_len.shape[0])

    @property
    def row_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.incr_len)]).astype(np.int64)

    def flops(self) -> int:
        """Algorithmic attention FLOPs: 4*d*Hq*(L*C + L*(L+1)/2) summed over rows."""
        C = self.ctx_len.astype(np.int64)
        L = self.incr_len.astype(np.int64)
        return int((4 * self.d * self.Hq * (L * C + L * (L + 1) // 2)).sum())

    def algorithmic_bytes(self, kv_bytes: int = 2) -> int:
        """Bytes the method must move once: K,V of every visible token, new K/V in and out,
        Q in, O out, block table (and scales for an 8-bit cache)."""
        C = self.ctx_len.astype(np.int64)
        L = self.incr_len.astype(np.int64)
        T = C + L
        pages = (T + self.P - 1) // self.P
        b = 2 * T * self.Hkv * self.d * kv_bytes
        b = b + 2 * L * self.Hkv * self.d * (2 + kv_bytes)
        b = b + 2 * L * self.Hq * self.d * 2
        b = b + 4 * pages
        if kv_bytes == 1:
            b = b + 2 * 4 * self.Hkv * pages
        return int(b.sum())


def make_batch(ctx_len, incr_len, Hq, Hkv, d, P, *, seed, scale=None, k_mult=1.0,
               pool_slack=0.10, poison=False, permute=True, name="", pool_pages=None) -> Batch:
    """Build a batch.  Draw order: block-table permutation, Q, K pool, V pool, K_new, V_new."""
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    incr_len = np.asarray(incr_len, dtype=np.int32)
    B = ctx_len.shape[0]
    T = ctx_len.astype(np.int64) + incr_len
    pages_per = ((T + P - 1) // P).astype(np.int64)
    used = int(pages_per.sum())
    num_pages = int(pool_pages) if pool_pages is not None else max(1, int(math.ceil(used * (1.0 + pool_slack))))
    assert num_pages >= used
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0])))
    perm = g.permutation(num_pages).astype(np.int32) if permute else np.arange(num_pages, dtype=np.int32)
    max_pages = max(1, int(pages_per.max())) if B else 1
    bt = np.full((B, max_pages), -1, dtype=np.int32)
    o = 0
    for r in range(B):
        n = int(pages_per[r])
        bt[r, :n] = perm[o:o + n]
        o += n
    sumL = int(incr_len.sum())
    q = _normal_bf16((sumL, Hq, d), seed, 1)
    k_pool = _normal_bf16((num_pages, Hkv, P, d), seed, 2, k_mult)
    v_pool = _normal_bf16((num_pages, Hkv, P, d), seed, 3)
    k_new = _normal_bf16((sumL, Hkv, d), seed, 4, k_mult)
    v_new = _normal_bf16((sumL, Hkv, d), seed, 5)
    if poison:
        hist = np.zeros((num_pages, P), dtype=bool)
        for r in range(B):
            c = int(ctx_len[r])
            full, rem = divmod(c, P)
            hist[bt[r, :full]] = True
            if rem:
                hist[bt[r, full], :rem] = True
        mask = ~hist
        k_pool[np.broadcast_to(mask[:, None, :, None], k_pool.shape)] = NAN_BF16
        v_pool[np.broadcast_to(mask[:, None, :, None], v_pool.shape)] = NAN_BF16
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    return Batch(Hq, Hkv, d, P, float(np.float32(scale)), ctx_len, incr_len, bt, num_pages,
                 k_pool, v_pool, q, k_new, v_new, name=name, meta={"seed": seed, "poison": poison})



def impose_key_ramp(b: Batch, per_key: float, jump_every: int = 0, jump: float = 0.0, q0: float = 8.0) -> Batch:
    """Overwrite channel 0 of every query with q0 and channel 0 of the key at token position t (cached or new) with
    per_key * t + jump * (t // jump_every), in place: logits then rise along the key axis, steadily and/or in steps,
    on top of the random part from the other channels."""
    def level(t):
        t = np.asarray(t, dtype=np.float64)
        v = per_key * t
        if jump_every:
            v = v + jump * np.floor(t / jump_every)
        return f32_to_bf16_bits(v.astype(np.float32))
    b.q[..., 0] = f32_to_bf16_bits(np.full(b.q.shape[:-1], q0, dtype=np.float32))
    off = b.row_offsets
    for r in range(b.num_reqs):
        c, L = int(b.ctx_len[r]), int(b.incr_len[r])
        t = np.arange(c)
        b.k_pool[b.block_table[r, t // b.P], :, t % b.P, 0] = level(t)[:, None]
        b.k_new[off[r]:off[r] + L, :, 0] = level(c + np.arange(L))[:, None]
    return b

# Layer shapes of the five benchmark configurations.
CONFIG_SHAPES = {
    1: dict(Hq=8, Hkv=2, d=64, P=16),
    2: dict(Hq=32, Hkv=8, d=128, P=16),
    3: dict(Hq=64, Hkv=8, d=128, P=16),
    4: dict(Hq=8, Hkv=1, d=128, P=32),
    5: dict(Hq=32, Hkv=8, d=128, P=16),
}


def config_lengths(k: int, seed: int | None = None, part: str = "all"):
    """(ctx_len, incr_len) of configuration k (1..4).  ``part`` selects a sub-batch of
    configuration 3 ("decode", "prefill") or the decode step that follows configuration 4
    ("decode": L=1 over C+4096)."""
    seed = BASE_SEED + k if seed is None else seed
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 100])))
    if k == 1:
        return np.array([256], np.int32), np.array([32], np.int32)
    if k == 2:
        C = g.integers(1024, 8192, size=16, endpoint=True)
        L = g.integers(64, 1024, size=16, endpoint=True)
        return C.astype(np.int32), L.astype(np.int32)
    if k == 3:
        Cd = g.integers(2048, 16384, size=96, endpoint=True)
        Lp = g.integers(256, 2048, size=8, endpoint=True)
        Cp = g.integers(1024, 8192, size=8, endpoint=True)
        if part == "decode":
            return Cd.astype(np.int32), np.ones(96, np.int32)
        if part == "prefill":
            return Cp.astype(np.int32), Lp.astype(np.int32)
        # prefill rows are spread among the decode rows (every 12th row)
        C = np.empty(104, np.int64)
        L = np.empty(104, np.int64)
        pos = set(range(6, 104, 13))
        di = pi = 0
        for r in range(104):
            if r in pos:
                C[r], L[r] = Cp[pi], Lp[pi]
                pi += 1
            else:
                C[r], L[r] = Cd[di], 1
                di += 1
        return C.astype(np.int32), L.astype(np.int32)
    if k == 4:
        C = g.integers(32768, 65536, size=4, endpoint=True)
        if part == "decode":
            return (C + 4096).astype(np.int32), np.ones(4, np.int32)
        return C.astype(np.int32), np.full(4, 4096, np.int32)
    raise ValueError("configuration 5 is a trace; see workloads.trace")


def make_config(k: int, *, seed: int | None = None, part: str = "all", poison=False, shrink: int = 1) -> Batch:
    """Benchmark configuration k.  ``shrink`` divides every length (for CPU-sized tests of the
    same shape family); shrink=1 is the full configuration."""
    seed = BASE_SEED + k if seed is None else seed
    C, L = config_lengths(k, seed, part)
    if shrink > 1:
        C = np.maximum(C // shrink, 0).astype(np.int32)
        L = np.maximum(L // shrink, 1).astype(np.int32)
    sh = CONFIG_SHAPES[k]
    permute = True
    pool_pages = 32 if (k == 1 and shrink == 1) else None
    return make_batch(C, L, sh["Hq"], sh["Hkv"], sh["d"], sh["P"], seed=seed,
                      k_mult=0.5 if k == 2 else 1.0, poison=poison, permute=permute,
                      name=f"cfg{k}" + ("" if part == "all" else f"-{part}") + (f"/s{shrink}" if shrink > 1 else ""),
                      pool_pages=pool_pages)
