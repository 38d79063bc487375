"""TEST INFRASTRUCTURE -- not the product.

fp64 definitions of: the paged KV append (an index map), incremental-prefill attention
(a wrapper that undoes the paging with a plain gather and calls the C definition in
attn_oracle.c), a pure-Python brute force for tiny shapes, and the split-KV combine rule.

Passages followed: a prefill task has history length l_hist and incremental length l_incr,
with initial prefill the l_hist = 0 case (paper Section 3, performance model T_pre); the
decode worker merges the incremental KV into the history KV it already stores (Section 3,
"Remote execution", footnote) and then holds all KV of the request and keeps decoding
(Section 3, step 4).  Layout readings (the paper fixes none): int32 block table of physical
page ids; K and V pools [num_pages][Hkv][P][d]; token t of request r lives in page
block_table[r][t // P], slot t % P.

Parity status: pinned by tests/test_oracle_pins.py (closed forms, brute force, a library
attention routine, invariants).  The paper prints no numeric value for this path.
"""
from __future__ import annotations

import ctypes
import math

import numpy as np

from .build import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.ampd_oracle_attn.restype = ctypes.c_int
        lib.ampd_oracle_attn.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_double, ip, ctypes.c_int, dp, dp]
        lib.ampd_oracle_probs.restype = ctypes.c_int
        lib.ampd_oracle_probs.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_int, dp]
        lib.ampd_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def oracle_threads() -> int:
    return int(_load().ampd_oracle_num_threads())


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _as_f64(x):
    x = np.asarray(x)
    return bf16_to_f64(x) if x.dtype == np.uint16 else np.ascontiguousarray(x, dtype=np.float64)


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


# ----------------------------------------------------------------------------- paging

def gather_request_kv(pool: np.ndarray, table_row: np.ndarray, n_tokens: int, P: int) -> np.ndarray:
    """Undo the paging: tokens 0..n_tokens-1 of one request as a contiguous [n, Hkv, d] array.
    pool is [num_pages, Hkv, P, d] (any dtype)."""
    n_pages = (n_tokens + P - 1) // P
    if n_pages == 0:
        return np.empty((0, pool.shape[1], pool.shape[3]), dtype=pool.dtype)
    pages = np.asarray(table_row[:n_pages], dtype=np.int64)
    assert (pages >= 0).all() and (pages < pool.shape[0]).all(), "block table entry out of range"
    x = pool[pages]                                   # [n_pages, Hkv, P, d]
    x = np.transpose(x, (0, 2, 1, 3)).reshape(n_pages * P, pool.shape[1], pool.shape[3])
    return np.ascontiguousarray(x[:n_tokens])


def kv_append_reference(k_pool, v_pool, block_table, ctx_len, incr_len, k_new, v_new, P):
    """The append as a plain index map, one element group at a time, on copies of the pools.
    Token i of request r (packed row off_r + i) goes to absolute position t = C_r + i:
    page block_table[r][t // P], slot t % P, for every KV head.  Returns (k_pool', v_pool')."""
    k_out = np.array(k_pool, copy=True)
    v_out = np.array(v_pool, copy=True)
    off = 0
    for r in range(len(ctx_len)):
        C, L = int(ctx_len[r]), int(incr_len[r])
        for i in range(L):
            t = C + i
            page = int(block_table[r][t // P])
            slot = t % P
            assert 0 <= page < k_out.shape[0]
            k_out[page, :, slot, :] = k_new[off + i]
            v_out[page, :, slot, :] = v_new[off + i]
        off += L
    return k_out, v_out


# ----------------------------------------------------------------------------- attention

def attn_oracle_request(q, K, V, C, L, scale, rows=None, want_psum=False):
    """One request.  q [L,Hq,d], K/V [C+L,Hkv,d] (fp64 or bf16 bits).  rows: optional new-token
    indices to compute.  Returns out [nrows,Hq,d] fp64 (and psum [nrows,Hq])."""
    q, K, V = _as_f64(q), _as_f64(K), _as_f64(V)
    L_, Hq, d = q.shape
    assert L_ == L and K.shape[0] == C + L and V.shape == K.shape
    Hkv = K.shape[1]
    if rows is None:
        rows_arr, nrows, rp = None, L, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32)
        nrows = rows_arr.shape[0]
        rp = rows_arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
    out = np.zeros((nrows, Hq, d), dtype=np.float64)
    psum = np.zeros((nrows, Hq), dtype=np.float64)
    rc = _load().ampd_oracle_attn(_dptr(q), _dptr(K), _dptr(V), C, L, Hq, Hkv, d, float(scale),
                                  rp, nrows, _dptr(out), _dptr(psum))
    if rc != 0:
        raise ValueError("ampd_oracle_attn rejected its arguments")
    return (out, psum) if want_psum else out


def attn_probs(q, K, C, L, scale, i, hq):
    """Normalised probabilities p[0..C+i] of one (query, head)."""
    q, K = _as_f64(q), _as_f64(K)
    _, Hq, d = q.shape
    p = np.zeros(C + i + 1, dtype=np.float64)
    rc = _load().ampd_oracle_probs(_dptr(q), _dptr(K), C, L, Hq, K.shape[1], d, float(scale), i, hq, _dptr(p))
    if rc != 0:
        raise ValueError("ampd_oracle_probs rejected its arguments")
    return p


def attn_oracle(k_pool, v_pool, block_table, ctx_len, incr_len, q, k_new, v_new, P, scale, rows=None):
    """Whole batch: append-then-attend.  Pools hold the history only; the new tokens are taken
    from k_new / v_new and placed at positions C_r .. C_r+L_r-1 of the contiguous copy.
    rows: optional dict {request: array of new-token indices}; requests not in the dict are
    skipped.  Returns a list (one entry per request, None if skipped) of fp64 [nrows,Hq,d]."""
    outs = []
    off = 0
    for r in range(len(ctx_len)):
        C, L = int(ctx_len[r]), int(incr_len[r])
        sel = None if rows is None else rows.get(r)
        if L == 0 or (rows is not None and sel is None):
            outs.append(None if L else np.zeros((0, q.shape[1], q.shape[2])))
            off += L
            continue
        Kh = gather_request_kv(k_pool, block_table[r], C, P)
        Vh = gather_request_kv(v_pool, block_table[r], C, P)
        K = np.concatenate([_as_f64(Kh), _as_f64(k_new[off:off + L])], axis=0)
        V = np.concatenate([_as_f64(Vh), _as_f64(v_new[off:off + L])], axis=0)
        outs.append(attn_oracle_request(q[off:off + L], K, V, C, L, scale, rows=sel))
        off += L
    return outs


def attn_bruteforce(q, K, V, C, L, scale):
    """Pure-Python loops with math.exp, independent of the C code; tiny shapes only."""
    q, K, V = _as_f64(q), _as_f64(K), _as_f64(V)
    _, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.zeros((L, Hq, d))
    for i in range(L):
        for h in range(Hq):
            kvh = h // G
            logits = [scale * sum(q[i, h, x] * K[j, kvh, x] for x in range(d)) for j in range(C + i + 1)]
            mx = max(logits)
            w = [math.exp(s - mx) for s in logits]
            z = sum(w)
            for j, wj in enumerate(w):
                for x in range(d):
                    out[i, h, x] += (wj / z) * V[j, kvh, x]
    return out


# ----------------------------------------------------------------------------- split-KV combine

def partial_attention(qv, K, V, scale):
    """Un-normalised attention of one query vector over a key sub-range:
    returns (m, l, O~) with m = max logit, l = sum exp(s-m), O~ = sum exp(s-m) V."""
    s = scale * (K @ qv)
    m = s.max() if s.size else -np.inf
    w = np.exp(s - m) if s.size else np.zeros(0)
    return m, w.sum(), w @ V if s.size else np.zeros(V.shape[1])


def combine_partials(parts):
    """Merge partial results over a partition of the key range:
    m = max m_s; l = sum l_s e^{m_s-m}; O = sum O~_s e^{m_s-m} / l."""
    m = max(p[0] for p in parts)
    l = sum(p[1] * math.exp(p[0] - m) for p in parts if p[1] > 0)
    O = sum(p[2] * math.exp(p[0] - m) for p in parts if p[1] > 0)
    return O / l
