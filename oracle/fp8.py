"""TEST INFRASTRUCTURE -- not the product.

Reference for the 8-bit KV-cache variant (benchmark configuration 5; the paper itself says
nothing about cache precision, so every rule here is this build's reading, listed in the
design notes):

* code format: OCP 8-bit float E4M3 ("e4m3fn": bias 7, no infinities, S.1111.111 = NaN,
  largest finite 448), encoded by round-to-nearest, ties to the even code, sign kept;
* one power-of-two scale 2^e per (page, KV head), separately for K and V, stored as fp32;
  e = the smallest integer with amax <= 448 * 2^e, clamped to [E_MIN, E_MAX];
* an append into a page that already holds tokens never lowers the page's exponent; if the
  new tokens need a larger one the old codes are re-encoded: code' = enc(dec(code) * 2^(e_old-e));
* stored value = dec(code) * 2^e.

Pinned by tests/test_oracle_fp8.py: exhaustive decode/encode round trip, tie cases, scale
covariance under 2^k, saturation bound, one-at-a-time vs all-at-once appends.
"""
from __future__ import annotations

import math

import numpy as np

E_MIN, E_MAX = -40, 119


def e4m3_decode(code) -> np.ndarray:
    """Value of every code (array of uint8) as float64; NaN for S.1111.111."""
    c = np.asarray(code, dtype=np.int64)
    s = (c >> 7) & 1
    e = (c >> 3) & 15
    m = c & 7
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    sub = (m / 8.0) * 2.0 ** -6
    v = np.where(e == 0, sub, normal)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return np.where(s == 1, -v, v)


_POS = e4m3_decode(np.arange(0, 0x7F))          # 127 non-negative finite values, ascending


def e4m3_encode_rne(x) -> np.ndarray:
    """Nearest finite E4M3 value, ties to the even code, saturating at +-448; sign kept
    (so -0.0 and negative values that round to zero give 0x80)."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    hi = np.clip(np.searchsorted(_POS, a, side="left"), 0, 0x7E)      # first value >= a
    lo = np.clip(hi - 1, 0, 0x7E)
    d_hi = np.abs(_POS[hi] - a)
    d_lo = np.abs(a - _POS[lo])
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi)
    code = np.where(a >= 448.0, 0x7E, code)
    sign = np.signbit(x)
    return (code | np.where(sign, 0x80, 0)).astype(np.uint8)


def scale_exponent(amax: float) -> int:
    """Smallest integer e with amax <= 448 * 2^e, clamped to [E_MIN, E_MAX]."""
    if not (amax > 0.0):
        return E_MIN
    m, x = math.frexp(amax)                     # amax = m * 2^x, m in [0.5, 1);  448 = 0.875 * 2^9
    e = x - 9 if m <= 0.875 else x - 8
    return max(E_MIN, min(E_MAX, e))


def _bf16_to_f64(bits):
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def fp8_append_reference(codes, scales, block_table, ctx_len, incr_len, x_new, P, in_place=False):
    """Append bf16 rows x_new [sumL, Hkv, d] into an 8-bit pool.

    codes [num_pages, Hkv, P, d] uint8 and scales [num_pages, Hkv] float32 are copied, the
    copies updated page by page in the order described in the module header, and returned.
    in_place=True updates the given arrays instead (a long replay would otherwise copy the
    whole pool at every step); the arithmetic is the same."""
    if not in_place:
        codes = np.array(codes, copy=True)
        scales = np.array(scales, dtype=np.float32, copy=True)
    assert codes.dtype == np.uint8 and scales.dtype == np.float32
    Hkv = codes.shape[1]
    off = 0
    for r in range(len(ctx_len)):
        C, L = int(ctx_len[r]), int(incr_len[r])
        if L == 0:
            continue
        x = _bf16_to_f64(x_new[off:off + L])                      # [L, Hkv, d]
        for pi in range(C // P, (C + L - 1) // P + 1):
            page = int(block_table[r][pi])
            t0, t1 = max(C, pi * P), min(C + L, (pi + 1) * P)
            n_old = max(0, C - pi * P)
            for h in range(Hkv):
                xn = x[t0 - C:t1 - C, h, :]
                e = scale_exponent(float(np.abs(xn).max()))
                if n_old > 0:
                    e_old = int(round(math.log2(float(scales[page, h]))))
                    if e > e_old:
                        old = e4m3_decode(codes[page, h, :n_old, :]) * 2.0 ** (e_old - e)
                        codes[page, h, :n_old, :] = e4m3_encode_rne(old)
                    else:
                        e = e_old
                codes[page, h, t0 - pi * P:t1 - pi * P, :] = e4m3_encode_rne(xn * 2.0 ** (-e))
                scales[page, h] = np.float32(2.0 ** e)
        off += L
    return codes, scales


def fp8_dequant_request(codes, scales, table_row, n_tokens, P):
    """Contiguous fp64 [n, Hkv, d] copy of a request's stored values dec(code) * scale."""
    n_pages = (n_tokens + P - 1) // P
    pages = np.asarray(table_row[:n_pages], dtype=np.int64)
    v = e4m3_decode(codes[pages]) * scales[pages].astype(np.float64)[:, :, None, None]
    v = np.transpose(v, (0, 2, 1, 3)).reshape(n_pages * P, codes.shape[1], codes.shape[3])
    return np.ascontiguousarray(v[:n_tokens])
