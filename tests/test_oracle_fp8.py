"""Pins of the 8-bit KV reference (E4M3 codes + power-of-two page scales).  CPU only."""
import math
import struct

import numpy as np
import pytest

import oracle
from oracle import fp8 as F
import workloads as W


def test_decode_table_matches_the_format_definition():
    # spot values fixed by the OCP E4M3 definition (bias 7, 3 mantissa bits, no infinities)
    d = oracle.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert d[0x00] == 0.0 and d[0x80] == 0.0 and np.signbit(d[0x80])
    assert d[0x01] == 2.0 ** -9 and d[0x07] == 7 * 2.0 ** -9            # subnormals
    assert d[0x08] == 2.0 ** -6 and d[0x38] == 1.0 and d[0x3C] == 1.5
    assert d[0x7E] == 448.0 and d[0xFE] == -448.0 and np.isnan(d[0x7F]) and np.isnan(d[0xFF])
    finite = d[:0x7F]
    assert np.all(np.diff(finite) > 0)                                   # strictly increasing
    # independent construction: every finite value is m * 2^k with integer m < 16
    for c in range(1, 0x7F):
        m, e = math.frexp(finite[c])
        assert (m * 16) == int(m * 16)


def test_encode_round_trips_every_finite_code():
    c = np.array([x for x in range(256) if x & 0x7F != 0x7F], dtype=np.uint8)
    assert np.array_equal(oracle.e4m3_encode_rne(oracle.e4m3_decode(c)), c)


def test_encode_rounds_to_nearest_ties_to_even():
    d = oracle.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    for c in range(0x7E):
        lo, hi = d[c], d[c + 1]
        mid = 0.5 * (lo + hi)
        even = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode_rne(mid) == even
        assert oracle.e4m3_encode_rne(np.nextafter(mid, 0.0)) == c
        assert oracle.e4m3_encode_rne(np.nextafter(mid, 1e9)) == c + 1
        assert oracle.e4m3_encode_rne(-mid) == (even | 0x80)
    assert oracle.e4m3_encode_rne(1e9) == 0x7E and oracle.e4m3_encode_rne(-500.0) == 0xFE   # saturates
    assert oracle.e4m3_encode_rne(-0.0) == 0x80 and oracle.e4m3_encode_rne(-1e-9) == 0x80


def test_encode_error_bound():
    x = np.random.default_rng(0).uniform(-448, 448, 20000)
    err = np.abs(oracle.e4m3_decode(oracle.e4m3_encode_rne(x)) - x)
    # half an ulp: 2^-4 relative for normals, 2^-10 absolute in the subnormal range
    assert np.all(err <= np.maximum(np.abs(x) * 2.0 ** -4, 2.0 ** -10) + 1e-18)


def test_scale_exponent_is_minimal_and_covariant():
    for amax in [448.0, 448.0001, 447.9, 1.0, 0.875, 0.8751, 3.5, 3.51, 1e-3, 7e4, 2.0 ** -20]:
        e = oracle.scale_exponent(amax)
        assert amax <= 448.0 * 2.0 ** e and amax > 448.0 * 2.0 ** (e - 1)
        for k in (-5, 3, 11):
            assert oracle.scale_exponent(amax * 2.0 ** k) == e + k
    assert oracle.scale_exponent(0.0) == F.E_MIN and oracle.scale_exponent(1e-30) == F.E_MIN


def _mk(seed, C, L, P=4, Hkv=2, d=8, mult=1.0):
    b = W.make_batch(C, L, 2 * Hkv, Hkv, d, P, seed=seed)
    x = W.bf16_bits_to_f64(b.k_new) * mult
    return b, W.f32_to_bf16_bits(x.astype(np.float32))


def test_append_quantises_within_half_ulp_of_page_amax_and_keeps_other_bytes():
    b, xn = _mk(1, [0, 0], [9, 5])
    codes = np.full(b.k_pool.shape, 0xAB, np.uint8)
    scales = np.full((b.num_pages, b.Hkv), 123.0, np.float32)
    c2, s2 = oracle.fp8_append_reference(codes, scales, b.block_table, b.ctx_len, b.incr_len, xn, b.P)
    off = b.row_offsets
    touched = np.zeros(codes.shape, bool)
    for r in range(2):
        L = int(b.incr_len[r])
        got = oracle.fp8_dequant_request(c2, s2, b.block_table[r], L, b.P)
        want = W.bf16_bits_to_f64(xn[off[r]:off[r + 1]])
        for t in range(L):
            page = b.block_table[r, t // b.P]
            touched[page, :, t % b.P, :] = True
            for h in range(b.Hkv):
                sc = float(s2[page, h])
                assert math.log2(sc) == int(math.log2(sc))                     # power of two
                assert np.all(np.abs(got[t, h] - want[t, h]) <= np.maximum(np.abs(want[t, h]) * 2.0 ** -4, sc * 2.0 ** -10))
    assert np.all(c2[~touched] == 0xAB)
    used = np.unique(b.block_table[b.block_table >= 0])
    unused = np.setdiff1d(np.arange(b.num_pages), used)
    assert np.all(s2[unused] == 123.0)


def test_scaling_inputs_by_power_of_two_shifts_scales_only():
    b, xn = _mk(2, [0], [11])
    b2, xn8 = _mk(2, [0], [11], mult=8.0)
    z = np.zeros(b.k_pool.shape, np.uint8); s = np.ones((b.num_pages, b.Hkv), np.float32)
    c1, s1 = oracle.fp8_append_reference(z, s, b.block_table, b.ctx_len, b.incr_len, xn, b.P)
    c8, s8 = oracle.fp8_append_reference(z, s, b.block_table, b.ctx_len, b.incr_len, xn8, b.P)
    pages = b.block_table[0, :3]
    assert np.array_equal(c1, c8) and np.array_equal(s8[pages], s1[pages] * 8)


def test_incremental_append_raises_scale_and_requantises_old_slots():
    P, Hkv, d = 4, 1, 4
    bt = np.array([[0]], np.int32)
    small = W.f32_to_bf16_bits(np.array([[[1.0, 0.5, 0.25, 0.40625]]], np.float32))      # amax 1 -> e=-8
    big = W.f32_to_bf16_bits(np.array([[[64.0, 3.0, -2.0, 1.0]]], np.float32))           # amax 64 -> e=-2
    z = np.zeros((1, Hkv, P, d), np.uint8); s = np.zeros((1, Hkv), np.float32)
    c1, s1 = oracle.fp8_append_reference(z, s, bt, [0], [1], small, P)
    assert s1[0, 0] == 2.0 ** -8
    assert np.array_equal(oracle.e4m3_decode(c1[0, 0, 0]) * 2.0 ** -8, [1.0, 0.5, 0.25, 0.40625])   # exact
    c2, s2 = oracle.fp8_append_reference(c1, s1, bt, [1], [1], big, P)
    assert s2[0, 0] == 2.0 ** -2
    # old slot: 1.0/2^-2 = 4 exact; 0.40625/2^-2 = 1.625 exact in e4m3; all still exact here
    assert np.array_equal(oracle.e4m3_decode(c2[0, 0, 0]) * 2.0 ** -2, [1.0, 0.5, 0.25, 0.40625])
    assert np.array_equal(oracle.e4m3_decode(c2[0, 0, 1]) * 2.0 ** -2, [64.0, 3.0, -2.0, 1.0])
    # a later small token does not lower the scale
    c3, s3 = oracle.fp8_append_reference(c2, s2, bt, [2], [1], small, P)
    assert s3[0, 0] == 2.0 ** -2 and np.array_equal(c3[0, 0, :2], c2[0, 0, :2])
    # re-issuing the same append is idempotent
    c4, s4 = oracle.fp8_append_reference(c3, s3, bt, [2], [1], small, P)
    assert np.array_equal(c4, c3) and np.array_equal(s4, s3)


def test_one_at_a_time_equals_all_at_once_when_nothing_falls_into_subnormals():
    rng = np.random.default_rng(5)
    P, Hkv, d, n = 8, 2, 16, 8
    # values with 3 significant bits spanning 2 octaves: every requantisation is an exact shift
    mant = rng.integers(8, 16, size=(n, Hkv, d)) / 8.0
    x = mant * 2.0 ** rng.integers(0, 3, size=(n, Hkv, d)) * rng.choice([-1.0, 1.0], size=(n, Hkv, d))
    xb = W.f32_to_bf16_bits(x.astype(np.float32))
    bt = np.array([[3]], np.int32)
    z = np.zeros((5, Hkv, P, d), np.uint8); s = np.zeros((5, Hkv), np.float32)
    ca, sa = oracle.fp8_append_reference(z, s, bt, [0], [n], xb, P)
    c, sc = z, s
    for t in range(n):
        c, sc = oracle.fp8_append_reference(c, sc, bt, [t], [1], xb[t:t + 1], P)
    assert np.array_equal(c, ca) and np.array_equal(sc, sa)
    assert np.array_equal(oracle.fp8_dequant_request(ca, sa, bt[0], n, P), x)   # and it is lossless here
