"""The piecewise alpha-beta fit (host code): recovers exact piecewise-linear data, and its size
functions match the closed forms used by the benchmark."""
import numpy as np
import pytest

from paper_2602_14516_amd.perf_model import (fit_piecewise_alpha_beta, fit_alpha_beta_family, prefill_flops,
                                              decode_bytes)


def test_fit_recovers_a_piecewise_linear_function():
    x = np.concatenate([np.linspace(1, 9, 9), np.linspace(20, 90, 8), np.linspace(200, 900, 8)])
    t = np.where(x < 10, 5 + 0.1 * x, np.where(x < 100, 4 + 0.2 * x, 14 + 0.1 * x))
    m = fit_piecewise_alpha_beta(x, t, knots=[10, 100])
    np.testing.assert_allclose(m.alpha, [5, 4, 14], atol=1e-9)
    np.testing.assert_allclose(m.beta, [0.1, 0.2, 0.1], atol=1e-9)
    assert m.rel_error(x, t).max() < 1e-12
    np.testing.assert_allclose([m(5.0), m(50.0), m(500.0)], [5.5, 14.0, 64.0], rtol=1e-12)


def test_fit_with_default_knots_and_noise_stays_close():
    rng = np.random.default_rng(0)
    x = np.exp(rng.uniform(np.log(1e6), np.log(1e12), 200))
    t = 30e-6 + x / 1e15 * (1 + 0.02 * rng.standard_normal(200))
    m = fit_piecewise_alpha_beta(x, t, segments=3)
    assert np.median(m.rel_error(x, t)) < 0.03
    # a segment without data inherits a neighbour
    m2 = fit_piecewise_alpha_beta(np.array([1.0, 2.0, 3.0]), np.array([2.0, 3.0, 4.0]), knots=[10.0])
    np.testing.assert_allclose(m2(100.0), 101.0, rtol=1e-12)


def test_size_functions():
    # one request, l_hist 3, l_incr 2, Hq 4, d 8: pairs = 2*3 + 3 = 9 -> 4*8*4*9
    assert prefill_flops(3, 2, 4, 8) == 4 * 8 * 4 * 9
    assert decode_bytes(100, 2, 8, 2, 16) == 2 * 102 * 2 * 16 * 2 + 2 * 2 * 2 * 16 * 4 + 2 * 2 * 8 * 16 * 2


def test_family_of_lines_recovers_each_bucket_and_interpolates():
    buckets = np.repeat([16.0, 256.0, 4096.0], 4)
    size = np.tile([0.0, 1e3, 1e4, 1e5], 3)
    a = {16.0: 1.0, 256.0: 2.0, 4096.0: 4.0}
    b = {16.0: 1e-3, 256.0: 2e-3, 4096.0: 8e-3}
    t = np.array([a[k] + b[k] * x for k, x in zip(buckets, size)])
    fam = fit_alpha_beta_family(buckets, size, t)
    np.testing.assert_allclose(fam(buckets, size), t, rtol=1e-9)
    # halfway (in log) between 16 and 256 is 64: the mean of the two lines
    np.testing.assert_allclose(fam(64.0, 1e4), 0.5 * ((1 + 10) + (2 + 20)), rtol=1e-9)
    np.testing.assert_allclose(fam(1.0, 1e3), 1 + 1.0, rtol=1e-9)            # clamped below the first bucket


def test_committed_cost_model_is_what_the_script_writes_and_what_the_simulator_reads():
    """mi355x_cost_model.json holds the sweep it was fitted from; refitting those points reproduces its lines, and the
    simulator's constants are the file's (nothing is typed in by hand)."""
    from paper_2602_14516_amd import simulator as S
    from paper_2602_14516_amd.perf_model import load_cost_model, LINK_BYTES_PER_S, LINK_LATENCY_S
    m = load_cost_model()
    pre = np.array(m["points"]["T_pre"], dtype=np.float64)
    fam = fit_alpha_beta_family(pre[:, 1], pre[:, 0], pre[:, 2])
    np.testing.assert_allclose(fam.alpha, m["tpre_alpha"], rtol=1e-9)
    np.testing.assert_allclose(fam.beta, m["tpre_beta"], rtol=1e-9)
    dec = np.array(m["points"]["T_dec"], dtype=np.float64)
    famd = fit_alpha_beta_family(dec[:, 0], dec[:, 1], dec[:, 2])
    np.testing.assert_allclose(famd.alpha, m["tdec_alpha"], rtol=1e-9)
    np.testing.assert_allclose(famd.beta, m["tdec_beta"], rtol=1e-9)
    kv = np.array(m["points"]["T_kv"], dtype=np.float64)
    for col, name in ((1, "kv_pack"), (2, "kv_unpack")):
        f = fit_piecewise_alpha_beta(kv[:, 0], kv[:, col], segments=1)
        np.testing.assert_allclose([f.alpha[0], f.beta[0]], m[name], rtol=1e-9)
    sh = m["layer_shapes"]["T_kv"]
    wire = 2 * sh["Hkv"] * sh["d"] * 2 / LINK_BYTES_PER_S
    assert m["kv_beta"] == pytest.approx(m["kv_pack"][1] + m["kv_unpack"][1] + wire, rel=1e-12)
    assert m["kv_alpha"] == pytest.approx(m["kv_pack"][0] + m["kv_unpack"][0] + LINK_LATENCY_S, rel=1e-12)
    np.testing.assert_array_equal(S.MI355X_ATTENTION["tpre_beta"], m["tpre_beta"])
    assert S.MI355X_ATTENTION["kv_beta"] == m["kv_beta"] and S.MI355X_ATTENTION["kv_alpha"] == m["kv_alpha"]
    # every fitted time is positive and grows with its size argument
    assert min(m["tpre_alpha"]) > 0 and min(m["tpre_beta"]) > 0 and min(m["tdec_beta"]) > 0 and m["kv_pack"][1] > 0
