"""The serving simulator (host only): closed forms on one session, conservation, determinism, and the qualitative
behaviour of the three routing policies and of the reordering window under overload (paper Sections 3, 4.1, 4.2)."""
import numpy as np
import pytest

from paper_2602_14516_amd import simulator as S


@pytest.fixture(scope="module")
def model():
    return S.CostModel(**S.MI355X_ATTENTION)


def test_one_session_local_matches_the_cost_model_by_hand(model):
    L, D = 300, 5
    sess = [(0.25, [S.Round(L, D, 0.0)])]
    r = S.simulate(sess, model, n_prefill=0, n_decode=1, policy="adaptive")
    t_pre = model.t_pre(0, L, False)
    assert r.routed_local == 1 and r.routed_remote == 0
    np.testing.assert_allclose(r.ttft, [t_pre], rtol=1e-12)
    steps = [model.t_dec(1, L + i) for i in range(D)]              # the context grows by one token per step
    np.testing.assert_allclose(r.itl, steps, rtol=1e-12)
    np.testing.assert_allclose(r.makespan, 0.25 + t_pre + sum(steps), rtol=1e-12)


def test_one_session_remote_pays_both_kv_transfers(model):
    L1, L2, D = 200, 64, 3
    sess = [(0.0, [S.Round(L1, D, 0.5), S.Round(L2, D, 0.0)])]
    r = S.simulate(sess, model, n_prefill=1, n_decode=1, policy="remote")
    # round 1: no history to move; first token when the remote prefill ends; decoding starts once the new KV is back
    ttft1 = model.t_pre(0, L1, True)
    t = ttft1 + model.t_kv(L1)
    first_gap = model.t_kv(L1) + model.t_dec(1, L1)
    t += sum(model.t_dec(1, L1 + i) for i in range(D))
    # round 2 after the tool delay: history (L1 + D tokens) travels to the prefill worker first
    hist = L1 + D
    ttft2 = model.t_kv(hist) + model.t_pre(hist, L2, True)
    np.testing.assert_allclose(r.ttft, [ttft1, ttft2], rtol=1e-12)
    np.testing.assert_allclose(r.itl[0], first_gap, rtol=1e-12)
    t += 0.5 + ttft2 + model.t_kv(L2) + sum(model.t_dec(1, hist + L2 + i) for i in range(D))
    np.testing.assert_allclose(r.makespan, t, rtol=1e-12)


def test_conservation_and_determinism(model):
    sess = S.make_sessions(3, num_sessions=40, rounds=4, tool_delay_mean=0.01, arrival_span=0.1, dec_lo=8, dec_hi=24)
    a = S.simulate(sess, model, n_prefill=2, n_decode=3, policy="adaptive", reorder_window=5, seed=7)
    b = S.simulate(sess, model, n_prefill=2, n_decode=3, policy="adaptive", reorder_window=5, seed=7)
    assert np.array_equal(a.ttft, b.ttft) and np.array_equal(a.itl, b.itl) and a.makespan == b.makespan
    assert len(a.ttft) == 40 * 4 == a.routed_local + a.routed_remote
    assert len(a.itl) == sum(r.n_dec for _, rounds in sess for r in rounds)
    assert all(0.0 <= v <= 1.0 + 1e-9 for v in a.per_worker_busy.values())


def test_remote_only_never_stalls_decoding_and_local_only_never_uses_prefill_workers(model):
    sess = S.make_sessions(5, num_sessions=64, rounds=4, median=1024, tool_delay_mean=0.01, arrival_span=0.1, dec_lo=16, dec_hi=48)
    rem = S.simulate(sess, model, n_prefill=8, n_decode=2, policy="remote")
    loc = S.simulate(sess, model, n_prefill=8, n_decode=2, policy="local")
    assert rem.routed_local == 0 and loc.routed_remote == 0
    assert loc.per_worker_busy["p0"] == 0.0
    # a decode step of at most 32 rows over this much context is the longest gap a session can see without stalls,
    # apart from the first gap of a round, which also holds the return of the incremental KV
    worst_ctx = 32 * max(sum(r.l_incr + r.n_dec for r in rounds) for _, rounds in sess)
    bound = model.t_dec(32, worst_ctx) + model.t_kv(8192)
    assert rem.itl.max() <= bound
    assert loc.itl.max() > rem.itl.max()                      # local prefills stall the decode rows


def test_policies_under_overload(model):
    """One prefill worker for four decode workers and long tool outputs: always-remote drowns the prefill worker
    (TTFT), always-local stalls decoding (ITL), Algorithm 1 uses both and finishes first; the reordering window
    raises the share of rounds that meet the TTFT threshold."""
    sess = S.make_sessions(1, num_sessions=256, rounds=8, median=2048, tool_delay_mean=0.02, arrival_span=0.2, dec_lo=16, dec_hi=64)
    kw = dict(n_prefill=1, n_decode=4, ttft_thres=0.03, itl_thres=0.012)
    rem = S.simulate(sess, model, policy="remote", **kw)
    loc = S.simulate(sess, model, policy="local", **kw)
    ada = S.simulate(sess, model, policy="adaptive", **kw)
    loc_w = S.simulate(sess, model, policy="local", reorder_window=5, **kw)
    assert rem.ttft_attainment < 0.05 and rem.itl_attainment > 0.99
    assert loc.ttft_attainment > 0.3 and loc.itl_attainment < 0.5
    assert ada.routed_local > 0 and ada.routed_remote > 0
    assert ada.makespan < min(rem.makespan, loc.makespan)
    assert ada.ttft_attainment > rem.ttft_attainment and ada.itl_attainment >= loc.itl_attainment
    assert loc_w.reorders > 0 and loc_w.ttft_attainment > loc.ttft_attainment
