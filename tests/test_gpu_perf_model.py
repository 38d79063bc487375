"""The committed cost model of the attention path (paper Section 3, offline stage: T_pre(l_hist, l_incr), T_dec(b),
T_kv(l_ctx)) against fresh measurements: a handful of points timed through the C ABI on this GPU must lie within 30 %
of what mi355x_cost_model.json predicts (the fit's own worst residual on its grid is 26 %), on and off the grid the lines
were fitted on."""
import os
import sys

import numpy as np
import pytest
import torch

import paper_2602_14516_amd as A
import workloads as W
from paper_2602_14516_amd import sched
from paper_2602_14516_amd.perf_model import AlphaBetaFamily, load_cost_model

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench as B   # the measurement helpers of the benchmark (device batches, timed loops)

pytestmark = pytest.mark.gpu
TOL = 0.30


def _median_ms(fn, reps=7):
    return float(np.median([B.time_calls(torch, fn, 10, 3) for _ in range(reps)]))


def test_measured_points_agree_with_the_committed_cost_model():
    m = load_cost_model()
    tpre = sched.TPreModel(np.array(m["tpre_l_incr"]), np.array(m["tpre_alpha"]), np.array(m["tpre_beta"]))
    tdec = AlphaBetaFamily(np.array(m["tdec_b"], float), np.array(m["tdec_alpha"], float), np.array(m["tdec_beta"], float))
    worst = 0.0
    sh = m["layer_shapes"]["T_pre"]
    assert sh == W.CONFIG_SHAPES[2] and m["layer_shapes"]["T_dec"] == W.CONFIG_SHAPES[3]
    # T_pre: three grid points (long history, long chunk, both) and two between the fitted incremental lengths
    for l_hist, l_incr in ((16384, 1024), (1024, 4096), (65536, 256), (8192, 512), (30000, 2048)):
        db = B.device_batch(torch, A, W, np.array([l_hist], np.int32), np.array([l_incr], np.int32), sh, seed=1)
        ms = _median_ms(B.make_runner(torch, A, db, "prefill"))
        pred = sched.t_pre(tpre, l_hist, l_incr) * 1e3
        print(f"  T_pre({l_hist}, {l_incr}): measured {ms * 1e3:.1f} us, model {pred * 1e3:.1f} us", flush=True)
        worst = max(worst, abs(ms - pred) / ms)
        assert abs(ms - pred) <= TOL * ms
        del db
    # T_dec: batch sizes on and between the fitted ones
    g = np.random.default_rng(1)
    for b, cmean in ((32, 4096), (96, 8192), (64, 2048)):
        C = g.integers(cmean // 2, cmean * 3 // 2, size=b, endpoint=True).astype(np.int32)
        db = B.device_batch(torch, A, W, C, np.ones(b, np.int32), m["layer_shapes"]["T_dec"], seed=2)
        ms = _median_ms(B.make_runner(torch, A, db, "mixed"))
        pred = float(tdec(b, int(C.sum()))[0]) * 1e3
        print(f"  T_dec(b={b}, sum C={int(C.sum())}): measured {ms * 1e3:.1f} us, model {pred * 1e3:.1f} us", flush=True)
        worst = max(worst, abs(ms - pred) / ms)
        assert abs(ms - pred) <= TOL * ms
        del db
    # T_kv: the two GPU halves of a transfer
    for l_ctx in (2048, 32768):
        T, zero = np.array([l_ctx], np.int32), np.zeros(1, np.int32)
        db = B.device_batch(torch, A, W, T, zero, sh, seed=3)
        kb = torch.empty(l_ctx, sh["Hkv"], sh["d"], dtype=torch.bfloat16, device="cuda")
        vb = torch.empty_like(kb)
        for name, fn in (("kv_pack", lambda: A.kv_pack(db["cache"], zero, T, db["bt"], 0, sh["Hkv"], kb, vb)),
                         ("kv_unpack", lambda: A.kv_unpack(db["cache"], zero, T, db["bt"], 0, sh["Hkv"], kb, vb))):
            ms = _median_ms(fn)
            pred = (m[name][0] + m[name][1] * l_ctx) * 1e3
            print(f"  {name}({l_ctx}): measured {ms * 1e3:.1f} us, model {pred * 1e3:.1f} us", flush=True)
            worst = max(worst, abs(ms - pred) / ms)
            assert abs(ms - pred) <= TOL * ms
        del db, kb, vb
    print(f"  worst relative deviation {worst:.2f}", flush=True)
