"""Piecewise alpha-beta cost model of the attention path, fitted from measured step times.

The paper's profiler turns measured execution times into cost functions that its planner
and online scheduler query (paper Section 3, "Offline stage": T_pre(l_hist, l_incr),
T_dec(b); the alpha-beta form is the latency + size/bandwidth model it cites).  For the
operator built here the natural "size" is the algorithmic work of a call:

    T_pre(l_hist, l_incr)  ~  alpha_s + beta_s * FLOPs,   FLOPs = 4 d Hq (l_incr l_hist + l_incr (l_incr+1)/2)
    T_dec(b, sum C)        ~  alpha_s + beta_s * bytes,   bytes = 2 (sum C + b) Hkv d b_kv + ...

with one (alpha_s, beta_s) pair per size segment s (small calls are launch-bound, large calls
run at the kernel's asymptotic rate).  The paper's T_dec takes only the batch size; the
measured cost of decode attention is set by the total context, so sum C is kept.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class PiecewiseAlphaBeta:
    """t(x) = alpha[s] + beta[s] * x on segment s, segments delimited by `knots` (ascending,
    len = segments - 1); x below the first knot uses segment 0."""
    knots: np.ndarray
    alpha: np.ndarray
    beta: np.ndarray

    def __call__(self, x):
        x = np.asarray(x, dtype=np.float64)
        s = np.searchsorted(self.knots, x, side="right")
        return self.alpha[s] + self.beta[s] * x

    def rel_error(self, x, t):
        t = np.asarray(t, dtype=np.float64)
        return np.abs(self(x) - t) / t


def fit_piecewise_alpha_beta(x, t, segments: int = 3, knots=None) -> PiecewiseAlphaBeta:
    """Least-squares fit of a piecewise alpha-beta model.  Knots default to equal-count
    quantiles of log(x); every segment needs at least two distinct sizes (else it inherits
    its neighbour's line)."""
    x = np.asarray(x, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    assert x.shape == t.shape and x.ndim == 1 and x.size >= 2
    if knots is None:
        qs = np.linspace(0, 1, segments + 1)[1:-1]
        knots = np.exp(np.quantile(np.log(np.maximum(x, 1e-30)), qs)) if segments > 1 else np.zeros(0)
    knots = np.asarray(knots, dtype=np.float64)
    nseg = len(knots) + 1
    seg = np.searchsorted(knots, x, side="right")
    alpha = np.full(nseg, np.nan)
    beta = np.full(nseg, np.nan)
    for s in range(nseg):
        m = seg == s
        if m.sum() >= 2 and np.ptp(x[m]) > 0:
            A = np.stack([np.ones(m.sum()), x[m]], axis=1)
            # relative least squares: every measurement counts equally whatever its size
            w = 1.0 / t[m]
            sol, *_ = np.linalg.lstsq(A * w[:, None], t[m] * w, rcond=None)
            alpha[s], beta[s] = sol
    for s in range(nseg):                       # segments without enough data copy the nearest fitted one
        if np.isnan(alpha[s]):
            ok = np.nonzero(~np.isnan(alpha))[0]
            assert ok.size, "no segment could be fitted"
            n = ok[np.argmin(np.abs(ok - s))]
            alpha[s], beta[s] = alpha[n], beta[n]
    return PiecewiseAlphaBeta(knots, alpha, beta)


def prefill_flops(l_hist, l_incr, Hq: int, d: int):
    l_hist = np.asarray(l_hist, dtype=np.float64)
    l_incr = np.asarray(l_incr, dtype=np.float64)
    return 4.0 * d * Hq * (l_incr * l_hist + l_incr * (l_incr + 1) / 2)


def decode_bytes(sum_ctx, b, Hq: int, Hkv: int, d: int, kv_bytes: int = 2):
    sum_ctx = np.asarray(sum_ctx, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return 2.0 * (sum_ctx + b) * Hkv * d * kv_bytes + 2 * b * Hkv * d * (2 + kv_bytes) + 2 * b * Hq * d * 2


@dataclass
class AlphaBetaFamily:
    """One alpha-beta line t = alpha + beta * size per bucket of a second variable (e.g. one line in
    l_hist per incremental length, one line in sum C per decode batch size); queries between
    buckets interpolate the two neighbouring lines linearly in log(bucket)."""
    buckets: np.ndarray
    alpha: np.ndarray
    beta: np.ndarray

    def __call__(self, bucket, size):
        bucket = np.atleast_1d(np.asarray(bucket, dtype=np.float64))
        size = np.atleast_1d(np.asarray(size, dtype=np.float64))
        lb = np.log(self.buckets)
        q = np.clip(np.log(np.maximum(bucket, 1e-30)), lb[0], lb[-1])
        hi = np.clip(np.searchsorted(lb, q, side="left"), 1, len(lb) - 1) if len(lb) > 1 else np.zeros_like(q, dtype=int)
        lo = np.maximum(hi - 1, 0)
        w = np.where(lb[hi] > lb[lo], (q - lb[lo]) / np.where(lb[hi] > lb[lo], lb[hi] - lb[lo], 1.0), 0.0)
        t_lo = self.alpha[lo] + self.beta[lo] * size
        t_hi = self.alpha[hi] + self.beta[hi] * size
        return (1 - w) * t_lo + w * t_hi


def fit_alpha_beta_family(bucket, size, t) -> AlphaBetaFamily:
    bucket = np.asarray(bucket, dtype=np.float64)
    size = np.asarray(size, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    bs = np.unique(bucket)
    alpha, beta = [], []
    for b in bs:
        m = bucket == b
        fit = fit_piecewise_alpha_beta(size[m], t[m], segments=1)
        alpha.append(fit.alpha[0])
        beta.append(fit.beta[0])
    return AlphaBetaFamily(bs, np.array(alpha), np.array(beta))


# ---------------------------------------------------------------------------------------------------------------------
# The committed cost model of one MI355X: written by `python -m paper_2602_14516_amd.perf_model <model.json>` from the
# output of `bench.py --only model`, read by the serving simulator and checked against fresh measurements by the GPU tests.

import json
import os

COST_MODEL_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mi355x_cost_model.json")
# What one GPU cannot measure: the wire between two workers.  One xGMI link of an MI355X moves ~153 GB/s; a transfer
# between two GPUs uses one link, and a message costs a few microseconds of latency on top.
LINK_BYTES_PER_S = 153e9
LINK_LATENCY_S = 10e-6


def cost_model_from_sweep(sweep: dict) -> dict:
    """Constants of the simulator's cost model from the output of `bench.py --only model`: the fitted T_pre and T_dec
    lines as they are, and T_kv(tokens) = alpha + beta * tokens (one layer) as pack + wire + unpack, the two GPU halves
    fitted from measured ampd_kv_pack / ampd_kv_unpack times and the wire from the link figures above."""
    pre, dec, kv = sweep["T_pre"]["per_l_incr_lines_in_l_hist"], sweep["T_dec"]["per_batch_lines_in_sum_ctx"], sweep["T_kv"]
    sh = sweep["layer_shapes"]["T_kv"]
    bytes_per_token = 2 * sh["Hkv"] * sh["d"] * 2                      # K and V rows of one token, bf16
    return {
        "source": "bench.py --only model on one MI355X; whole C-ABI calls; one attention layer",
        "layer_shapes": sweep["layer_shapes"],
        "tpre_l_incr": pre["l_incr"], "tpre_alpha": pre["alpha_s"], "tpre_beta": pre["beta_s_per_token"],
        "tpre_rel_err": [pre["rel_err_mean"], pre["rel_err_max"]],
        "tdec_b": dec["b"], "tdec_alpha": dec["alpha_s"], "tdec_beta": dec["beta_s_per_token"],
        "tdec_rel_err": [dec["rel_err_mean"], dec["rel_err_max"]],
        "kv_pack": [kv["pack"]["alpha_s"], kv["pack"]["beta_s_per_token"]],
        "kv_unpack": [kv["unpack"]["alpha_s"], kv["unpack"]["beta_s_per_token"]],
        "kv_link": [LINK_LATENCY_S, bytes_per_token / LINK_BYTES_PER_S],
        "kv_alpha": kv["pack"]["alpha_s"] + kv["unpack"]["alpha_s"] + LINK_LATENCY_S,
        "kv_beta": kv["pack"]["beta_s_per_token"] + kv["unpack"]["beta_s_per_token"] + bytes_per_token / LINK_BYTES_PER_S,
        "points": {"T_pre": sweep["T_pre"]["points_l_hist_l_incr_seconds"], "T_dec": sweep["T_dec"]["points_b_sum_ctx_seconds"],
                   "T_kv": kv["points_l_ctx_pack_s_unpack_s"]},
    }


def load_cost_model(path: str = COST_MODEL_PATH) -> dict:
    with open(path) as f:
        return json.load(f)


def render_markdown(model: dict) -> str:
    """The measured points and fitted lines of a cost model as markdown tables (the text under profiles/ is this)."""
    sh = model["layer_shapes"]
    pre = AlphaBetaFamily(np.array(model["tpre_l_incr"]), np.array(model["tpre_alpha"]), np.array(model["tpre_beta"]))
    dec = AlphaBetaFamily(np.array(model["tdec_b"]), np.array(model["tdec_alpha"]), np.array(model["tdec_beta"]))
    o = ["## Measured points", "", "| l_hist | l_incr | step us | algorithmic TFLOP/s | fitted line us |", "|---|---|---|---|---|"]
    for h, l, t in model["points"]["T_pre"]:
        fl = float(prefill_flops(h, l, sh["T_pre"]["Hq"], sh["T_pre"]["d"]))
        o.append(f"| {int(h)} | {int(l)} | {t * 1e6:.1f} | {fl / t / 1e12:.0f} | {float(pre(l, h)[0]) * 1e6:.1f} |")
    o += ["", "| b | sum C | step us | K/V GB/s | fitted line us |", "|---|---|---|---|---|"]
    for b, c, t in model["points"]["T_dec"]:
        by = float(decode_bytes(c, b, sh["T_dec"]["Hq"], sh["T_dec"]["Hkv"], sh["T_dec"]["d"]))
        o.append(f"| {int(b)} | {int(c)} | {t * 1e6:.1f} | {by / t / 1e9:.0f} | {float(dec(b, c)[0]) * 1e6:.1f} |")
    o += ["", "| l_ctx | pack us | unpack us | read + write GB/s (pack) |", "|---|---|---|---|"]
    per_token = 2 * sh["T_kv"]["Hkv"] * sh["T_kv"]["d"] * 2
    for l, tp, tu in model["points"]["T_kv"]:
        o.append(f"| {int(l)} | {tp * 1e6:.1f} | {tu * 1e6:.1f} | {2 * per_token * l / tp / 1e9:.0f} |")
    o += ["", "## Fitted lines (relative least squares)", "",
          "T_pre(l_hist; l_incr) = alpha + beta x l_hist, one line per incremental length, interpolated in log(l_incr) between lines:", "",
          "| l_incr | alpha us | beta ns per history token |", "|---|---|---|"]
    for l, a, b in zip(model["tpre_l_incr"], model["tpre_alpha"], model["tpre_beta"]):
        o.append(f"| {int(l)} | {a * 1e6:.1f} | {b * 1e9:.2f} |")
    o += ["", f"residual on the grid: mean {model['tpre_rel_err'][0] * 100:.1f} %, max {model['tpre_rel_err'][1] * 100:.0f} %", "",
          "T_dec(sum C; b) = alpha + beta x sum C, one line per batch size:", "", "| b | alpha us | beta ns per context token |", "|---|---|---|"]
    for bb, a, b in zip(model["tdec_b"], model["tdec_alpha"], model["tdec_beta"]):
        o.append(f"| {int(bb)} | {a * 1e6:.1f} | {b * 1e9:.3f} |")
    kp, ku, kl = model["kv_pack"], model["kv_unpack"], model["kv_link"]
    o += ["", f"residual on the grid: mean {model['tdec_rel_err'][0] * 100:.1f} %, max {model['tdec_rel_err'][1] * 100:.1f} %", "",
          f"T_kv(l) per layer = pack + wire + unpack: pack {kp[0] * 1e6:.1f} us + {kp[1] * 1e9:.2f} ns/token, unpack {ku[0] * 1e6:.1f} us + "
          f"{ku[1] * 1e9:.2f} ns/token (measured), wire {kl[0] * 1e6:.0f} us + {kl[1] * 1e9:.1f} ns/token (one xGMI link at its nominal "
          f"{LINK_BYTES_PER_S / 1e9:.0f} GB/s, {per_token} bytes of K and V per token: not measurable on one GPU); "
          f"kv_alpha = {model['kv_alpha'] * 1e6:.1f} us, kv_beta = {model['kv_beta'] * 1e9:.1f} ns/token."]
    return "\n".join(o) + "\n"


def _main(argv):
    if len(argv) == 2 and argv[1] == "--render":
        print(render_markdown(load_cost_model()), end="")
        return 0
    if len(argv) != 2:
        print("usage: python -m paper_2602_14516_amd.perf_model <output of `bench.py --only model`>   (writes the cost model)\n"
              "       python -m paper_2602_14516_amd.perf_model --render                             (prints it as markdown tables)")
        return 2
    lines = [l for l in open(argv[1]).read().splitlines() if l.startswith("{")]
    model = cost_model_from_sweep(json.loads(lines[-1]))
    with open(COST_MODEL_PATH, "w") as f:
        json.dump(model, f, indent=1)
        f.write("\n")
    print("wrote", COST_MODEL_PATH)
    return 0


if __name__ == "__main__":
    import sys
    sys.exit(_main(sys.argv))
