"""Helpers for the GPU parity tests: move a synthetic batch to the device, run the library
through its C ABI binding, and compare with the CPU oracle."""
import numpy as np
import torch

import oracle
import paper_2602_14516_amd as A
import workloads as W

TOL_BF16 = (2e-2, 2e-3)     # max-abs, mean-abs for bf16 inputs
TOL_FP8 = (6e-2, 6e-3)


def to_dev_bits(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> device bf16 tensor (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


def from_dev_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


class DevBatch:
    def __init__(self, b: W.Batch):
        self.b = b
        self.k_pool = to_dev_bits(b.k_pool)
        self.v_pool = to_dev_bits(b.v_pool)
        self.q = to_dev_bits(b.q)
        self.k_new = to_dev_bits(b.k_new)
        self.v_new = to_dev_bits(b.v_new)
        self.bt = torch.from_numpy(b.block_table).cuda()
        self.cache = A.KVCache(b.Hq, b.Hkv, b.d, b.P, self.k_pool, self.v_pool, b.scale)


def sample_rows(b: W.Batch, per_req: int, seed: int = 0):
    """Dict request -> sorted new-token indices: first, last, page-boundary neighbours and random ones."""
    g = np.random.default_rng(seed)
    rows = {}
    for r in range(b.num_reqs):
        C, L = int(b.ctx_len[r]), int(b.incr_len[r])
        if L == 0:
            continue
        pick = {0, L - 1}
        pb = (-C) % b.P                       # first new token that starts a page
        for x in (pb - 1, pb, pb + 1):
            if 0 <= x < L:
                pick.add(x)
        if L > len(pick):
            pick.update(g.choice(L, size=min(per_req, L), replace=False).tolist())
        rows[r] = np.array(sorted(pick), np.int32)
    return rows


def compare(b: W.Batch, out_bits: np.ndarray, rows=None, tol=TOL_BF16, label=""):
    """Element-wise comparison with the oracle (all rows, or the sampled ones)."""
    ref = oracle.attn_oracle(b.k_pool, b.v_pool, b.block_table, b.ctx_len, b.incr_len,
                             b.q, b.k_new, b.v_new, b.P, b.scale, rows=rows)
    got = W.bf16_bits_to_f64(out_bits)
    off = b.row_offsets
    errs = []
    for r in range(b.num_reqs):
        if ref[r] is None or ref[r].shape[0] == 0:
            continue
        g = got[off[r]:off[r + 1]]
        if rows is not None:
            g = g[rows[r]]
        assert np.isfinite(g).all(), f"{label}: non-finite output in request {r}"
        errs.append(np.abs(g - ref[r]).ravel())
    e = np.concatenate(errs)
    mx, mean = float(e.max()), float(e.mean())
    assert mx <= tol[0] and mean <= tol[1], f"{label}: max-abs {mx:.3e} mean-abs {mean:.3e} exceed {tol}"
    return mx, mean


# ---- 8-bit cache: bounds against the oracle on the UNQUANTISED inputs ------------------------------------------------
#
# Rows that see at least FP8_MANY_KEYS keys are held to the stated 6e-2 / 6e-3.  A row that sees few keys mixes few
# E4M3-rounded V rows, so its error is bounded by the rounding of V itself: |sum_j p_j dV_j| <= max_j |dV_j| <=
# 2^-4 max|V| over the visible keys of its KV head (half an ulp of a 3-bit mantissa), to which the bf16 tolerance is
# added for everything else; on average a rounding error is a quarter ulp, so the mean over such rows is held to
# 2^-5 x the largest mean |V row| among the visible keys, plus the stated 6e-3.
FP8_MANY_KEYS = 256


def fp8_row_bounds(V_f64, C, rows, G):
    """V_f64 [T, Hkv, d] unquantised values of one request; rows: new-token indices.  Returns per (row, query head):
    keys seen [n], max-abs bound [n, Hq], mean-abs bound [n, Hq] (used for the rows that see few keys)."""
    a = np.abs(V_f64)
    run_max = np.maximum.accumulate(a.max(axis=2), axis=0)            # [T, Hkv] largest |V| among keys 0..t
    run_row = np.maximum.accumulate(a.mean(axis=2), axis=0)           # largest mean |V row| among keys 0..t
    idx = int(C) + np.asarray(rows, dtype=np.int64)
    return idx + 1, np.repeat(run_max[idx] / 16.0 + TOL_BF16[0], G, axis=1), np.repeat(run_row[idx] / 32.0 + TOL_FP8[1], G, axis=1)


class Fp8UnquantisedCheck:
    """Accumulates |got - oracle(unquantised)| over many (tick, request) groups and asserts the bounds above."""

    def __init__(self):
        self.many_max = 0.0
        self.many_sum = 0.0
        self.many_n = 0
        self.few_ratio = 0.0          # worst element error / its bound
        self.few_sum = 0.0
        self.few_bound_sum = 0.0
        self.few_n = 0

    def add(self, got, ref, V_f64, C, rows, G, label=""):
        """got, ref: [n, Hq, d] for the new-token indices `rows` of one request."""
        e = np.abs(got - ref)
        assert np.isfinite(e).all(), f"{label}: non-finite output"
        seen, bmax, bmean = fp8_row_bounds(V_f64, C, rows, G)
        many = seen >= FP8_MANY_KEYS
        if many.any():
            em = e[many]
            assert em.max() <= TOL_FP8[0], f"{label}: max-abs {em.max():.3e} > {TOL_FP8[0]} on a row that sees >= {FP8_MANY_KEYS} keys"
            self.many_max = max(self.many_max, float(em.max()))
            self.many_sum += float(em.sum())
            self.many_n += em.size
        few = ~many
        if few.any():
            ef = e[few]
            ratio = float((ef.max(axis=2) / bmax[few]).max())
            assert ratio <= 1.0, f"{label}: a row that sees < {FP8_MANY_KEYS} keys exceeds 2^-4 max|V| + {TOL_BF16[0]} ({ratio:.2f} x)"
            self.few_ratio = max(self.few_ratio, ratio)
            self.few_sum += float(ef.sum())
            self.few_bound_sum += float(bmean[few].sum()) * ef.shape[2]
            self.few_n += ef.size

    def finish(self, label=""):
        msg = []
        if self.many_n:
            mean = self.many_sum / self.many_n
            assert mean <= TOL_FP8[1], f"{label}: mean-abs {mean:.3e} > {TOL_FP8[1]} over rows that see >= {FP8_MANY_KEYS} keys"
            msg.append(f">= {FP8_MANY_KEYS} keys: max-abs {self.many_max:.2e} mean-abs {mean:.2e}")
        if self.few_n:
            mean, bound = self.few_sum / self.few_n, self.few_bound_sum / self.few_n
            assert mean <= bound, f"{label}: mean-abs {mean:.3e} > derived bound {bound:.3e} over rows that see few keys"
            msg.append(f"< {FP8_MANY_KEYS} keys: worst error / bound {self.few_ratio:.2f}, mean-abs {mean:.2e} (bound {bound:.2e})")
        return "; ".join(msg)
