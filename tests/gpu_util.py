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
