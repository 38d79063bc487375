"""ctypes binding of libampd.so: argument marshalling only.

Every step of the hot path (append, attention, combine) runs in the library's HIP kernels;
PyTorch is used for device memory and streams.  Function names mirror the C entry points.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

LIB_PATH = os.environ.get("AMPD_LIB_PATH") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libampd.so")

EXPORTED_SYMBOLS = [
    "ampd_workspace_bytes", "ampd_workspace_bytes_opts", "ampd_kv_append",
    "ampd_incr_prefill_attn", "ampd_mixed_batch_attn", "ampd_incr_prefill_attn_opts",
    "ampd_mixed_batch_attn_opts", "ampd_paged_attn", "ampd_plan_describe", "ampd_plan_items",
    "ampd_set_timing", "ampd_last_timing", "ampd_status_string", "ampd_version", "ampd_kv_pack", "ampd_kv_unpack",
    "ampd_init", "ampd_mixed_batch_attn_static", "ampd_static_workspace_limit",
]

AMPD_KV_BF16, AMPD_KV_FP8_E4M3 = 0, 1


class AmpdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _Cache(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("kv_dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("num_pages", ctypes.c_int64),
                ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
                ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
                ("softmax_scale", ctypes.c_float), ("reserved2", ctypes.c_int32)]


class _Batch(ctypes.Structure):
    _fields_ = [("num_reqs", ctypes.c_int32), ("max_pages_per_req", ctypes.c_int32),
                ("h_ctx_len", ctypes.c_void_p), ("h_incr_len", ctypes.c_void_p),
                ("d_block_table", ctypes.c_void_p), ("h_block_table", ctypes.c_void_p)]


class _Opts(ctypes.Structure):
    _fields_ = [("force_kv_splits", ctypes.c_int32), ("reserved", ctypes.c_int32 * 7)]


class _PlanInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("num_items", "num_wide_items", "num_narrow_items",
                                              "num_combine_items", "num_append_launches",
                                              "partial_bytes", "plan_bytes", "num_append_items", "num_workgroups")]


HOST_ONLY_SYMBOLS = ["ampd_workspace_bytes", "ampd_workspace_bytes_opts", "ampd_plan_describe", "ampd_plan_items",
                     "ampd_status_string", "ampd_version"]


class _HostOnly:
    """Stands in for an entry point that a host-only build of the library (the sanitizer build of the planner and
    of argument validation: AMPD_HOST_ONLY=1 next to AMPD_LIB_PATH) does not hold: attributes can be set, a call raises."""

    def __init__(self, name):
        self._name = name

    def __call__(self, *a):
        raise RuntimeError(f"{self._name} is not part of a host-only build of libampd")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2602_14516_amd/build.py` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    if os.environ.get("AMPD_HOST_ONLY") == "1":
        for name in EXPORTED_SYMBOLS:
            if name not in HOST_ONLY_SYMBOLS:
                setattr(L, name, _HostOnly(name))
    vp, sz, i32, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64
    cp, bp, op = ctypes.POINTER(_Cache), ctypes.POINTER(_Batch), ctypes.POINTER(_Opts)
    L.ampd_workspace_bytes.restype = sz
    L.ampd_workspace_bytes.argtypes = [cp, bp]
    L.ampd_workspace_bytes_opts.restype = sz
    L.ampd_workspace_bytes_opts.argtypes = [cp, bp, op]
    L.ampd_kv_append.restype = i32
    L.ampd_kv_append.argtypes = [cp, bp, vp, vp, vp]
    for name in ("ampd_kv_pack", "ampd_kv_unpack"):
        f = getattr(L, name)
        f.restype = i32
        f.argtypes = [cp, bp, i32, i32, vp, vp, vp]
    for name in ("ampd_incr_prefill_attn", "ampd_mixed_batch_attn"):
        f = getattr(L, name)
        f.restype = i32
        f.argtypes = [cp, bp, vp, vp, vp, vp, vp, sz, vp]
        f = getattr(L, name + "_opts")
        f.restype = i32
        f.argtypes = [cp, bp, vp, vp, vp, vp, vp, sz, vp, op]
    L.ampd_paged_attn.restype = i32
    L.ampd_paged_attn.argtypes = [cp, bp, vp, vp, vp, sz, vp, op]
    L.ampd_init.restype = i32
    L.ampd_init.argtypes = []
    L.ampd_static_workspace_limit.restype = sz
    L.ampd_static_workspace_limit.argtypes = []
    L.ampd_mixed_batch_attn_static.restype = i32
    L.ampd_mixed_batch_attn_static.argtypes = [cp, bp, vp, vp, vp, vp, vp]
    L.ampd_plan_describe.restype = i32
    L.ampd_plan_describe.argtypes = [cp, bp, op, ctypes.POINTER(_PlanInfo)]
    L.ampd_plan_items.restype = i64
    L.ampd_plan_items.argtypes = [cp, bp, op, vp, i64]
    L.ampd_set_timing.restype = None
    L.ampd_set_timing.argtypes = [ctypes.c_int]
    L.ampd_last_timing.restype = i32
    L.ampd_last_timing.argtypes = [ctypes.POINTER(ctypes.c_float)] * 3
    L.ampd_status_string.restype = ctypes.c_char_p
    L.ampd_status_string.argtypes = [i32]
    L.ampd_version.restype = ctypes.c_char_p
    return L


lib = _load()


def status_string(s: int) -> str:
    return lib.ampd_status_string(int(s)).decode()


def version() -> str:
    return lib.ampd_version().decode()


def _ptr(t):
    """Device/host address of a torch tensor or numpy array (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


@dataclass
class KVCache:
    """Shape of a paged pool plus the (torch, device) tensors that back it.

    k_pool / v_pool: [num_pages, Hkv, P, d]; dtype bfloat16 (or int16/uint16 bit patterns)
    for a bf16 cache, uint8 for an E4M3 cache (then k_scale / v_scale: float32 [num_pages, Hkv]).
    """
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    k_pool: object
    v_pool: object
    softmax_scale: float
    k_scale: object = None
    v_scale: object = None
    kv_dtype: int = AMPD_KV_BF16

    def c_struct(self, with_pools=True) -> _Cache:
        num_pages = int(self.k_pool.shape[0]) if self.k_pool is not None else int(getattr(self, "num_pages_hint", 1))
        return _Cache(self.num_q_heads, self.num_kv_heads, self.head_dim, self.page_size, self.kv_dtype, 0,
                      num_pages, _ptr(self.k_pool), _ptr(self.v_pool), _ptr(self.k_scale), _ptr(self.v_scale),
                      float(self.softmax_scale), 0)


def _batch(ctx_len, incr_len, block_table_dev, block_table_host=None, max_pages=None):
    ctx = np.ascontiguousarray(ctx_len, dtype=np.int32)
    inc = np.ascontiguousarray(incr_len, dtype=np.int32)
    assert ctx.shape == inc.shape and ctx.ndim == 1
    if block_table_dev is not None:
        max_pages = int(block_table_dev.shape[1]) if block_table_dev.ndim == 2 else int(max_pages)
    bth = None
    if block_table_host is not None:
        bth = np.ascontiguousarray(block_table_host, dtype=np.int32)
    b = _Batch(ctx.shape[0], int(max_pages or 0), ctx.ctypes.data, inc.ctypes.data,
               _ptr(block_table_dev), None if bth is None else bth.ctypes.data)
    return b, (ctx, inc, bth)          # keep the host arrays alive for the duration of the call


def _opts(force_kv_splits=0):
    if not force_kv_splits:
        return None
    o = _Opts()
    o.force_kv_splits = int(force_kv_splits)
    return ctypes.byref(o)


def _stream_ptr(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(st, where):
    if st != 0:
        raise AmpdError(int(st), where)


def workspace_bytes(cache: KVCache, ctx_len, incr_len, max_pages, force_kv_splits=0) -> int:
    b, keep = _batch(ctx_len, incr_len, None, max_pages=max_pages)
    c = cache.c_struct()
    return int(lib.ampd_workspace_bytes_opts(ctypes.byref(c), ctypes.byref(b), _opts(force_kv_splits)))


def plan_describe(cache: KVCache, ctx_len, incr_len, max_pages, force_kv_splits=0) -> dict:
    b, keep = _batch(ctx_len, incr_len, None, max_pages=max_pages)
    c = cache.c_struct()
    info = _PlanInfo()
    _check(lib.ampd_plan_describe(ctypes.byref(c), ctypes.byref(b), _opts(force_kv_splits), ctypes.byref(info)),
           "ampd_plan_describe")
    return {n: int(getattr(info, n)) for n, _ in _PlanInfo._fields_}


def plan_items(cache: KVCache, ctx_len, incr_len, max_pages, force_kv_splits=0) -> np.ndarray:
    """int32 [n, 10]: request, kind, kv_head, first_head_in_group, heads, first_token, tokens, key_begin,
    key_end, partial_offset."""
    b, keep = _batch(ctx_len, incr_len, None, max_pages=max_pages)
    c = cache.c_struct()
    o = _opts(force_kv_splits)
    n = int(lib.ampd_plan_items(ctypes.byref(c), ctypes.byref(b), o, None, 0))
    if n < 0:
        raise AmpdError(n, "ampd_plan_items")
    items = np.zeros((n, 10), dtype=np.int32)
    if n:
        lib.ampd_plan_items(ctypes.byref(c), ctypes.byref(b), o, items.ctypes.data, n)
    return items


def kv_append(cache: KVCache, ctx_len, incr_len, block_table, k_new, v_new, *, stream=None,
              block_table_host=None) -> None:
    b, keep = _batch(ctx_len, incr_len, block_table, block_table_host)
    c = cache.c_struct()
    _check(lib.ampd_kv_append(ctypes.byref(c), ctypes.byref(b), _ptr(k_new), _ptr(v_new), _stream_ptr(stream)),
           "ampd_kv_append")


def kv_pack(cache: KVCache, first_token, num_tokens, block_table, head_begin, head_count, k_out, v_out, *, stream=None,
            block_table_host=None) -> None:
    """Pages -> packed rows [sum tokens, head_count, d] for KV heads [head_begin, head_begin + head_count)."""
    b, keep = _batch(first_token, num_tokens, block_table, block_table_host)
    c = cache.c_struct()
    _check(lib.ampd_kv_pack(ctypes.byref(c), ctypes.byref(b), int(head_begin), int(head_count), _ptr(k_out), _ptr(v_out),
                            _stream_ptr(stream)), "ampd_kv_pack")


def kv_unpack(cache: KVCache, first_token, num_tokens, block_table, head_begin, head_count, k_in, v_in, *, stream=None,
              block_table_host=None) -> None:
    """Packed rows -> pages, the inverse of kv_pack."""
    b, keep = _batch(first_token, num_tokens, block_table, block_table_host)
    c = cache.c_struct()
    _check(lib.ampd_kv_unpack(ctypes.byref(c), ctypes.byref(b), int(head_begin), int(head_count), _ptr(k_in), _ptr(v_in),
                              _stream_ptr(stream)), "ampd_kv_unpack")


def _temp_workspace(need, q, stream):
    """A workspace for one call: allocated, and later returned to torch's caching allocator, on the stream the call
    runs on, so that the block cannot be handed out again while that stream still uses it."""
    import torch
    if stream is None or isinstance(stream, int):
        # a raw hipStream_t cannot be named to the allocator: the caller passes workspace= in that case
        if isinstance(stream, int) and stream != torch.cuda.current_stream().cuda_stream:
            raise ValueError("pass workspace= when stream= is a raw stream handle other than torch's current stream")
        return torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    with torch.cuda.stream(stream):
        return torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)


def _attn_call(fn_name, cache, ctx_len, incr_len, block_table, q, k_new, v_new, out, workspace, stream,
               block_table_host, force_kv_splits):
    import torch
    b, keep = _batch(ctx_len, incr_len, block_table, block_table_host)
    c = cache.c_struct()
    o = _opts(force_kv_splits)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = int(lib.ampd_workspace_bytes_opts(ctypes.byref(c), ctypes.byref(b), o))
        workspace = _temp_workspace(need, q, stream)
    fn = getattr(lib, fn_name + "_opts")
    _check(fn(ctypes.byref(c), ctypes.byref(b), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _ptr(workspace),
              workspace.numel() * workspace.element_size(), _stream_ptr(stream), o), fn_name)
    return out


def incr_prefill_attn(cache: KVCache, ctx_len, incr_len, block_table, q, k_new, v_new, *, out=None,
                      workspace=None, stream=None, block_table_host=None, force_kv_splits=0):
    """Append k_new/v_new, then causal GQA attention of the new queries; returns out (bf16 [sum L, Hq, d])."""
    return _attn_call("ampd_incr_prefill_attn", cache, ctx_len, incr_len, block_table, q, k_new, v_new, out,
                      workspace, stream, block_table_host, force_kv_splits)


def mixed_batch_attn(cache: KVCache, ctx_len, incr_len, block_table, q, k_new, v_new, *, out=None,
                     workspace=None, stream=None, block_table_host=None, force_kv_splits=0):
    """The same for a batch mixing decode rows (L=1) and prefill rows (L>1): one fused attention launch."""
    return _attn_call("ampd_mixed_batch_attn", cache, ctx_len, incr_len, block_table, q, k_new, v_new, out,
                      workspace, stream, block_table_host, force_kv_splits)


def init() -> None:
    """One-time set-up of the current device (pins the staging ring, resolves the static workspace)."""
    _check(lib.ampd_init(), "ampd_init")


def static_workspace_limit() -> int:
    return int(lib.ampd_static_workspace_limit())


def mixed_batch_attn_static(cache: KVCache, ctx_len, incr_len, block_table, q, k_new, v_new, out, *, stream=None,
                            block_table_host=None):
    """mixed_batch_attn on the library's static workspace: the call allocates nothing (out is required)."""
    b, keep = _batch(ctx_len, incr_len, block_table, block_table_host)
    c = cache.c_struct()
    _check(lib.ampd_mixed_batch_attn_static(ctypes.byref(c), ctypes.byref(b), _ptr(q), _ptr(k_new), _ptr(v_new),
                                            _ptr(out), _stream_ptr(stream)), "ampd_mixed_batch_attn_static")
    return out


def paged_attn(cache: KVCache, ctx_len, incr_len, block_table, q, *, out=None, workspace=None, stream=None,
               block_table_host=None, force_kv_splits=0):
    """Attention only; the pools must already hold all C + L tokens of every row."""
    import torch
    b, keep = _batch(ctx_len, incr_len, block_table, block_table_host)
    c = cache.c_struct()
    o = _opts(force_kv_splits)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need = int(lib.ampd_workspace_bytes_opts(ctypes.byref(c), ctypes.byref(b), o))
        workspace = _temp_workspace(need, q, stream)
    _check(lib.ampd_paged_attn(ctypes.byref(c), ctypes.byref(b), _ptr(q), _ptr(out), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream_ptr(stream), o),
           "ampd_paged_attn")
    return out


def set_timing(enabled: bool) -> None:
    lib.ampd_set_timing(1 if enabled else 0)


def last_timing():
    """(attention ms, combine ms, append+plan-copy ms) of the last call on this thread; sync the stream first."""
    a, c, p = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _check(lib.ampd_last_timing(ctypes.byref(a), ctypes.byref(c), ctypes.byref(p)), "ampd_last_timing")
    return a.value, c.value, p.value
