"""ctypes binding over libmedha.so: argument marshalling only.

Device tensors are torch tensors (PyTorch is used for device memory and streams
only); host-side length arrays are numpy / lists.  Every function enqueues on
torch's current stream and returns without synchronising.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmedha.so")
_LIB = None

EXPORTS = (
    "medha_chunked_prefill_attn",
    "medha_chunked_prefill_workspace_bytes",
    "medha_chunked_prefill_attn_noalloc",
    "medha_decode_partial_attn",
    "medha_decode_partial_workspace_bytes",
    "medha_chunk_partial_attn",
    "medha_chunk_partial_workspace_bytes",
    "medha_lse_merge",
    "medha_kv_append",
    "medha_describe_plan",
    "medha_describe_slot",
    "medha_strerror",
    "medha_abi_version",
)


class MedhaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"medha error {code}: {text}")
        self.code = code


class PlanEntry(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("mode", "rows_per_wg", "tile_keys", "n_row_tiles",
                                              "n_split", "tiles_per_split", "work_start",
                                              "n_slots")]


class _KvCache(ctypes.Structure):
    _fields_ = [("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
                ("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libmedha.so (built in-tree by ``paper_2409_17264_amd.build``).
    There is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2409_17264_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float,
                             ctypes.c_size_t)
    lib.medha_chunked_prefill_attn.restype = ctypes.c_int
    lib.medha_chunked_prefill_attn.argtypes = [vp, ctypes.POINTER(_KvCache), vp, vp, vp, vp, i32,
                                               i32, f32, vp, vp, vp, sz, vp]
    lib.medha_chunked_prefill_workspace_bytes.restype = sz
    lib.medha_chunked_prefill_workspace_bytes.argtypes = [vp, vp, i32, i32, i32, i32]
    lib.medha_decode_partial_attn.restype = ctypes.c_int
    lib.medha_decode_partial_attn.argtypes = [vp, i32, ctypes.POINTER(_KvCache), vp, vp, vp, vp,
                                              i32, i32, f32, vp, vp, vp, sz, vp]
    lib.medha_chunked_prefill_attn_noalloc.restype = ctypes.c_int
    lib.medha_chunked_prefill_attn_noalloc.argtypes = [vp, ctypes.POINTER(_KvCache), vp, vp, vp,
                                                       vp, i32, i32, f32, vp, vp, vp]
    lib.medha_decode_partial_workspace_bytes.restype = sz
    lib.medha_decode_partial_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.medha_chunk_partial_attn.restype = ctypes.c_int
    lib.medha_chunk_partial_attn.argtypes = [vp, i32, ctypes.POINTER(_KvCache), vp, vp, vp, vp, vp,
                                             vp, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.medha_chunk_partial_workspace_bytes.restype = sz
    lib.medha_chunk_partial_workspace_bytes.argtypes = [vp, vp, i32, i32, i32, i32]
    lib.medha_lse_merge.restype = ctypes.c_int
    lib.medha_lse_merge.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp, vp]
    lib.medha_kv_append.restype = ctypes.c_int
    lib.medha_kv_append.argtypes = [vp, vp, ctypes.POINTER(_KvCache), vp, vp, vp, vp, i32, vp]
    lib.medha_describe_plan.restype = ctypes.c_int
    lib.medha_describe_plan.argtypes = [vp, vp, i32, i32, i32, i32, i32, ctypes.POINTER(PlanEntry),
                                        ctypes.POINTER(i32), ctypes.POINTER(i32),
                                        ctypes.POINTER(sz)]
    lib.medha_describe_slot.restype = ctypes.c_int
    lib.medha_describe_slot.argtypes = [i32, i32, i32, i32, ctypes.POINTER(i32),
                                        ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.medha_strerror.restype = ctypes.c_char_p
    lib.medha_strerror.argtypes = [ctypes.c_int]
    lib.medha_abi_version.restype = ctypes.c_int
    lib.medha_abi_version.argtypes = []
    _LIB = lib
    return lib


def _check(code: int):
    if code != 0:
        raise MedhaError(code, load_library().medha_strerror(code).decode())


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a).reshape(-1), dtype=dtype)


def _hp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dp(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _kv(k_pool: torch.Tensor, v_pool: torch.Tensor) -> _KvCache:
    assert k_pool.dtype == torch.bfloat16 and v_pool.dtype == torch.bfloat16
    assert k_pool.is_contiguous() and v_pool.is_contiguous() and k_pool.shape == v_pool.shape
    num_pages, h_kv, page_size, d = k_pool.shape
    return _KvCache(k_pool.data_ptr(), v_pool.data_ptr(), num_pages, page_size, h_kv, d)


def chunked_prefill_workspace_bytes(prefix_len, chunk_len, num_q_heads: int, num_kv_heads: int,
                                    head_dim: int) -> int:
    pre, chk = _host(prefix_len, np.int32), _host(chunk_len, np.int32)
    return int(load_library().medha_chunked_prefill_workspace_bytes(
        _hp(pre), _hp(chk), len(pre), num_q_heads, num_kv_heads, head_dim))


def decode_partial_workspace_bytes(kv_len, num_q_heads: int, num_kv_heads: int,
                                   head_dim: int) -> int:
    kl = _host(kv_len, np.int32)
    return int(load_library().medha_decode_partial_workspace_bytes(
        _hp(kl), len(kl), num_q_heads, num_kv_heads, head_dim))


def describe_plan(prefix_len, chunk_len, num_q_heads: int, num_kv_heads: int, head_dim: int,
                  num_cus: int = 0):
    """Host-only: (entries, grid_rows, grid_keys, workspace_bytes) of the launch plan."""
    lib = load_library()
    pre, chk = _host(prefix_len, np.int32), _host(chunk_len, np.int32)
    entries = (PlanEntry * max(1, len(pre)))()
    g_rows, g_keys, ws = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_size_t(0)
    _check(lib.medha_describe_plan(_hp(pre), _hp(chk), len(pre), num_q_heads, num_kv_heads,
                                   head_dim, num_cus, entries, ctypes.byref(g_rows),
                                   ctypes.byref(g_keys), ctypes.byref(ws)))
    return list(entries)[:len(pre)], g_rows.value, g_keys.value, ws.value


def describe_slot(slot: int, num_kv_heads: int, n_split: int, n_row_tiles: int):
    """Host-only: (kv_head, split, row_tile) of a workgroup slot, or None if idle."""
    lib = load_library()
    h, s, r = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib.medha_describe_slot(slot, num_kv_heads, n_split, n_row_tiles, ctypes.byref(h),
                                 ctypes.byref(s), ctypes.byref(r))
    if rc < 0:
        _check(rc)
    return (h.value, s.value, r.value) if rc == 1 else None


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def chunked_prefill_attn(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                         page_table: torch.Tensor, page_table_offs, prefix_len, chunk_len,
                         softmax_scale: float, out: Optional[torch.Tensor] = None,
                         lse: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None):
    """q bf16 [tokens][h_q][d] (device); page_table int32 (device); the three
    length arrays live on the host.  Returns (out fp32 [tokens][h_q][d],
    lse fp32 [tokens][h_q])."""
    lib = load_library()
    assert q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous() and q.dim() == 3
    assert page_table.is_cuda and page_table.dtype == torch.int32 and page_table.is_contiguous()
    tokens, h_q, d = q.shape
    kv = _kv(k_pool, v_pool)
    offs = _host(page_table_offs, np.int64)
    pre, chk = _host(prefix_len, np.int32), _host(chunk_len, np.int32)
    batch = len(pre)
    assert len(chk) == batch and len(offs) == batch + 1 and int(chk.sum()) == tokens
    assert int(offs[-1]) <= page_table.numel()
    if out is None:
        out = torch.empty((tokens, h_q, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((tokens, h_q), dtype=torch.float32, device=q.device)
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == (tokens, h_q, d)
    assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.shape == (tokens, h_q)
    if workspace is None:
        workspace = _workspace(lib.medha_chunked_prefill_workspace_bytes(
            _hp(pre), _hp(chk), batch, h_q, kv.num_kv_heads, d), q.device)
    _check(lib.medha_chunked_prefill_attn(
        _dp(q), ctypes.byref(kv), _dp(page_table), _hp(offs), _hp(pre), _hp(chk), batch, h_q,
        float(softmax_scale), _dp(out), _dp(lse), _dp(workspace), workspace.numel(), _stream()))
    return out, lse


NOALLOC_SCRATCH_BYTES = 64 << 20


def chunked_prefill_attn_noalloc(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                                 page_table: torch.Tensor, page_table_offs, prefix_len, chunk_len,
                                 softmax_scale: float, out: torch.Tensor, lse: torch.Tensor):
    """chunked_prefill_attn through the entry point that allocates nothing: the caller passes
    every tensor, the split-KV partials go to the library's own scratch array."""
    lib = load_library()
    assert q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous() and q.dim() == 3
    assert page_table.is_cuda and page_table.dtype == torch.int32 and page_table.is_contiguous()
    tokens, h_q, d = q.shape
    kv = _kv(k_pool, v_pool)
    offs = _host(page_table_offs, np.int64)
    pre, chk = _host(prefix_len, np.int32), _host(chunk_len, np.int32)
    batch = len(pre)
    assert len(chk) == batch and len(offs) == batch + 1 and int(chk.sum()) == tokens
    assert int(offs[-1]) <= page_table.numel()
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == (tokens, h_q, d)
    assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.shape == (tokens, h_q)
    _check(lib.medha_chunked_prefill_attn_noalloc(
        _dp(q), ctypes.byref(kv), _dp(page_table), _hp(offs), _hp(pre), _hp(chk), batch, h_q,
        float(softmax_scale), _dp(out), _dp(lse), _stream()))
    return out, lse


def decode_partial_attn(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                        page_table: torch.Tensor, page_table_offs, q_index, kv_len,
                        softmax_scale: float, out_partial: Optional[torch.Tensor] = None,
                        lse_partial: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None):
    """q bf16 [num_queries][h_q][d]; returns (out_partial fp32 [items][h_q][d],
    lse_partial fp32 [items][h_q])."""
    lib = load_library()
    assert q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous() and q.dim() == 3
    assert page_table.is_cuda and page_table.dtype == torch.int32 and page_table.is_contiguous()
    num_queries, h_q, d = q.shape
    kv = _kv(k_pool, v_pool)
    offs = _host(page_table_offs, np.int64)
    qi, kl = _host(q_index, np.int32), _host(kv_len, np.int32)
    items = len(qi)
    assert len(kl) == items and len(offs) == items + 1
    assert int(offs[-1]) <= page_table.numel()
    if out_partial is None:
        out_partial = torch.empty((items, h_q, d), dtype=torch.float32, device=q.device)
    if lse_partial is None:
        lse_partial = torch.empty((items, h_q), dtype=torch.float32, device=q.device)
    assert out_partial.dtype == torch.float32 and out_partial.is_contiguous()
    assert lse_partial.dtype == torch.float32 and lse_partial.is_contiguous()
    assert out_partial.shape == (items, h_q, d) and lse_partial.shape == (items, h_q)
    if workspace is None:
        workspace = _workspace(lib.medha_decode_partial_workspace_bytes(
            _hp(kl), items, h_q, kv.num_kv_heads, d), q.device)
    _check(lib.medha_decode_partial_attn(
        _dp(q), num_queries, ctypes.byref(kv), _dp(page_table), _hp(offs), _hp(qi), _hp(kl), items,
        h_q, float(softmax_scale), _dp(out_partial), _dp(lse_partial), _dp(workspace),
        workspace.numel(), _stream()))
    return out_partial, lse_partial


def chunk_partial_workspace_bytes(chunk_len, kv_len, num_q_heads: int, num_kv_heads: int,
                                  head_dim: int) -> int:
    chk, kl = _host(chunk_len, np.int32), _host(kv_len, np.int32)
    return int(load_library().medha_chunk_partial_workspace_bytes(
        _hp(chk), _hp(kl), len(chk), num_q_heads, num_kv_heads, head_dim))


def chunk_partial_attn(q: torch.Tensor, k_pool: torch.Tensor, v_pool: torch.Tensor,
                       page_table: torch.Tensor, page_table_offs, q_row, chunk_len, kv_len,
                       visible0, softmax_scale: float,
                       out_partial: Optional[torch.Tensor] = None,
                       lse_partial: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None):
    """Item i: rows q_row[i] .. +chunk_len[i] of q bf16 [tokens][h_q][d] against the kv_len[i]
    keys of its page-table slice, row j seeing the first min(kv_len, max(0, visible0 + j)).
    Returns (out_partial fp32 [sum chunk_len][h_q][d], lse_partial fp32 [sum chunk_len][h_q])."""
    lib = load_library()
    assert q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous() and q.dim() == 3
    assert page_table.is_cuda and page_table.dtype == torch.int32 and page_table.is_contiguous()
    tokens, h_q, d = q.shape
    kv = _kv(k_pool, v_pool)
    offs = _host(page_table_offs, np.int64)
    qr, chk = _host(q_row, np.int32), _host(chunk_len, np.int32)
    kl, v0 = _host(kv_len, np.int32), _host(visible0, np.int32)
    items = len(qr)
    assert len(chk) == items and len(kl) == items and len(v0) == items and len(offs) == items + 1
    assert int(offs[-1]) <= page_table.numel()
    rows = int(chk.sum())
    if out_partial is None:
        out_partial = torch.empty((rows, h_q, d), dtype=torch.float32, device=q.device)
    if lse_partial is None:
        lse_partial = torch.empty((rows, h_q), dtype=torch.float32, device=q.device)
    assert out_partial.dtype == torch.float32 and out_partial.is_contiguous()
    assert lse_partial.dtype == torch.float32 and lse_partial.is_contiguous()
    assert out_partial.shape == (rows, h_q, d) and lse_partial.shape == (rows, h_q)
    if workspace is None:
        workspace = _workspace(lib.medha_chunk_partial_workspace_bytes(
            _hp(chk), _hp(kl), items, h_q, kv.num_kv_heads, d), q.device)
    _check(lib.medha_chunk_partial_attn(
        _dp(q), tokens, ctypes.byref(kv), _dp(page_table), _hp(offs), _hp(qr), _hp(chk), _hp(kl),
        _hp(v0), items, h_q, float(softmax_scale), _dp(out_partial), _dp(lse_partial),
        _dp(workspace), workspace.numel(), _stream()))
    return out_partial, lse_partial


def lse_merge(out_partial: torch.Tensor, lse_partial: torch.Tensor,
              out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None):
    """out_partial fp32 [S][rows][h_q][d], lse_partial fp32 [S][rows][h_q]."""
    lib = load_library()
    assert out_partial.is_cuda and out_partial.dtype == torch.float32
    assert lse_partial.dtype == torch.float32
    assert out_partial.is_contiguous() and lse_partial.is_contiguous() and out_partial.dim() == 4
    s, rows, h_q, d = out_partial.shape
    assert lse_partial.shape == (s, rows, h_q)
    if out is None:
        out = torch.empty((rows, h_q, d), dtype=torch.float32, device=out_partial.device)
    if lse is None:
        lse = torch.empty((rows, h_q), dtype=torch.float32, device=out_partial.device)
    assert out.is_contiguous() and lse.is_contiguous()
    assert out.shape == (rows, h_q, d) and lse.shape == (rows, h_q)
    _check(lib.medha_lse_merge(_dp(out_partial), _dp(lse_partial), s, rows, h_q, d, _dp(out),
                               _dp(lse), _stream()))
    return out, lse


def kv_append(k_new: torch.Tensor, v_new: torch.Tensor, k_pool: torch.Tensor,
              v_pool: torch.Tensor, page_table: torch.Tensor, page_table_offs, prefix_len,
              chunk_len) -> None:
    """k_new, v_new bf16 [tokens][h_kv][d] (device) are written into the pools in place."""
    lib = load_library()
    for t in (k_new, v_new):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 3
    assert k_new.shape == v_new.shape
    assert page_table.is_cuda and page_table.dtype == torch.int32 and page_table.is_contiguous()
    kv = _kv(k_pool, v_pool)
    tokens, h_kv, d = k_new.shape
    assert h_kv == kv.num_kv_heads and d == kv.head_dim
    offs = _host(page_table_offs, np.int64)
    pre, chk = _host(prefix_len, np.int32), _host(chunk_len, np.int32)
    batch = len(pre)
    assert len(chk) == batch and len(offs) == batch + 1 and int(chk.sum()) == tokens
    assert int(offs[-1]) <= page_table.numel()
    _check(lib.medha_kv_append(_dp(k_new), _dp(v_new), ctypes.byref(kv), _dp(page_table),
                               _hp(offs), _hp(pre), _hp(chk), batch, _stream()))
