"""fp64 CPU oracle for the paged attention path (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrapper over ``medha_oracle.c``; see that file's header for what is
computed and which passages of the paper it follows.  Only tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; the
product package never does.

All tensors are numpy arrays.  bf16 data travels as ``uint16`` bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i32, i64, f64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.medha_oracle_chunked_prefill.restype = ctypes.c_int
        lib.medha_oracle_chunked_prefill.argtypes = [
            vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, i32, i32, f64, vp, i64, vp, vp]
        lib.medha_oracle_decode_partial.restype = ctypes.c_int
        lib.medha_oracle_decode_partial.argtypes = [
            vp, i32, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, i32, i32, f64, vp, vp]
        lib.medha_oracle_chunk_partial.restype = ctypes.c_int
        lib.medha_oracle_chunk_partial.argtypes = [
            vp, i32, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, i32, i32, f64, vp, vp]
        lib.medha_oracle_lse_merge.restype = ctypes.c_int
        lib.medha_oracle_lse_merge.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp]
        lib.medha_oracle_num_threads.restype = ctypes.c_int
        lib.medha_oracle_num_threads.argtypes = []
        _LIB = lib
    return _LIB


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_lib().medha_oracle_num_threads())


def chunked_prefill_attn(q, k_pool, v_pool, page_table, page_table_offs, prefix_len, chunk_len,
                         scale, rows=None):
    """q uint16 [tokens][h_q][d]; pools uint16 [pages][h_kv][page_size][d].

    Returns (out float64 [R][h_q][d], lse float64 [R][h_q]) where R is every
    token row, or ``len(rows)`` when a list of token-row indices is given.
    """
    q, qp = _arr(q, np.uint16)
    k_pool, kp = _arr(k_pool, np.uint16)
    v_pool, vpp = _arr(v_pool, np.uint16)
    assert q.ndim == 3 and k_pool.ndim == 4 and k_pool.shape == v_pool.shape
    tokens, h_q, d = q.shape
    num_pages, h_kv, page_size, d2 = k_pool.shape
    assert d2 == d
    pt, ptp = _arr(page_table, np.int32)
    offs, offp = _arr(page_table_offs, np.int64)
    pre, prep = _arr(prefix_len, np.int32)
    chk, chkp = _arr(chunk_len, np.int32)
    batch = pre.shape[0]
    assert chk.shape[0] == batch and offs.shape[0] == batch + 1
    assert int(chk.sum()) == tokens and int(offs[-1]) <= pt.shape[0]
    if rows is None:
        n_rows, rp = tokens, None
    else:
        rows, rp = _arr(rows, np.int64)
        n_rows = rows.shape[0]
    out = np.empty((n_rows, h_q, d), np.float64)
    lse = np.empty((n_rows, h_q), np.float64)
    rc = _lib().medha_oracle_chunked_prefill(
        qp, kp, vpp, num_pages, page_size, h_kv, d, ptp, offp, prep, chkp, batch, h_q,
        float(scale), rp, n_rows, out.ctypes.data_as(ctypes.c_void_p),
        lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"oracle chunked_prefill failed with code {rc}")
    return out, lse


def decode_partial_attn(q, k_pool, v_pool, page_table, page_table_offs, q_index, kv_len, scale):
    """q uint16 [num_queries][h_q][d]. Returns (out [items][h_q][d], lse [items][h_q])."""
    q, qp = _arr(q, np.uint16)
    k_pool, kp = _arr(k_pool, np.uint16)
    v_pool, vpp = _arr(v_pool, np.uint16)
    num_queries, h_q, d = q.shape
    num_pages, h_kv, page_size, d2 = k_pool.shape
    assert d2 == d and k_pool.shape == v_pool.shape
    pt, ptp = _arr(page_table, np.int32)
    offs, offp = _arr(page_table_offs, np.int64)
    qi, qip = _arr(q_index, np.int32)
    kl, klp = _arr(kv_len, np.int32)
    items = qi.shape[0]
    assert kl.shape[0] == items and offs.shape[0] == items + 1 and int(offs[-1]) <= pt.shape[0]
    out = np.empty((items, h_q, d), np.float64)
    lse = np.empty((items, h_q), np.float64)
    rc = _lib().medha_oracle_decode_partial(
        qp, num_queries, kp, vpp, num_pages, page_size, h_kv, d, ptp, offp, qip, klp, items, h_q,
        float(scale), out.ctypes.data_as(ctypes.c_void_p), lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"oracle decode_partial failed with code {rc}")
    return out, lse


def chunk_partial_attn(q, k_pool, v_pool, page_table, page_table_offs, q_row, chunk_len, kv_len,
                       visible0, scale):
    """Item i: query rows q_row[i] .. +chunk_len[i] of q (uint16 [tokens][h_q][d]) against the
    kv_len[i] keys of its page-table slice; row j sees the first
    min(kv_len, max(0, visible0[i] + j)) of them.
    Returns (out [sum chunk_len][h_q][d], lse [sum chunk_len][h_q])."""
    q, qp = _arr(q, np.uint16)
    k_pool, kp = _arr(k_pool, np.uint16)
    v_pool, vpp = _arr(v_pool, np.uint16)
    tokens, h_q, d = q.shape
    num_pages, h_kv, page_size, d2 = k_pool.shape
    assert d2 == d and k_pool.shape == v_pool.shape
    pt, ptp = _arr(page_table, np.int32)
    offs, offp = _arr(page_table_offs, np.int64)
    qr, qrp = _arr(q_row, np.int32)
    chk, chkp = _arr(chunk_len, np.int32)
    kl, klp = _arr(kv_len, np.int32)
    v0, v0p = _arr(visible0, np.int32)
    items = qr.shape[0]
    assert chk.shape[0] == items and kl.shape[0] == items and v0.shape[0] == items
    assert offs.shape[0] == items + 1 and int(offs[-1]) <= pt.shape[0]
    rows = int(chk.sum())
    out = np.empty((rows, h_q, d), np.float64)
    lse = np.empty((rows, h_q), np.float64)
    rc = _lib().medha_oracle_chunk_partial(
        qp, tokens, kp, vpp, num_pages, page_size, h_kv, d, ptp, offp, qrp, chkp, klp, v0p, items,
        h_q, float(scale), out.ctypes.data_as(ctypes.c_void_p),
        lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"oracle chunk_partial failed with code {rc}")
    return out, lse


def lse_merge(out_partial, lse_partial):
    """out_partial float64 [S][rows][h_q][d], lse_partial [S][rows][h_q]."""
    op, opp = _arr(out_partial, np.float64)
    lp, lpp = _arr(lse_partial, np.float64)
    s, rows, h_q, d = op.shape
    assert lp.shape == (s, rows, h_q)
    out = np.empty((rows, h_q, d), np.float64)
    lse = np.empty((rows, h_q), np.float64)
    rc = _lib().medha_oracle_lse_merge(opp, lpp, s, rows, h_q, d,
                                       out.ctypes.data_as(ctypes.c_void_p),
                                       lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"oracle lse_merge failed with code {rc}")
    return out, lse


def kv_append(k_new, v_new, k_pool, v_pool, page_table, page_table_offs, prefix_len, chunk_len):
    """The definition of the cache append, token by token (paper section 3.1: a chunk's keys
    and values join the paged cache): token j of sequence b, row sum(chunk_len[:b]) + j of the
    new arrays, lands at position prefix_len[b] + j, i.e. page
    page_table[offs[b] + position // page_size], slot position % page_size, for every KV head.

    k_new, v_new uint16 [tokens][h_kv][d]; pools uint16 [pages][h_kv][page_size][d] are
    modified IN PLACE (and returned).  Plain Python loop: meant for test-sized inputs.
    """
    assert k_pool.dtype == np.uint16 and v_pool.dtype == np.uint16
    assert k_new.shape == v_new.shape and k_pool.shape == v_pool.shape
    page_size = k_pool.shape[2]
    row = 0
    for b in range(len(prefix_len)):
        for j in range(int(chunk_len[b])):
            position = int(prefix_len[b]) + j
            page = int(page_table[int(page_table_offs[b]) + position // page_size])
            slot = position % page_size
            k_pool[page, :, slot, :] = k_new[row]
            v_pool[page, :, slot, :] = v_new[row]
            row += 1
    return k_pool, v_pool
