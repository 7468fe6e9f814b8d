"""Test-side helpers: an independent numpy brute force and small utilities.

The brute force is a second, differently structured statement of the same
definition the C oracle follows (gather to contiguous K/V, materialise the full
score matrix, mask, library log-sum-exp, matmul); it is used to pin the oracle
on tiny shapes and is never used by the product.
"""
import numpy as np
from scipy.special import logsumexp


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def gather_contiguous(pool_bits, pages, n):
    """[num_pages][h_kv][16][d] + page ids -> fp64 [h_kv][n][d]."""
    sel = bf16_to_f64(pool_bits[np.asarray(pages)])          # [np][h_kv][16][d]
    npg, h_kv, ps, d = sel.shape
    return sel.transpose(1, 0, 2, 3).reshape(h_kv, npg * ps, d)[:, :n]


def brute_force_prefill(q_bits, k_bits, v_bits, page_table, offs, prefix_len, chunk_len, scale):
    tokens, h_q, d = q_bits.shape
    h_kv, ps = k_bits.shape[1], k_bits.shape[2]
    group = h_q // h_kv
    qf = bf16_to_f64(q_bits)
    out = np.zeros((tokens, h_q, d))
    lse = np.zeros((tokens, h_q))
    start = 0
    for b in range(len(prefix_len)):
        p, c = int(prefix_len[b]), int(chunk_len[b])
        n = p + c
        pages = page_table[int(offs[b]):int(offs[b]) + (n + ps - 1) // ps]
        kk = gather_contiguous(k_bits, pages, n)
        vv = gather_contiguous(v_bits, pages, n)
        visible = np.arange(n)[None, :] <= (p + np.arange(c))[:, None]      # [c][n]
        for h in range(h_q):
            s = float(scale) * (qf[start:start + c, h] @ kk[h // group].T)   # [c][n]
            s = np.where(visible, s, -np.inf)
            z = logsumexp(s, axis=1)
            out[start:start + c, h] = np.exp(s - z[:, None]) @ vv[h // group]
            lse[start:start + c, h] = z
        start += c
    return out, lse
