"""Seeded synthetic inputs shaped like the paper's long-context workloads.

This module holds no attention arithmetic: it only draws random tensors, page
tables and length mixes.  It is the one module shared by the HIP path's tests,
the benchmark and the CPU oracle's tests, so both sides see the same bits.

Recipe (stands in for the Llama-3 8B / 70B long-context serving workloads of the
paper's evaluation, of which only shapes and lengths matter to this path):
Q, K, V are i.i.d. N(0,1) drawn in fp32 and rounded to bf16; the KV cache is a
pool of 16-token pages ``[num_pages][h_kv][16][d]`` and each sequence's page
table is a slice of one seeded permutation of the pool; softmax scale is
``1/sqrt(d)``; decode context lengths in the mixed batch are log-normal
(median 2048, sigma 1.0) clipped to [256, 16384].
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

PAGE_SIZE = 16


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def randn_bf16(shape, seed: int, device="cpu", slab: int = 1 << 26) -> torch.Tensor:
    """N(0,1) in fp32 rounded to bf16 (RNE), drawn slab by slab to bound memory."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    g = _gen(seed, device)
    for lo in range(0, n, slab):
        hi = min(n, lo + slab)
        out[lo:hi] = torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32).to(
            torch.bfloat16)
    return out.view(*shape)


def pages_for(n_tokens: int, page_size: int = PAGE_SIZE) -> int:
    return (int(n_tokens) + page_size - 1) // page_size


def permuted_page_tables(pages_per_seq: List[int], num_pages: int, seed: int):
    """One seeded permutation of [0, num_pages) cut into per-sequence slices.

    Returns (page_table int32 [sum pages], offsets int64 [len+1])."""
    total = int(sum(pages_per_seq))
    assert total <= num_pages
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    perm = rng.permutation(num_pages).astype(np.int32)
    offs = np.zeros(len(pages_per_seq) + 1, np.int64)
    offs[1:] = np.cumsum(np.asarray(pages_per_seq, np.int64))
    return perm[:total].copy(), offs


def lognormal_lengths(n: int, seed: int, median: float = 2048.0, sigma: float = 1.0,
                      lo: int = 256, hi: int = 16384) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    z = rng.standard_normal(n)
    return np.clip(np.rint(np.exp(math.log(median) + sigma * z)), lo, hi).astype(np.int32)


@dataclass
class PrefillBatch:
    """A batch for the chunked-prefill entry point (a decode is chunk_len 1)."""
    name: str
    h_q: int
    h_kv: int
    d: int
    prefix_len: np.ndarray            # int32 [batch]
    chunk_len: np.ndarray             # int32 [batch]
    page_table: np.ndarray            # int32, concatenated
    page_table_offs: np.ndarray       # int64 [batch+1]
    num_pages: int
    q: torch.Tensor                   # bf16 [sum chunk][h_q][d]
    k_pool: torch.Tensor              # bf16 [num_pages][h_kv][16][d]
    v_pool: torch.Tensor
    scale: float
    page_size: int = PAGE_SIZE
    meta: dict = field(default_factory=dict)

    @property
    def tokens(self) -> int:
        return int(self.chunk_len.sum())

    def algorithmic_flops(self) -> float:
        """4*d*h_q per visible (query, key) pair, exact causal count."""
        p = self.prefix_len.astype(np.float64)
        c = self.chunk_len.astype(np.float64)
        pairs = (c * p + c * (c + 1) / 2).sum()
        return 4.0 * self.d * self.h_q * float(pairs)

    def algorithmic_kv_bytes(self) -> float:
        """bf16 K and V of every token attended to, read once per sequence."""
        n = (self.prefix_len.astype(np.float64) + self.chunk_len).sum()
        return 2.0 * 2.0 * self.d * self.h_kv * float(n)


def make_prefill_batch(name: str, h_q: int, h_kv: int, d: int, prefix_len, chunk_len, seed: int,
                       device="cpu", num_pages: Optional[int] = None,
                       poison_unused: bool = False) -> PrefillBatch:
    prefix_len = np.asarray(prefix_len, np.int32).reshape(-1)
    chunk_len = np.asarray(chunk_len, np.int32).reshape(-1)
    need = [pages_for(int(p) + int(c)) for p, c in zip(prefix_len, chunk_len)]
    if num_pages is None:
        num_pages = max(1, int(sum(need)))
    pt, offs = permuted_page_tables(need, num_pages, seed * 1000 + 3)
    q = randn_bf16((int(chunk_len.sum()), h_q, d), seed * 1000 + 0, device)
    k_pool = randn_bf16((num_pages, h_kv, PAGE_SIZE, d), seed * 1000 + 1, device)
    v_pool = randn_bf16((num_pages, h_kv, PAGE_SIZE, d), seed * 1000 + 2, device)
    if poison_unused:
        poison_unused_slots(k_pool, v_pool, pt, offs, prefix_len + chunk_len)
    return PrefillBatch(name, h_q, h_kv, d, prefix_len, chunk_len, pt, offs, num_pages, q,
                        k_pool, v_pool, 1.0 / math.sqrt(d))


def poison_unused_slots(k_pool, v_pool, page_table, offs, kv_len) -> None:
    """NaN in every pool slot no sequence's token occupies (pages outside every
    table, and the tail slots of a partly filled last page)."""
    num_pages = k_pool.shape[0]
    used = torch.zeros(num_pages, PAGE_SIZE, dtype=torch.bool)
    for b, n in enumerate(np.asarray(kv_len).reshape(-1)):
        n = int(n)
        pages = page_table[int(offs[b]):int(offs[b]) + pages_for(n)]
        for i, pg in enumerate(pages):
            hi = min(PAGE_SIZE, n - i * PAGE_SIZE)
            used[int(pg), :hi] = True
    mask = (~used).to(k_pool.device)[:, None, :, None].expand_as(k_pool)
    k_pool.masked_fill_(mask, float("nan"))
    v_pool.masked_fill_(mask, float("nan"))


# ----------------------------------------------------------------------------
# The five named workloads.  ``scale_down`` shrinks the long axes for tests that
# run the full oracle; 1 gives the published shape.
# ----------------------------------------------------------------------------

def config1_tiny(device="cpu", seed: int = 1) -> PrefillBatch:
    """1 sequence, 2 q heads / 1 kv head, d 64, prefix 1024 + chunk 256, 80 pages."""
    return make_prefill_batch("cfg1_tiny", 2, 1, 64, [1024], [256], seed, device)


def config2_llama8b(device="cpu", seed: int = 2, prefix: int = 32768,
                    chunk: int = 2048) -> PrefillBatch:
    """Llama-3-8B layer: 32/8 heads, d 128, prefix 32768 + chunk 2048, 2176 pages."""
    return make_prefill_batch("cfg2_llama8b_prefill", 32, 8, 128, [prefix], [chunk], seed, device)


def config4_llama70b_tp(chunk: int, device="cpu", seed: int = 4, prefix: int = 1 << 20,
                        max_chunk: int = 8192) -> PrefillBatch:
    """One GPU's share of Llama-3-70B under TP8: 8 q heads / 1 kv head, d 128,
    prefix 1M; the pool is sized for the largest chunk of the sweep and reused."""
    return make_prefill_batch(f"cfg4_llama70b_tp_c{chunk}", 8, 1, 128, [prefix], [chunk], seed,
                              device, num_pages=pages_for(prefix + max_chunk))


def config5_mixed(device="cpu", seed: int = 5, prefix: int = 524288, chunk: int = 1024,
                  n_decode: int = 64) -> PrefillBatch:
    """One long request's prefill chunk plus 64 decodes (chunk_len 1) whose
    context lengths are log-normal; one shared pool, per-request page tables."""
    lens = lognormal_lengths(n_decode, seed * 1000 + 7)
    prefix_len = np.concatenate([[prefix], lens - 1]).astype(np.int32)
    chunk_len = np.concatenate([[chunk], np.ones(n_decode, np.int32)]).astype(np.int32)
    b = make_prefill_batch("cfg5_mixed", 32, 8, 128, prefix_len, chunk_len, seed, device)
    b.meta["decode_lens"] = lens
    b.meta["sigma"] = 1.0
    return b


@dataclass
class DecodeShards:
    """KV-cache-parallel decode: one query token, context cut into contiguous
    page-aligned shards, each an item of the decode-partial entry point."""
    name: str
    h_q: int
    h_kv: int
    d: int
    q: torch.Tensor                   # bf16 [1][h_q][d]
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    num_pages: int
    page_table: np.ndarray            # int32 [pages of the whole context]
    shard_offs: np.ndarray            # int64 [shards+1] page offsets of the shards
    shard_len: np.ndarray             # int32 [shards] tokens per shard
    q_index: np.ndarray               # int32 [shards] (all 0)
    scale: float
    page_size: int = PAGE_SIZE

    @property
    def context(self) -> int:
        return int(self.shard_len.sum())

    def algorithmic_kv_bytes(self) -> float:
        return 2.0 * 2.0 * self.d * self.h_kv * float(self.context)

    def algorithmic_flops(self) -> float:
        return 4.0 * self.d * self.h_q * float(self.context)


def config3_kvp_decode(device="cpu", seed: int = 3, context: int = 1 << 20,
                       shards: int = 4, h_q: int = 32, h_kv: int = 8, d: int = 128) -> DecodeShards:
    """1 request, 1,048,576-token context, 4 contiguous shards of 262,144."""
    assert context % (shards * PAGE_SIZE) == 0
    per = context // shards
    num_pages = pages_for(context)
    pt, _ = permuted_page_tables([num_pages], num_pages, seed * 1000 + 3)
    shard_offs = (np.arange(shards + 1, dtype=np.int64) * (per // PAGE_SIZE))
    q = randn_bf16((1, h_q, d), seed * 1000 + 0, device)
    k_pool = randn_bf16((num_pages, h_kv, PAGE_SIZE, d), seed * 1000 + 1, device)
    v_pool = randn_bf16((num_pages, h_kv, PAGE_SIZE, d), seed * 1000 + 2, device)
    return DecodeShards("cfg3_kvp_decode", h_q, h_kv, d, q, k_pool, v_pool, num_pages, pt,
                        shard_offs, np.full(shards, per, np.int32), np.zeros(shards, np.int32),
                        1.0 / math.sqrt(d))


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def sample_rows(total: int, seed: int, head: int = 16, tail: int = 16, rand: int = 96) -> np.ndarray:
    """First ``head``, last ``tail`` and ``rand`` seeded random token rows."""
    if total <= head + tail + rand:
        return np.arange(total, dtype=np.int64)
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    mid = rng.choice(np.arange(head, total - tail), size=rand, replace=False)
    rows = np.concatenate([np.arange(head), np.sort(mid), np.arange(total - tail, total)])
    return rows.astype(np.int64)
