"""GPU parity on the named workloads: scaled-down versions against the full
oracle, and the published sizes against oracle rows sampled one by one."""
import numpy as np
import pytest
import torch

import oracle
import paper_2409_17264_amd as medha
from paper_2409_17264_amd import workloads as wl
from tests.gpu_util import check, edge_rows, gpu_prefill, oracle_prefill, to_dev

pytestmark = pytest.mark.gpu


def test_config2_scaled_full_oracle():
    b = to_dev(wl.config2_llama8b("cpu", prefix=2048, chunk=384))
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, "cfg2 scaled (P2048 c384)")


def test_config4_scaled_split_kv_full_oracle():
    """8 q heads / 1 kv head with a long prefix and a small chunk: few row tiles,
    so the KV axis is split across workgroups and merged."""
    b = to_dev(wl.config4_llama70b_tp(128, "cpu", prefix=40000, max_chunk=128))
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, "cfg4 scaled (P40000 c128)")


def test_config5_scaled_mixed_batch_full_oracle():
    b = to_dev(wl.config5_mixed("cpu", prefix=8192, chunk=256, n_decode=64))
    out, lse = gpu_prefill(b)
    rows = np.concatenate([wl.sample_rows(256, 5, 8, 8, 32), np.arange(256, 256 + 64)])
    ro, rl = oracle_prefill(b, rows)
    check(out[rows], lse[rows], ro, rl, "cfg5 scaled (P8192 c256 + 64 decodes)")


def test_config2_full_size_sampled_rows():
    b = wl.config2_llama8b("cuda:0")
    out, lse = gpu_prefill(b)
    rows = edge_rows(b, 2, 16, 16, 32, 16)
    ro, rl = oracle_prefill(b, rows)
    check(out[rows], lse[rows], ro, rl, f"cfg2 full size, {len(rows)} sampled rows x 32 heads")


@pytest.mark.parametrize("chunk", [512, 1024, 2048, 4096, 8192])
def test_config4_full_size_sampled_rows(chunk):
    """Every chunk length of the adaptive-chunk sweep at the 1,048,576-token prefix, in the
    launch shape the benchmark times (16-way down to no KV split; 256-row workgroups)."""
    b = wl.config4_llama70b_tp(chunk, "cuda:0")
    out, lse = gpu_prefill(b)
    rows = edge_rows(b, 40 + chunk, 8, 8, 16, 8)
    ro, rl = oracle_prefill(b, rows)
    check(out[rows], lse[rows], ro, rl,
          f"cfg4 c{chunk} full size, {len(rows)} sampled rows x 8 heads")
    del b
    torch.cuda.empty_cache()


def test_config3_full_size_kvp_decode():
    """1M-token context, 4 shards of 262,144, merged; the oracle computes the
    unsplit attention of all 32 heads."""
    c = wl.config3_kvp_decode("cuda:0")
    pt = torch.from_numpy(c.page_table).cuda()
    po, pl = medha.decode_partial_attn(c.q, c.k_pool, c.v_pool, pt, c.shard_offs, c.q_index,
                                       c.shard_len, c.scale)
    o, l = medha.lse_merge(po[:, None].contiguous(), pl[:, None].contiguous())
    torch.cuda.synchronize()
    ro, rl = oracle.decode_partial_attn(wl.bf16_bits(c.q), wl.bf16_bits(c.k_pool),
                                        wl.bf16_bits(c.v_pool), c.page_table,
                                        np.array([0, len(c.page_table)], np.int64), [0],
                                        [c.context], c.scale)
    check(o.cpu().numpy(), l.cpu().numpy(), ro, rl, "cfg3 full size merged vs unsplit oracle")


def test_config5_full_size_sampled_rows():
    b = wl.config5_mixed("cuda:0")
    out, lse = gpu_prefill(b)
    pre = edge_rows(b, 5, 16, 16, 32, 8)
    rows = np.concatenate([pre, np.arange(1024, 1024 + 64)]).astype(np.int64)
    ro, rl = oracle_prefill(b, rows)
    check(out[rows], lse[rows], ro, rl,
          f"cfg5 full size: {len(pre)} prefill rows + all 64 decodes")


def test_config4_full_size_chunk_kvp_and_small_chunk():
    """The other launch shapes bench.py times on the 1M-token cache: a 2048-token chunk
    against 4 page-aligned KV shards (only the last causal) merged with the LSE merge, a
    32-token chunk whose KV axis is split 253 ways and a 128-token chunk (4 row tiles x 64 KV
    ranges); all against oracle rows sampled one by one from plain chunked prefill."""
    b = wl.config4_llama70b_tp(2048, "cuda:0")
    prefix, chunk, shards = int(b.prefix_len[0]), 2048, 4
    n = prefix + chunk
    per = ((n + shards - 1) // shards + 15) // 16 * 16
    cuts = [min(n, i * per) for i in range(shards + 1)]
    slices = [b.page_table[lo // 16:(hi + 15) // 16] for lo, hi in zip(cuts[:-1], cuts[1:])]
    pto = np.concatenate([[0], np.cumsum([len(s) for s in slices])]).astype(np.int64)
    po, pl = medha.chunk_partial_attn(
        b.q, b.k_pool, b.v_pool, torch.from_numpy(np.concatenate(slices)).cuda(), pto,
        np.zeros(shards, np.int32), np.full(shards, chunk, np.int32),
        np.diff(cuts).astype(np.int32), np.array([prefix + 1 - lo for lo in cuts[:-1]], np.int32),
        b.scale)
    o, l = medha.lse_merge(po.view(shards, chunk, b.h_q, b.d), pl.view(shards, chunk, b.h_q))
    torch.cuda.synchronize()
    rows = edge_rows(b, 77, 4, 4, 6, 2)
    ro, rl = oracle_prefill(b, rows)
    check(o.cpu().numpy()[rows], l.cpu().numpy()[rows], ro, rl,
          f"cfg4 c2048 as 4 KV shards + merge, {len(rows)} sampled rows x 8 heads")
    # the same cache, first 32 tokens of the chunk only
    small = wl.PrefillBatch("cfg4_c32", b.h_q, b.h_kv, b.d, b.prefix_len, np.array([32], np.int32),
                            b.page_table, b.page_table_offs, b.num_pages, b.q[:32].contiguous(),
                            b.k_pool, b.v_pool, b.scale)
    e, _, _, _ = medha.describe_plan(small.prefix_len, small.chunk_len, small.h_q, small.h_kv,
                                     small.d)
    assert e[0].n_split > 200
    out, lse = gpu_prefill(small)
    rows = np.arange(32, dtype=np.int64)
    ro, rl = oracle_prefill(small, rows)
    check(out[rows], lse[rows], ro, rl, "cfg4 c32 (253-way split), all 32 rows x 8 heads")
    # and the first 128 tokens: 4 row tiles x 64 KV ranges
    mid = wl.PrefillBatch("cfg4_c128", b.h_q, b.h_kv, b.d, b.prefix_len, np.array([128], np.int32),
                          b.page_table, b.page_table_offs, b.num_pages, b.q[:128].contiguous(),
                          b.k_pool, b.v_pool, b.scale)
    e, _, _, _ = medha.describe_plan(mid.prefix_len, mid.chunk_len, mid.h_q, mid.h_kv, mid.d)
    assert e[0].n_row_tiles == 4 and e[0].n_split == 64
    out, lse = gpu_prefill(mid)
    rows = edge_rows(mid, 78, 4, 4, 8, 4)
    ro, rl = oracle_prefill(mid, rows)
    check(out[rows], lse[rows], ro, rl,
          f"cfg4 c128 (4 row tiles x 64 KV ranges), {len(rows)} sampled rows x 8 heads")
