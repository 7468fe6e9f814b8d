"""The entry point that allocates nothing (for callers that cannot call hipMalloc: graph
capture, tight serving loops): its split-KV partials live in a scratch array inside the
library's device image.  Checked against the ordinary entry point, bit for bit (the plan and the
kernels are the same), on calls in a row that share the array, the later ones smaller."""
import numpy as np
import pytest
import torch

import paper_2409_17264_amd as medha
from paper_2409_17264_amd import binding
from paper_2409_17264_amd import workloads as wl
from tests.gpu_util import check, oracle_prefill, to_dev

pytestmark = pytest.mark.gpu


def _both(b):
    pt = torch.from_numpy(b.page_table).cuda()
    ref_o, ref_l = medha.chunked_prefill_attn(b.q, b.k_pool, b.v_pool, pt, b.page_table_offs,
                                              b.prefix_len, b.chunk_len, b.scale)
    out = torch.full((b.tokens, b.h_q, b.d), float("nan"), device="cuda")
    lse = torch.full((b.tokens, b.h_q), float("nan"), device="cuda")
    medha.chunked_prefill_attn_noalloc(b.q, b.k_pool, b.v_pool, pt, b.page_table_offs,
                                       b.prefix_len, b.chunk_len, b.scale, out, lse)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy(), ref_o.cpu().numpy(), ref_l.cpu().numpy()


def test_noalloc_entry_point_matches_the_workspace_one_on_consecutive_calls():
    # first call: 128 tokens x 8 heads against 40,000 keys, KV split many ways (partials fill
    # a few MB of the scratch array); second: a smaller split batch that lands on the same
    # bytes; third: a batch that is not split at all
    shapes = [([40000], [128]), ([9000, 3000, 17], [40, 1, 5]), ([100], [300])]
    for i, (prefix, chunk) in enumerate(shapes):
        b = wl.make_prefill_batch("noalloc", 8, 1, 128, prefix, chunk, seed=60 + i,
                                  poison_unused=True)
        need = medha.chunked_prefill_workspace_bytes(b.prefix_len, b.chunk_len, 8, 1, 128)
        assert (need > 256) == (i < 2)
        ro, rl = oracle_prefill(b)
        b = to_dev(b)
        out, lse, ref_o, ref_l = _both(b)
        assert np.array_equal(out, ref_o) and np.array_equal(lse, ref_l), f"call {i}"
        check(out, lse, ro, rl, f"no-alloc entry point, call {i}")


def test_noalloc_entry_point_refuses_what_does_not_fit():
    # 8160 tokens x 8 heads are 255 row tiles, one short of filling 256 compute units, so the
    # planner splits the keys in two and the partials are twice the output: more than the
    # scratch array holds.  Refused before anything is enqueued (the pools here are tiny:
    # nothing may touch them).
    prefix, chunk = [100000], [8160]
    need = medha.chunked_prefill_workspace_bytes(prefix, chunk, 8, 1, 128)
    assert need > binding.NOALLOC_SCRATCH_BYTES
    q = wl.randn_bf16((8160, 8, 128), 1, "cuda:0")
    pool = wl.randn_bf16((4, 1, 16, 128), 2, "cuda:0")
    pt = torch.zeros(7000, dtype=torch.int32, device="cuda")
    out = torch.full((8160, 8, 128), 7.0, device="cuda")
    lse = torch.full((8160, 8), 7.0, device="cuda")
    with pytest.raises(medha.MedhaError) as e:
        medha.chunked_prefill_attn_noalloc(q, pool, pool, pt, [0, 7000], prefix, chunk, 0.1,
                                           out, lse)
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()) and bool((lse == 7.0).all())
