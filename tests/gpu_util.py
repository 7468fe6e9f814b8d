"""Glue for the GPU parity tests: run a workload through the C ABI (via the
binding) and through the CPU oracle on the same bits."""
import numpy as np
import torch

import oracle
import paper_2409_17264_amd as medha
from paper_2409_17264_amd import workloads as wl

O_TOL = 1e-2      # max-abs tolerance on O   (bf16 inputs, fp32 accumulation)
LSE_TOL = 1e-3    # max-abs tolerance on LSE


def to_dev(batch):
    dev = torch.device("cuda:0")
    batch.q = batch.q.to(dev)
    batch.k_pool = batch.k_pool.to(dev)
    batch.v_pool = batch.v_pool.to(dev)
    return batch


def gpu_prefill(batch):
    pt = torch.from_numpy(batch.page_table).to("cuda:0")
    out, lse = medha.chunked_prefill_attn(batch.q, batch.k_pool, batch.v_pool, pt,
                                          batch.page_table_offs, batch.prefix_len,
                                          batch.chunk_len, batch.scale)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def oracle_prefill(batch, rows=None):
    return oracle.chunked_prefill_attn(wl.bf16_bits(batch.q), wl.bf16_bits(batch.k_pool),
                                       wl.bf16_bits(batch.v_pool), batch.page_table,
                                       batch.page_table_offs, batch.prefix_len, batch.chunk_len,
                                       batch.scale, rows)


def edge_rows(batch, seed, head=8, tail=8, rand=16, edges=8, seq=0):
    """Token rows of sequence `seq` to compare one by one at full size: the first `head` and
    last `tail` rows and `rand` seeded random ones (wl.sample_rows), plus up to `edges` rows
    that sit where the kernels change regime: on either side of a 256-row workgroup edge and
    of a 128-row one (row = token * group + head-in-group), and rows whose last visible key is
    the last or the first key of a 64-key tile."""
    c, p = int(batch.chunk_len[seq]), int(batch.prefix_len[seq])
    g = batch.h_q // batch.h_kv
    rows = set(wl.sample_rows(c, seed, head, tail, rand).tolist())
    rng = np.random.Generator(np.random.PCG64(seed + 77))
    cand = []
    for rows_per_wg in (256, 128):
        tok = max(1, rows_per_wg // g)
        cand += [t + o for t in range(tok, c, tok) for o in (-1, 0)]
    first = (-(p + 1)) % 64                 # first row whose last visible key ends a tile
    cand += [j + o for j in range(first, c, 64) for o in (0, 1) if j + o < c]
    cand = sorted(set(cand) - rows)
    if cand:
        pick = rng.choice(len(cand), size=min(edges, len(cand)), replace=False)
        rows |= {cand[i] for i in pick}
    return np.array(sorted(rows), np.int64)


def check(out, lse, ref_out, ref_lse, what=""):
    assert np.isfinite(out).all(), f"{what}: non-finite O"
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isneginf(lse), np.isneginf(ref_lse)), f"{what}: -inf pattern"
    eo = float(np.max(np.abs(out - ref_out))) if out.size else 0.0
    el = float(np.max(np.abs(lse[fin] - ref_lse[fin]))) if fin.any() else 0.0
    scale = float(np.max(np.abs(ref_out))) if out.size else 1.0
    print(f"[parity] {what}: max|dO|={eo:.3e} (max|O|={scale:.3e}) max|dLSE|={el:.3e}", flush=True)
    assert eo <= O_TOL, f"{what}: O error {eo}"
    assert el <= LSE_TOL, f"{what}: LSE error {el}"
    # tighter, relative: bf16 rounding of the probabilities is the only large error source
    assert eo <= 2e-2 * max(scale, 1e-6) + 1e-6, f"{what}: relative O error {eo / scale}"
    return eo, el
