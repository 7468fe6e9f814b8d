"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2409_17264_amd as medha
from paper_2409_17264_amd import workloads as wl
from tests.gpu_util import (LSE_TOL, O_TOL, check, edge_rows, gpu_prefill, oracle_prefill,
                            to_dev)

pytestmark = pytest.mark.gpu


# ----------------------------------------------------------------- lse merge
@pytest.mark.parametrize("splits,rows,h_q,d", [(1, 3, 2, 64), (4, 1, 32, 128), (7, 33, 5, 128),
                                               (2, 1000, 8, 64), (16, 17, 3, 32)])
def test_lse_merge_matches_oracle(splits, rows, h_q, d):
    rng = np.random.default_rng(splits * 1000 + rows)
    po = rng.standard_normal((splits, rows, h_q, d)).astype(np.float32)
    pl = (rng.standard_normal((splits, rows, h_q)) * 4).astype(np.float32)
    if splits > 1:
        pl[0, 0, :] = -np.inf              # an empty shard
        pl[:, rows - 1, 0] = -np.inf       # a row with no keys at all
    ro, rl = oracle.lse_merge(po.astype(np.float64), pl.astype(np.float64))
    o, l = medha.lse_merge(torch.from_numpy(po).cuda(), torch.from_numpy(pl).cuda())
    torch.cuda.synchronize()
    o, l = o.cpu().numpy(), l.cpu().numpy()
    assert np.array_equal(np.isneginf(l), np.isneginf(rl))
    fin = np.isfinite(rl)
    assert np.max(np.abs(o - ro)) < 1e-5
    assert np.max(np.abs(l[fin] - rl[fin])) < 1e-5


# ------------------------------------------------------------ config 1, tiny
def test_config1_tiny_full_parity():
    b = to_dev(wl.config1_tiny("cpu"))
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, "cfg1")


# ------------------------------------------------- adversarial small shapes
SHAPES = [(2, 1, 64), (8, 2, 128), (4, 4, 64), (8, 1, 128), (32, 8, 128)]
CASES = [(0, 1), (0, 17), (1, 2), (15, 16), (16, 33), (63, 1), (64, 64), (65, 100), (200, 300),
         (1000, 70), (37, 513)]


@pytest.mark.parametrize("h_q,h_kv,d", SHAPES)
@pytest.mark.parametrize("prefix,chunk", CASES)
def test_small_shapes(h_q, h_kv, d, prefix, chunk):
    b = to_dev(wl.make_prefill_batch("s", h_q, h_kv, d, [prefix], [chunk],
                                     seed=prefix * 7 + chunk, poison_unused=True))
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, f"hq{h_q} hkv{h_kv} d{d} P{prefix} c{chunk}")


def test_ragged_batch_mixed_modes():
    """Prefill chunks of several sizes and decodes (chunk_len 1) in one call,
    with NaN in every unused pool slot and extra unreferenced pages."""
    prefix = [300, 0, 77, 1500, 15, 16, 4000, 0]
    chunk = [130, 40, 1, 1, 1, 2, 260, 1]
    b = to_dev(wl.make_prefill_batch("rag", 8, 2, 128, prefix, chunk, seed=123,
                                     num_pages=600, poison_unused=True))
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, "ragged batch")


# ------------------------------------------------------------------ decode
@pytest.mark.parametrize("h_q,h_kv,d", [(32, 8, 128), (8, 1, 128), (2, 1, 64), (4, 4, 64),
                                        (64, 1, 128), (48, 1, 64)])
def test_decode_partial_lengths(h_q, h_kv, d):
    """Lengths from empty to 20000 keys; groups of more than 32 query heads per KV head take
    the row-split kernel instead of the key-split one."""
    lens = np.array([0, 1, 15, 16, 17, 127, 128, 129, 511, 1000, 5000, 20000], np.int32)
    items = len(lens)
    need = [wl.pages_for(int(n)) for n in lens]
    num_pages = sum(need) + 5
    pt, offs = wl.permuted_page_tables(need, num_pages, 77)
    q = wl.randn_bf16((3, h_q, d), 1, "cpu")
    k = wl.randn_bf16((num_pages, h_kv, 16, d), 2, "cpu")
    v = wl.randn_bf16((num_pages, h_kv, 16, d), 3, "cpu")
    wl.poison_unused_slots(k, v, pt, offs, lens)
    q_index = (np.arange(items) % 3).astype(np.int32)
    scale = d ** -0.5
    ro, rl = oracle.decode_partial_attn(wl.bf16_bits(q), wl.bf16_bits(k), wl.bf16_bits(v), pt,
                                        offs, q_index, lens, scale)
    o, l = medha.decode_partial_attn(q.cuda(), k.cuda(), v.cuda(), torch.from_numpy(pt).cuda(),
                                     offs, q_index, lens, scale)
    torch.cuda.synchronize()
    check(o.cpu().numpy(), l.cpu().numpy(), ro, rl, f"decode hq{h_q} hkv{h_kv} d{d}")


def test_kvp_shards_merge_equals_unsplit_scaled_config3():
    """Config 3 at 1/16 scale: 65,536-token context in 4 shards, merged, against
    the oracle's unsplit attention (full oracle)."""
    c = wl.config3_kvp_decode("cpu", context=65536)
    ro, rl = oracle.decode_partial_attn(wl.bf16_bits(c.q), wl.bf16_bits(c.k_pool),
                                        wl.bf16_bits(c.v_pool), c.page_table,
                                        np.array([0, len(c.page_table)], np.int64), [0],
                                        [c.context], c.scale)
    pto = c.shard_offs
    po, pl = medha.decode_partial_attn(c.q.cuda(), c.k_pool.cuda(), c.v_pool.cuda(),
                                       torch.from_numpy(c.page_table).cuda(), pto, c.q_index,
                                       c.shard_len, c.scale)
    # per-shard partials against the oracle's partials
    so, sl = oracle.decode_partial_attn(wl.bf16_bits(c.q), wl.bf16_bits(c.k_pool),
                                        wl.bf16_bits(c.v_pool), c.page_table, pto, c.q_index,
                                        c.shard_len, c.scale)
    torch.cuda.synchronize()
    check(po.cpu().numpy(), pl.cpu().numpy(), so, sl, "cfg3/16 shard partials")
    o, l = medha.lse_merge(po[:, None].contiguous(), pl[:, None].contiguous())
    torch.cuda.synchronize()
    check(o.cpu().numpy(), l.cpu().numpy(), ro, rl, "cfg3/16 merged vs unsplit")


# -------------------------------------------- bit-exact indexing through attention
def test_needle_is_bit_exact_on_gpu():
    """A key scoring far above all others takes the whole softmax mass in fp32
    too, so O must equal that key's V row bit for bit: an end-to-end check of the
    page-table gather through the attention kernels (row-split and key-split)."""
    h_q, h_kv, d, P = 8, 2, 128, 700
    for chunk in (1, 70):
        for needle in (0, 15, 16, 63, 64, 127, 128, 511, 699, P + chunk - 1, P + 5):
            if needle >= P + chunk:
                continue
            b = wl.make_prefill_batch("n", h_q, h_kv, d, [P], [chunk], seed=needle + chunk,
                                      poison_unused=True)
            b.q.fill_(1.0)
            valid = ~torch.isnan(b.k_pool.float())
            b.k_pool[valid] = 0
            page, slot = int(b.page_table[needle // 16]), needle % 16
            b.k_pool[page, :, slot, :] = 64.0
            b = to_dev(b)
            out, lse = gpu_prefill(b)
            v = b.v_pool.float().cpu().numpy()
            s_needle = np.float32(b.scale) * np.float32(d * 64.0)
            for j in range(chunk):
                for h in range(h_q):
                    if needle <= P + j:
                        assert np.array_equal(out[j, h], v[page, h // (h_q // h_kv), slot]), \
                            (chunk, needle, j, h)
                        assert abs(lse[j, h] - s_needle) < 1e-3
                    else:
                        assert abs(lse[j, h] - np.log(P + j + 1)) < 1e-3


# ------------------------------------- scores that outgrow the softmax reference point
def _rising_keys(profile, n_keys, rng):
    """Per-key score level g(t); the key vector is g(t) plus small noise in every dim."""
    t = np.arange(n_keys)
    if profile == "staircase":       # near the end, every 16-key slice far above the one before
        return 2.5 * np.maximum(0, t // 16 - (n_keys // 16 - 20))
    if profile == "jumps":           # flat stretches, rare large jumps at arbitrary keys
        return np.cumsum(np.where(rng.random(n_keys) < 1 / 200, 4.0, 0.0)) + 0.1 * rng.standard_normal(n_keys)
    if profile == "ramp":            # slow drift: many tiles pass before the reference must move
        return 0.003 * t
    if profile == "sawtooth":        # up and far down again
        return 3.0 * ((t // 40) % 5)
    raise ValueError(profile)


@pytest.mark.parametrize("d,h_q,h_kv", [(128, 8, 2), (64, 4, 1)])
@pytest.mark.parametrize("profile", ["staircase", "jumps", "ramp", "sawtooth"])
def test_scores_rising_along_the_sequence(profile, d, h_q, h_kv):
    """The prefill kernel exponentiates fully visible tiles against the reference point it
    already holds and falls back to the exact route when a checked row sum says the
    scores outgrew it; these inputs make that happen in every position of a tile."""
    P, chunk = 2000, 130
    rng = np.random.default_rng(len(profile) * 100 + d)
    b = wl.make_prefill_batch("rise", h_q, h_kv, d, [P], [chunk], seed=d + len(profile),
                              poison_unused=True)
    g = _rising_keys(profile, P + chunk, rng)
    b.q.fill_(1.0)
    b.q[:, ::2, :] *= 0.5   # every other head at half the slope
    for t in range(P + chunk):
        page, slot = int(b.page_table[t // 16]), t % 16
        noise = 0.25 * rng.standard_normal((h_kv, d))
        b.k_pool[page, :, slot, :] = torch.from_numpy(g[t] + noise).to(torch.bfloat16)
    b = to_dev(b)
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, f"rising {profile} d{d}")


def test_page_permutation_is_bitwise_invariant_on_gpu():
    a = wl.make_prefill_batch("a", 8, 2, 128, [1000, 300], [200, 1], seed=5)
    num_pages = a.num_pages + 11
    rng = np.random.default_rng(3)
    perm = rng.permutation(num_pages).astype(np.int32)[:len(a.page_table)]
    k2 = torch.zeros(num_pages, 2, 16, 128, dtype=torch.bfloat16)
    v2 = torch.zeros_like(k2)
    k2[perm.astype(np.int64)] = a.k_pool[a.page_table.astype(np.int64)]
    v2[perm.astype(np.int64)] = a.v_pool[a.page_table.astype(np.int64)]
    wl.poison_unused_slots(k2, v2, perm, a.page_table_offs, a.prefix_len + a.chunk_len)
    a = to_dev(a)
    o1, l1 = gpu_prefill(a)
    o1b, l1b = gpu_prefill(a)
    assert np.array_equal(o1, o1b) and np.array_equal(l1, l1b)      # run-to-run determinism
    a.k_pool, a.v_pool, a.page_table = k2.cuda(), v2.cuda(), perm
    o2, l2 = gpu_prefill(a)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_chunk_by_chunk_equals_one_shot_on_gpu():
    """Processing a sequence in ragged chunks gives the same rows as one causal
    pass (within tolerance; the tile schedule differs)."""
    n = 900
    full = to_dev(wl.make_prefill_batch("f", 8, 2, 128, [0], [n], seed=17))
    fo, fl = gpu_prefill(full)
    ro, rl = oracle_prefill(full)
    check(fo, fl, ro, rl, "one-shot causal")
    start = 0
    for c in (1, 100, 33, 256, 510):
        part = wl.PrefillBatch("p", 8, 2, 128, np.array([start], np.int32),
                               np.array([c], np.int32), full.page_table, full.page_table_offs,
                               full.num_pages, full.q[start:start + c].contiguous(), full.k_pool,
                               full.v_pool, full.scale)
        o, l = gpu_prefill(part)
        check(o, l, ro[start:start + c], rl[start:start + c], f"chunk@{start}+{c}")
        start += c
    assert start == n


# ---------------------------------------------------------- error handling
def test_invalid_arguments_are_rejected_without_writing():
    b = to_dev(wl.make_prefill_batch("e", 8, 2, 128, [100], [10], seed=1))
    pt = torch.from_numpy(b.page_table).cuda()
    out = torch.full((10, 8, 128), 7.0, device="cuda")
    lse = torch.full((10, 8), 7.0, device="cuda")
    with pytest.raises(medha.MedhaError) as e:       # page table too short
        medha.chunked_prefill_attn(b.q, b.k_pool, b.v_pool, pt, [0, 3], [100], [10], b.scale,
                                   out, lse)
    assert e.value.code == -1
    with pytest.raises(medha.MedhaError) as e:       # chunk_len 0
        medha.chunked_prefill_attn(b.q[:0], b.k_pool, b.v_pool, pt, b.page_table_offs, [100], [0],
                                   b.scale, out[:0], lse[:0])
    assert e.value.code == -1
    with pytest.raises(medha.MedhaError) as e:       # heads not divisible
        medha.chunked_prefill_attn(b.q[:, :7].contiguous(), b.k_pool, b.v_pool, pt,
                                   b.page_table_offs, [100], [10], b.scale,
                                   out[:, :7].contiguous(), lse[:, :7].contiguous())
    assert e.value.code == -1
    k32 = b.k_pool[..., :32].contiguous()
    with pytest.raises(medha.MedhaError) as e:       # unsupported head_dim
        medha.chunked_prefill_attn(b.q[..., :32].contiguous(), k32, k32, pt, b.page_table_offs,
                                   [100], [10], b.scale)
    assert e.value.code == -2
    # a split plan without enough workspace
    big = to_dev(wl.make_prefill_batch("w", 8, 1, 128, [20000], [64], seed=2))
    need = medha.chunked_prefill_workspace_bytes(big.prefix_len, big.chunk_len, 8, 1, 128)
    assert need > 256
    with pytest.raises(medha.MedhaError) as e:
        medha.chunked_prefill_attn(big.q, big.k_pool, big.v_pool,
                                   torch.from_numpy(big.page_table).cuda(), big.page_table_offs,
                                   big.prefix_len, big.chunk_len, big.scale,
                                   workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()) and bool((lse == 7.0).all())


def test_other_entry_points_reject_bad_arguments_without_writing():
    """Every validation failure of the decode-partial, chunk-partial, merge and append entry
    points returns its code with nothing enqueued: sentinel-filled outputs and pools stay
    as they were."""
    b = to_dev(wl.make_prefill_batch("e2", 8, 2, 128, [100], [20], seed=3))
    pt = torch.from_numpy(b.page_table).cuda()
    offs = b.page_table_offs
    out = torch.full((20, 8, 128), 7.0, device="cuda")
    lse = torch.full((20, 8), 7.0, device="cuda")
    k_before, v_before = b.k_pool.clone(), b.v_pool.clone()

    def expect(code, fn, *a, **kw):
        with pytest.raises(medha.MedhaError) as e:
            fn(*a, **kw)
        assert e.value.code == code, (fn.__name__, e.value.code)

    q1 = b.q[:2].contiguous()
    o1, l1 = out[:1], lse[:1]
    dec = medha.decode_partial_attn
    expect(-1, dec, q1, b.k_pool, b.v_pool, pt, offs, [0], [-1], b.scale, o1, l1)    # kv_len < 0
    expect(-1, dec, q1, b.k_pool, b.v_pool, pt, offs, [2], [50], b.scale, o1, l1)    # q_index
    expect(-1, dec, q1, b.k_pool, b.v_pool, pt, offs, [0], [500], b.scale, o1, l1)   # table short
    expect(-1, dec, q1, b.k_pool, b.v_pool, pt, [3, 1], [0], [10], b.scale, o1, l1)  # offsets
    expect(-1, dec, q1, b.k_pool, b.v_pool, pt, offs, [0], [50], float("nan"), o1, l1)
    k32 = b.k_pool[..., :32].contiguous()
    expect(-2, dec, q1[..., :32].contiguous(), k32, k32, pt, offs, [0], [50], b.scale)
    long = to_dev(wl.make_prefill_batch("e3", 8, 2, 128, [99999], [1], seed=4))
    assert medha.decode_partial_workspace_bytes([100000], 8, 2, 128) > 256
    expect(-3, dec, long.q, long.k_pool, long.v_pool, torch.from_numpy(long.page_table).cuda(),
           long.page_table_offs, [0], [100000], long.scale, o1, l1,
           workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))

    chk = medha.chunk_partial_attn
    for q_row, c, n, vis, code in (([1], [20], [120], [101], -1), ([0], [0], [120], [101], -1),
                                   ([0], [20], [-1], [101], -1), ([0], [20], [1000], [101], -1),
                                   ([0], [20], [120], [(1 << 30) + 1], -1)):
        rows = int(sum(c))
        expect(code, chk, b.q, b.k_pool, b.v_pool, pt, offs, q_row, c, n, vis, b.scale,
               out[:rows], lse[:rows])

    po = torch.ones((3, 20, 8, 128), device="cuda")
    pl = torch.ones((3, 20, 8), device="cuda")
    lib = medha.load_library()
    dp = lambda t: t.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream
    assert lib.medha_lse_merge(dp(po), dp(pl), 0, 20, 8, 128, dp(out), dp(lse), stream) == -1
    assert lib.medha_lse_merge(dp(po), dp(pl), 3, -1, 8, 128, dp(out), dp(lse), stream) == -1
    assert lib.medha_lse_merge(dp(po), dp(pl), 3, 20, 8, 126, dp(out), dp(lse), stream) == -2
    assert lib.medha_lse_merge(dp(po) + 4, dp(pl), 3, 20, 8, 128, dp(out), dp(lse), stream) == -1
    assert lib.medha_lse_merge(dp(po), dp(pl), 3, 20, 8, 128, None, dp(lse), stream) == -1

    k_new = torch.ones((20, 2, 128), dtype=torch.bfloat16, device="cuda")
    app = medha.kv_append
    expect(-1, app, k_new, k_new, b.k_pool, b.v_pool, pt, offs, [-1], [20])          # prefix < 0
    expect(-1, app, k_new[:0], k_new[:0], b.k_pool, b.v_pool, pt, offs, [100], [0])  # empty chunk
    expect(-1, app, k_new, k_new, b.k_pool, b.v_pool, pt, [0, 3], [100], [20])       # table short
    k40 = torch.ones((40, 2, 128), dtype=torch.bfloat16, device="cuda")
    # the second sequence is the bad one: nothing of the first may be written either
    expect(-1, app, k40, k40, b.k_pool, b.v_pool, pt, [0, 8, 8], [100, 0], [20, 20])
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()) and bool((lse == 7.0).all())
    assert torch.equal(b.k_pool.view(torch.int16), k_before.view(torch.int16))
    assert torch.equal(b.v_pool.view(torch.int16), v_before.view(torch.int16))


@pytest.mark.parametrize("n_seq,h_q,h_kv,d", [(150, 8, 2, 128), (200, 4, 4, 64)])
def test_batches_of_more_than_64_sequences_per_kernel(n_seq, h_q, h_kv, d):
    """More than 64 sequences in BOTH kernels of one call (descriptors travel in the kernel
    arguments, 64 per launch): every third sequence is a multi-row chunk, some long enough to be
    KV-split and merged, the others decodes of assorted lengths."""
    rng = np.random.default_rng(n_seq)
    chunk = np.where(np.arange(n_seq) % 3 == 0, rng.integers(9, 60, n_seq), 1).astype(np.int32)
    prefix = rng.integers(0, 700, n_seq).astype(np.int32)
    prefix[::29] += 6000
    b = wl.make_prefill_batch("many", h_q, h_kv, d, prefix, chunk, seed=n_seq, poison_unused=True)
    e, gr, gk, _ = medha.describe_plan(b.prefix_len, b.chunk_len, h_q, h_kv, d)
    assert sum(x.mode == 0 for x in e) > 0 and sum(x.mode == 1 for x in e) > 64
    if h_q // h_kv * 9 > 32:
        assert sum(x.mode == 0 for x in e) > 0
    ro, rl = oracle_prefill(b)
    b = to_dev(b)
    out, lse = gpu_prefill(b)
    check(out, lse, ro, rl, f"{n_seq} sequences hq{h_q} hkv{h_kv} d{d}")


# ------------------------------------------------------------------- KV append
@pytest.mark.parametrize("h_kv,d,n_seq", [(2, 64, 1), (8, 128, 5), (1, 128, 70)])
def test_kv_append_is_bit_exact(h_kv, d, n_seq):
    """Pools after the GPU append equal the pools after the oracle's append, bit for bit:
    every new row in its (page, slot), nothing else touched.  70 sequences take two launches."""
    rng = np.random.default_rng(h_kv * 100 + n_seq)
    prefix = rng.integers(0, 70, n_seq).astype(np.int32)
    chunk = rng.integers(1, 50, n_seq).astype(np.int32)
    prefix[0], chunk[0] = 0, 1
    pages_per = (prefix + chunk + 15) // 16
    num_pages = int(pages_per.sum()) + 5
    offs = np.concatenate([[0], np.cumsum(pages_per)]).astype(np.int64)
    pt = rng.permutation(num_pages).astype(np.int32)[:offs[-1]]
    k_pool = rng.integers(0, 1 << 16, (num_pages, h_kv, 16, d)).astype(np.uint16)
    v_pool = rng.integers(0, 1 << 16, (num_pages, h_kv, 16, d)).astype(np.uint16)
    tokens = int(chunk.sum())
    k_new = rng.integers(0, 1 << 16, (tokens, h_kv, d)).astype(np.uint16)
    v_new = rng.integers(0, 1 << 16, (tokens, h_kv, d)).astype(np.uint16)

    def dev(a):
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    kp, vp = dev(k_pool), dev(v_pool)
    medha.kv_append(dev(k_new), dev(v_new), kp, vp, torch.from_numpy(pt).cuda(), offs, prefix,
                    chunk)
    torch.cuda.synchronize()
    oracle.kv_append(k_new, v_new, k_pool, v_pool, pt, offs, prefix, chunk)
    assert np.array_equal(kp.view(torch.int16).cpu().numpy().view(np.uint16), k_pool)
    assert np.array_equal(vp.view(torch.int16).cpu().numpy().view(np.uint16), v_pool)


def test_kv_append_skips_page_ids_outside_the_pool():
    h_kv, d = 2, 64
    k_pool = torch.zeros(4, h_kv, 16, d, dtype=torch.bfloat16, device="cuda")
    v_pool = torch.zeros_like(k_pool)
    new = torch.ones(20, h_kv, d, dtype=torch.bfloat16, device="cuda")
    pt = torch.tensor([2, 1 << 20], dtype=torch.int32, device="cuda")   # second page id is bad
    medha.kv_append(new, new, k_pool, v_pool, pt, [0, 2], [0], [20])
    torch.cuda.synchronize()
    assert float(k_pool[2].float().sum()) == 16 * h_kv * d              # first 16 tokens landed
    assert float(k_pool.float().sum()) == 16 * h_kv * d                 # the other 4 went nowhere


def test_chunk_by_chunk_prefill_on_the_gpu_equals_one_shot_oracle():
    """End to end on the device: empty (NaN) cache, then per chunk append + attention; all rows
    against the oracle's one-shot causal pass over the full cache."""
    n = 1500
    full = wl.make_prefill_batch("e2e", 8, 2, 128, [0], [n], seed=77)
    ro, rl = oracle_prefill(full)
    pages = full.page_table[:(n + 15) // 16].astype(np.int64)
    k_seq = full.k_pool[pages].permute(0, 2, 1, 3).reshape(-1, 2, 128)[:n].contiguous().cuda()
    v_seq = full.v_pool[pages].permute(0, 2, 1, 3).reshape(-1, 2, 128)[:n].contiguous().cuda()
    k_live = torch.full_like(full.k_pool, float("nan")).cuda()
    v_live = torch.full_like(full.v_pool, float("nan")).cuda()
    pt = torch.from_numpy(full.page_table).cuda()
    q = full.q.cuda()
    outs, lses, start = [], [], 0
    for c in [1, 300, 17, 512, 70, 600]:
        medha.kv_append(k_seq[start:start + c], v_seq[start:start + c], k_live, v_live, pt,
                        full.page_table_offs, [start], [c])
        o, l = medha.chunked_prefill_attn(q[start:start + c].contiguous(), k_live, v_live, pt,
                                          full.page_table_offs, [start], [c], full.scale)
        outs.append(o)
        lses.append(l)
        start += c
    assert start == n
    torch.cuda.synchronize()
    check(torch.cat(outs).cpu().numpy(), torch.cat(lses).cpu().numpy(), ro, rl, "chunk-by-chunk")


# ------------------------------------- KV-cache-parallel partials of a prefill chunk
def _oracle_chunk_partial(b, pt, pto, q_row, chunk_len, kv_len, vis0):
    return oracle.chunk_partial_attn(wl.bf16_bits(b.q), wl.bf16_bits(b.k_pool),
                                     wl.bf16_bits(b.v_pool), pt, pto, q_row, chunk_len, kv_len,
                                     vis0, b.scale)


@pytest.mark.parametrize("h_q,h_kv,d", [(8, 2, 128), (4, 4, 64), (32, 8, 128)])
def test_chunk_partial_items_match_oracle(h_q, h_kv, d):
    """Items of every kind in one call: unmasked shards, causal shards, rows that see nothing,
    an empty shard, ragged lengths, chunks small enough for the key-split kernel."""
    n = 900
    b = wl.make_prefill_batch("cp", h_q, h_kv, d, [n - 200], [200], seed=h_q + d,
                              poison_unused=True)
    #        q_row chunk kv_len visible0   slice (first page, of the one sequence)
    items = [(0, 200, 700, 700, 0),      # shard before the chunk: everything visible
             (0, 200, 900, 701, 0),      # the whole sequence, causal: plain chunked prefill
             (0, 200, 132, -67, 48),     # shard starting at key 768: early rows see nothing
             (10, 150, 0, 5, 0),         # empty shard
             (0, 3, 333, 2000, 16),      # tiny chunk (key-split kernel), no mask
             (197, 3, 100, 98, 0),       # tiny chunk, causal tail
             (5, 64, 77, 30, 32),        # ragged, mask starts inside the first tile
             (0, 200, 64, 64, 0)]        # exactly one tile
    if h_q // h_kv > 8:
        pytest.skip("group size")
    q_row, chunk, kv_len, vis0, first = (np.array(x, np.int32) for x in zip(*items))
    slices = [b.page_table[f:f + (kl + 15) // 16] for f, kl in zip(first, kv_len)]
    pt = np.concatenate(slices)
    pto = np.concatenate([[0], np.cumsum([len(s) for s in slices])]).astype(np.int64)
    ro, rl = _oracle_chunk_partial(b, pt, pto, q_row, chunk, kv_len, vis0)
    b = to_dev(b)
    o, l = medha.chunk_partial_attn(b.q, b.k_pool, b.v_pool, torch.from_numpy(pt).cuda(), pto,
                                    q_row, chunk, kv_len, vis0, b.scale)
    torch.cuda.synchronize()
    check(o.cpu().numpy(), l.cpu().numpy(), ro, rl, f"chunk partial hq{h_q} d{d}")


@pytest.mark.parametrize("prefix,chunk,shards", [(4096, 512, 4), (1000, 300, 3), (0, 700, 2),
                                                 (8192, 8, 8)])
def test_chunk_kvp_shards_merge_to_unsplit_attention(prefix, chunk, shards):
    """A chunk against page-aligned KV shards (only the last ones causal), merged with the LSE
    merge, against the oracle's plain chunked prefill and the library's own unsplit call."""
    h_q, h_kv, d = 8, 2, 128
    b = wl.make_prefill_batch("kvp", h_q, h_kv, d, [prefix], [chunk], seed=prefix + shards)
    ro, rl = oracle_prefill(b)
    n = prefix + chunk
    per = ((n + shards - 1) // shards + 15) // 16 * 16
    cuts = [min(n, i * per) for i in range(shards + 1)]
    slices = [b.page_table[lo // 16:(hi + 15) // 16] for lo, hi in zip(cuts[:-1], cuts[1:])]
    pt = np.concatenate(slices)
    pto = np.concatenate([[0], np.cumsum([len(s) for s in slices])]).astype(np.int64)
    kv_len = np.diff(cuts).astype(np.int32)
    vis0 = np.array([prefix + 1 - lo for lo in cuts[:-1]], np.int32)
    b = to_dev(b)
    po, pl = medha.chunk_partial_attn(b.q, b.k_pool, b.v_pool, torch.from_numpy(pt).cuda(), pto,
                                      np.zeros(shards, np.int32), np.full(shards, chunk, np.int32),
                                      kv_len, vis0, b.scale)
    o, l = medha.lse_merge(po.view(shards, chunk, h_q, d), pl.view(shards, chunk, h_q))
    torch.cuda.synchronize()
    check(o.cpu().numpy(), l.cpu().numpy(), ro, rl, f"chunk KVP P{prefix} c{chunk} S{shards}")
    uo, ul = gpu_prefill(b)
    assert np.max(np.abs(o.cpu().numpy() - uo)) < 2e-3
    assert np.max(np.abs(l.cpu().numpy() - ul)) < 1e-4


def test_chunk_partial_rejects_bad_arguments():
    b = to_dev(wl.make_prefill_batch("bad", 8, 2, 128, [100], [20], seed=1))
    pt = torch.from_numpy(b.page_table).cuda()
    args = dict(q_row=[0], chunk_len=[20], kv_len=[120], visible0=[101])
    for key, bad in (("q_row", [1]), ("chunk_len", [0]), ("kv_len", [-1]), ("kv_len", [1000]),
                     ("visible0", [(1 << 30) + 1])):
        a = dict(args)
        a[key] = bad
        with pytest.raises(medha.MedhaError):
            medha.chunk_partial_attn(b.q, b.k_pool, b.v_pool, pt, b.page_table_offs, a["q_row"],
                                     a["chunk_len"], a["kv_len"], a["visible0"], b.scale)


# ------------------------------------------ small chunks against a long cache
@pytest.mark.parametrize("h_q,h_kv,d,prefix,chunk", [(8, 1, 128, 150_000, 32), (8, 2, 64, 70_000, 8),
                                                     (16, 4, 128, 60_000, 40)])
def test_small_chunk_long_prefix_many_way_split(h_q, h_kv, d, prefix, chunk):
    """The regime adaptive chunking ends in (section 3.2): a few dozen tokens against a very long
    cache.  The KV axis is split tens to hundreds of ways and the partials are merged by the
    workgroup-per-row merge kernel."""
    b = wl.make_prefill_batch("small", h_q, h_kv, d, [prefix], [chunk], seed=chunk + d)
    e, _, _, _ = medha.describe_plan(b.prefix_len, b.chunk_len, h_q, h_kv, d)
    assert e[0].n_split > 16
    ro, rl = oracle_prefill(b)
    b = to_dev(b)
    out, lse = gpu_prefill(b)
    check(out, lse, ro, rl, f"small chunk hq{h_q} d{d} P{prefix} c{chunk} split{e[0].n_split}")


# ------------------------------------------------------------ softmax scale values
@pytest.mark.parametrize("d,prefix", [(128, 64 * 20 + 7), (128, 64 * 23), (64, 64 * 22 - 1)])
def test_walks_that_end_around_the_exact_route_warm_up(d, prefix):
    """A launch that fills the device without a KV split (8 kv heads x 32 row tiles), whose
    walks are 21 to 56 tiles long: they leave the exact-route head of the walk (24 tiles) after
    0 to 32 speculative tiles, at every position of the 4-stage ring."""
    b = to_dev(wl.make_prefill_batch("warm", 32, 8, d, [prefix], [2048], seed=prefix + d))
    e, grid_rows, _, _ = medha.describe_plan(b.prefix_len, b.chunk_len, b.h_q, b.h_kv, b.d)
    assert e[0].n_split == 1 and grid_rows == 256
    out, lse = gpu_prefill(b)
    rows = edge_rows(b, prefix, 8, 8, 40, 24)
    ro, rl = oracle_prefill(b, rows)
    check(out[rows], lse[rows], ro, rl, f"d{d} P{prefix} c2048, {len(rows)} sampled rows")


@pytest.mark.parametrize("scale", [0.0, -0.1, 0.5, 1e-3, -2.0])
def test_softmax_scale_values(scale):
    """The scale is an argument, not 1/sqrt(d) by construction: zero (uniform weights), negative
    (its sign is folded into Q inside the kernels), large (sharply peaked rows), tiny.  One
    batch through both kernels: a chunk of 150 tokens and three decodes."""
    b = wl.make_prefill_batch("sc", 8, 2, 128, [600, 0, 77, 1000], [150, 1, 1, 1], seed=17,
                              poison_unused=True)
    b.scale = scale
    ro, rl = oracle_prefill(b)
    b = to_dev(b)
    out, lse = gpu_prefill(b)
    # LSE grows with |scale| * |q.k|: keep the absolute tolerance where fp32 can hold it
    assert np.max(np.abs(rl)) < 2000
    # |scale| >= 0.2 gives sharply peaked rows (one or two keys carry a row); the contract is
    # the same for them
    check(out, lse, ro, rl, f"scale {scale}")


@pytest.mark.parametrize("d,scale", [(64, 1.0), (128, 1.0), (128, -1.0), (64, 0.5)])
def test_peaked_rows_long_prefix(d, scale):
    """Rows carried by one or two keys (scores with a standard deviation of several nats),
    through the row-split kernel's unmasked tile walk over a prefix of several thousand keys and
    through its KV-split + merge: the weight of a dominant key must come through the bf16
    rounding of P intact, wherever along the walk that key sits."""
    b = wl.make_prefill_batch("peak", 8, 2, d, [4500, 9000], [96, 40], seed=300 + d,
                              poison_unused=True)
    b.scale = scale
    ro, rl = oracle_prefill(b)
    # peaked indeed: the largest weight of a typical row exceeds one half
    assert np.median(np.max(np.abs(ro), axis=2)) > 0.5
    b = to_dev(b)
    out, lse = gpu_prefill(b)
    check(out, lse, ro, rl, f"peaked rows d{d} scale {scale}")


# ------------------------------------------------------ seeded random batch mixes
@pytest.mark.parametrize("seed", range(12))
def test_random_batches(seed):
    """Seeded random batches: head counts, head dim, 1..70 sequences (more than 64 are
    launched in groups), prefixes 0..3000 and chunks 1..260 in any mix, so that
    sequences of both kernels, split and unsplit, share one call."""
    rng = np.random.default_rng(1000 + seed)
    h_kv = int(rng.choice([1, 2, 4, 8]))
    h_q = h_kv * int(rng.choice([1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    n = int(rng.choice([1, 2, 5, 17, 70]))
    prefix = rng.integers(0, 3000, n).astype(np.int32)
    chunk = np.where(rng.random(n) < 0.5, 1, rng.integers(1, 260, n)).astype(np.int32)
    if n >= 17:                       # keep the oracle's share of the run short
        prefix = (prefix // 4).astype(np.int32)
        chunk = np.minimum(chunk, 40).astype(np.int32)
    b = to_dev(wl.make_prefill_batch("rnd", h_q, h_kv, d, prefix, chunk, seed=seed + 500,
                                     poison_unused=True))
    out, lse = gpu_prefill(b)
    ro, rl = oracle_prefill(b)
    check(out, lse, ro, rl, f"random batch seed {seed}: hq{h_q} hkv{h_kv} d{d} n{n}")
