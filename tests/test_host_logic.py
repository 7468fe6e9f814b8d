"""CPU-only tests of the C-ABI library: it loads, exports every symbol the
header declares, and its host-side planner covers the work exactly once."""
import os
import re

import numpy as np
import pytest

import paper_2409_17264_amd as medha
from paper_2409_17264_amd import binding, policy, yardstick

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    declared = {}
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", name)).read()
        body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)      # drop comments
        declared[name] = set(re.findall(r"\b(medha_[a-z0-9_]+)\s*\(", body))
    assert sorted(declared) == ["medha.h", "medha_policy.h", "medha_yardstick.h"]
    product = declared["medha.h"] | declared["medha_policy.h"]
    bound = set(binding.EXPORTS) | set(policy.EXPORTS)
    assert product == bound, product ^ bound
    assert declared["medha_yardstick.h"] == set(yardstick.EXPORTS)
    lib = medha.load_library()
    for name in product:
        assert getattr(lib, name) is not None
    ylib = yardstick.load_library()
    for name in yardstick.EXPORTS:
        assert getattr(ylib, name) is not None
        assert not hasattr(lib, name)          # the yardsticks are not in the product's ABI
    assert lib.medha_abi_version() == 1
    assert lib.medha_strerror(0) == b"ok"
    assert b"workspace" in lib.medha_strerror(-3)


def test_workspace_queries_reject_bad_arguments():
    assert medha.chunked_prefill_workspace_bytes([10], [0], 8, 2, 128) == 0       # empty chunk
    assert medha.chunked_prefill_workspace_bytes([10], [4], 7, 2, 128) == 0       # 7 % 2
    assert medha.chunked_prefill_workspace_bytes([10], [4], 8, 2, 96) == 0        # head_dim
    assert medha.decode_partial_workspace_bytes([-1], 8, 2, 128) == 0
    assert medha.decode_partial_workspace_bytes([5], 64, 1, 128) >= 256           # group > 32: row-split
    assert medha.chunked_prefill_workspace_bytes([100], [16], 8, 2, 128) >= 256


def _check_plan(prefix, chunk, h_q, h_kv, d, num_cus):
    entries, grid_rows, grid_keys, ws = medha.describe_plan(prefix, chunk, h_q, h_kv, d, num_cus)
    gqa = h_q // h_kv
    spans = {0: [], 1: []}
    part_rows = 0
    for p, c, e in zip(prefix, chunk, entries):
        n_rows = c * gqa
        assert e.mode == (1 if n_rows <= 32 else 0)
        assert e.rows_per_wg in ((32,) if e.mode else (128, 256))
        assert e.tile_keys == (128 if e.mode else 64)
        assert e.n_row_tiles == -(-n_rows // e.rows_per_wg)
        kv_tiles = max(1, -(-(p + c) // e.tile_keys))
        # the splits tile the KV axis: enough to cover it, none empty
        assert e.n_split * e.tiles_per_split >= kv_tiles
        assert (e.n_split - 1) * e.tiles_per_split < kv_tiles
        items = h_kv * e.n_split * e.n_row_tiles
        assert e.n_slots == 8 * -(-items // 8)
        spans[e.mode].append((e.work_start, e.n_slots, min(e.tiles_per_split, kv_tiles)))
        # every (kv head, split, row tile) is owned by exactly one slot
        seen = set()
        for s in range(e.n_slots):
            it = medha.describe_slot(s, h_kv, e.n_split, e.n_row_tiles)
            if it is not None:
                assert it not in seen
                assert 0 <= it[0] < h_kv and 0 <= it[1] < e.n_split and 0 <= it[2] < e.n_row_tiles
                seen.add(it)
        assert len(seen) == items
        # row tiles sharing (kv head, split) sit on one die (slot % 8) when they fit
        per_die = -(-items // 8)
        if per_die % e.n_row_tiles == 0:
            dies = {}
            for s in range(e.n_slots):
                it = medha.describe_slot(s, h_kv, e.n_split, e.n_row_tiles)
                if it is not None:
                    dies.setdefault(it[:2], set()).add(s % 8)
            assert all(len(v) == 1 for v in dies.values())
        if e.n_split > 1:
            part_rows += e.n_split * c
    # per launch the sequences' slot ranges tile [0, grid) in some order, and that order puts
    # the workgroups with the longest walks first
    for mode, grid in ((0, grid_rows), (1, grid_keys)):
        end, prev_walk = 0, None
        for start, n_slots, walk in sorted(spans[mode]):
            assert start == end
            end += n_slots
            assert prev_walk is None or walk <= prev_walk
            prev_walk = walk
        assert end == grid
    need = part_rows * h_q * (d + 1) * 4
    assert need <= ws <= need + 1024 + 64 * len(prefix)
    return entries, grid_rows, grid_keys


def test_plans_of_the_named_workloads():
    # cfg2: 8 kv heads x 32 row tiles of 256 rows fill 256 compute units, no KV split
    e, gr, gk = _check_plan([32768], [2048], 32, 8, 128, 256)
    assert (e[0].n_row_tiles, e[0].n_split, gr, gk) == (32, 1, 256, 0)
    # cfg4: few row tiles -> KV split so that about 256 workgroups exist
    for c, tiles, split in [(512, 16, 16), (1024, 32, 8), (2048, 64, 4), (4096, 128, 2),
                            (8192, 256, 1)]:
        e, gr, _ = _check_plan([1 << 20], [c], 8, 1, 128, 256)
        assert (e[0].n_row_tiles, e[0].n_split) == (tiles, split) and gr == 256
    # cfg3: 4 shards x 8 kv heads, split into 8 workgroups per compute unit
    e, _, gk = _check_plan([262143] * 4, [1] * 4, 32, 8, 128, 256)
    assert all(x.mode == 1 and x.n_split == 64 for x in e) and gk == 2048
    # cfg1
    e, gr, _ = _check_plan([1024], [256], 2, 1, 64, 256)
    assert e[0].n_row_tiles == 2 and e[0].n_split > 1


def test_plans_of_ragged_batches():
    rng = np.random.default_rng(0)
    for trial in range(30):
        batch = int(rng.integers(1, 12))
        h_kv = int(rng.choice([1, 2, 4, 8]))
        gqa = int(rng.choice([1, 2, 4, 8]))
        prefix = [int(x) for x in rng.integers(0, 70000, batch)]
        chunk = [int(rng.choice([1, 1, 2, 5, 40, 300, 2000])) for _ in range(batch)]
        _check_plan(prefix, chunk, h_kv * gqa, h_kv, int(rng.choice([64, 128])),
                    int(rng.choice([8, 64, 256, 304])))
    # a decode over zero keys is planned too
    e, _, _ = _check_plan([-1, 0], [1, 1], 8, 2, 128, 256)
    assert e[0].n_split == 1


def test_bench_refuses_more_than_one_gpu_and_finds_its_traffic_figures():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr
    # every counter summary bench.py reads an HBM figure from is there and holds one
    src = open(os.path.join(ROOT, "bench.py")).read()
    names = set(re.findall(r'"([a-z0-9_]+\.txt)"', src))
    names |= {f"prefill_kernel_cfg4_c{c}.txt" for c in (32, 128, 512, 1024, 2048, 4096, 8192)}
    assert {"prefill_kernel_cfg2.txt", "decode_kernel_cfg3.txt", "mixed_cfg5.txt"} <= names
    for name in sorted(names):
        lines = [l for l in open(os.path.join(ROOT, "profiles", name))
                 if l.startswith("hbm_bytes_per_launch")]
        assert lines and float(lines[0].split("=")[1].split()[0]) > 1e6, name
