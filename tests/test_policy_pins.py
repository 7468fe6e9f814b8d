"""Pins of the policy oracle (chunk-size selection, prefill-time estimation, relative-slack
scheduling) against what the paper prints and what the mathematics fixes.  No GPU."""
import math

import numpy as np
import pytest

from oracle import policy as P


def _golden():
    vals = {}
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    for line in open(path):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            vals[k.strip()] = float(v)
    return vals


def test_space_sharing_example_from_the_paper():
    """Section 4.3: a long prefill with 20 % relative slack yields 20 % of a 20 ms budget and
    uses 16 ms.  With a pure per-token model the chunk is then floor(16 ms / t_token)."""
    g = _golden()
    m = P.TimeModel(t_token=7e-6)
    c = P.get_chunk_size(m, 0, 10**9, True, False, g["space_sharing_rel_slack"], 0.4, 0.0,
                         g["space_sharing_t_target_s"], 10**6)
    assert c == math.floor(g["space_sharing_t_used_s"] / 7e-6) == 2285
    # the yielded fraction is capped (Algorithm 2's rho_max = 0.4) and never negative
    assert P.get_chunk_size(m, 0, 10**9, True, False, 0.9, 0.4, 0.0, 0.020, 10**6) == 1714
    assert P.get_chunk_size(m, 0, 10**9, True, False, -3.0, 0.4, 0.0, 0.020, 10**6) == 2857
    # a second long prefill is refused; an exhausted budget gives 0; the request's end caps it
    assert P.get_chunk_size(m, 0, 10**9, True, True, 0.0, 0.4, 0.0, 0.020, 10**6) == 0
    assert P.get_chunk_size(m, 0, 10**9, False, True, 0.0, 0.4, 0.0, 0.020, 10**6) == 2857
    assert P.get_chunk_size(m, 0, 10**9, False, False, 0.0, 0.4, 0.020, 0.020, 10**6) == 0
    assert P.get_chunk_size(m, 0, 37, False, False, 0.0, 0.4, 0.0, 0.020, 10**6) == 37


@pytest.mark.parametrize("kv", [0, 1000, 10**6])
def test_max_chunk_closed_form_for_the_attention_term(kv):
    """t_pair * (c*kv + c(c+1)/2) <= T  <=>  c <= (-(2kv+1) + sqrt((2kv+1)^2 + 8T/t_pair)) / 2."""
    tp, T = 2e-12, 0.004
    m = P.TimeModel(t_pair=tp)
    want = int(math.floor((-(2 * kv + 1) + math.sqrt((2 * kv + 1) ** 2 + 8 * T / tp)) / 2))
    got = P.max_chunk_within(m, kv, T, 10**6)
    assert got == want
    assert P.chunk_time(m, kv, got) <= T < P.chunk_time(m, kv, got + 1)


def test_chunks_shrink_as_the_cache_grows_and_iteration_time_stays_within_target():
    """Section 3.2: with a fixed iteration budget, early chunks are large and late ones small."""
    m = P.TimeModel(t_fixed=1e-3, t_token=2e-6, t_pair=1e-11)
    sizes = [P.max_chunk_within(m, kv, 0.020 - m.t_fixed, 8192) for kv in (0, 10**5, 10**6, 4 * 10**6)]
    assert sizes == sorted(sizes, reverse=True) and sizes[0] > 4 * sizes[-1] > 0
    for kv, c in zip((0, 10**5, 10**6, 4 * 10**6), sizes):
        assert m.t_fixed + P.chunk_time(m, kv, c) <= 0.020


def test_simulated_prefill_time_closed_forms():
    """Per-token model: L tokens in ceil(L / c*) iterations, total = L*t_token + iterations*t_fixed.
    Pair-only model with a generous target: every chunk is max_chunk and the pair counts of the
    chunks add up to the full causal triangle L(L+1)/2, whatever the chunking."""
    m = P.TimeModel(t_fixed=1e-3, t_token=1.1e-5)
    cstar = math.floor((0.020 - 1e-3) / 1.1e-5)
    assert cstar == 1727
    for L in (1, cstar, cstar + 1, 10 * cstar + 7):
        want = L * 1.1e-5 + math.ceil(L / cstar) * 1e-3
        assert abs(P.simulate_prefill(m, L, 0.020, 10**6) - want) < 1e-12
    m = P.TimeModel(t_pair=1e-12)
    for L, mc in ((1000, 64), (1000, 1000), (777, 100)):
        assert abs(P.simulate_prefill(m, L, 1.0, mc) - 1e-12 * L * (L + 1) / 2) < 1e-15
    # nothing fits: the estimate stops where it is (Algorithm 3's early exit)
    assert P.simulate_prefill(P.TimeModel(t_fixed=0.03, t_token=1e-5), 100, 0.020, 64) == 0.0


def test_prefill_cache_and_remaining_time():
    m = P.TimeModel(t_fixed=1e-3, t_token=2e-6, t_pair=1e-11)
    cache = P.build_prefill_cache(m, 20000, 1000, 0.020, 4096)
    assert len(cache) == 21 and cache[0] == 0.0
    assert all(b > a for a, b in zip(cache, cache[1:]))
    assert cache[7] == P.simulate_prefill(m, 7000, 0.020, 4096)
    assert P.remaining_time(cache, 1000, 20000, 0) == cache[-1]
    assert P.remaining_time(cache, 1000, 20000, 20000) == 0.0
    mid = P.lookup(cache, 1000, 7500)
    assert abs(mid - (cache[7] + cache[8]) / 2) < 1e-15
    assert abs(P.remaining_time(cache, 1000, 12000, 7500) - (cache[12] - mid)) < 1e-15


def test_three_request_scenario_of_the_paper():
    """Section 4: r_L (work 10 s, deadline 16 s, arrives at 0) and two shorts (work 0.5 s,
    deadline 1 s, arrive at 5).  Printed: rho_L = 0.6 and rho_S = 1.0 at arrival; FCFS runs
    r_L from 0 to 10 and the shorts miss their deadline at 6; EDF lets the shorts preempt at 5."""
    g = _golden()
    arrival, work, deadline = [0.0, 5.0, 5.0], [10.0, 0.5, 0.5], [16.0, 1.0, 1.0]
    assert abs(P.relative_slack(0, 16, 0, 10, 10) - g["lars_rho_long"]) < 1e-12
    assert abs(P.relative_slack(5, 1, 5, 0.5, 0.5) - g["lars_rho_short"]) < 1e-12
    # a running request keeps its slack; a waiting one loses it second for second
    assert abs(P.relative_slack(0, 16, 5, 5, 10) - 0.6) < 1e-12
    assert abs(P.relative_slack(5, 1, 5.2, 0.5, 0.5) - 0.6) < 1e-9
    f, _ = P.simulate_schedule("fcfs", arrival, work, deadline, 0.01)
    assert abs(f[0] - 10.0) < 1e-6 and abs(f[1] - 10.5) < 1e-6 and abs(f[2] - 11.0) < 1e-6
    assert f[1] > 6 and f[2] > 6                       # the convoy: both shorts miss
    f, st = P.simulate_schedule("edf", arrival, work, deadline, 0.01)
    assert abs(st[1] - 5.0) < 1e-9
    assert abs(f[1] - 5.5) < 1e-6 and abs(f[2] - 6.0) < 1e-6 and abs(f[0] - 11.0) < 1e-6
    # LARS: the shorts wait until their relative slack has fallen to the long request's 0.6,
    # i.e. until t = 5.2 (closed form above); from then on they hold the lower relative slack
    # (a waiting request loses slack, the running one keeps it, so the two alternate) until
    # their 1.0 s of work is done at 6.2; the long request still meets its 16 s
    f, st = P.simulate_schedule("lars", arrival, work, deadline, 0.01)
    assert abs(st[1] - 5.2) < 0.011 and abs(st[2] - 5.2) < 0.025
    assert abs(max(f[1], f[2]) - 6.2) < 0.011
    assert abs(f[0] - 11.0) < 1e-6 and f[0] <= 16.0    # total work is conserved
