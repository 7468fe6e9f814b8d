"""Plain statements of the paper's chunk-size policy, prefill-time estimation and the
relative-slack scheduling example (TEST INFRASTRUCTURE ONLY, like the rest of this package).

Everything here is the paper's procedure written out with the simplest possible search
(linear scans where the paper says "binary search": the result is defined as the LARGEST
chunk that fits, however it is found), in Python floats and ints.

Passages followed: appendix "Adaptive Chunk Size Selection" (Algorithm 2), appendix
"Prefill Time Estimation" (Algorithm 3), section 4 "Length-Aware Relative Slack" and its
three-request scenario, section 4.3 "Space Sharing" (the 20 % slack -> 16 ms of 20 ms example).

Runtime model (the paper uses an external simulator; this build fits its own to measured
kernel times): the predicted time of one prefill chunk of c tokens on a cache of kv tokens is
    t_token * c + t_pair * (c * kv + c * (c + 1) / 2)
(linear layers per token; attention per visible (query, key) pair, exact causal count) and
an iteration adds t_fixed once, t_decode per decode request and t_decode_key per cached key
of the decodes.
"""
from dataclasses import dataclass


@dataclass
class TimeModel:
    t_fixed: float = 0.0
    t_token: float = 0.0
    t_pair: float = 0.0
    t_decode: float = 0.0
    t_decode_key: float = 0.0


def chunk_time(m: TimeModel, kv_size: int, chunk: int) -> float:
    return m.t_token * chunk + m.t_pair * (chunk * kv_size + chunk * (chunk + 1) / 2)


def max_chunk_within(m: TimeModel, kv_size: int, t_budget: float, max_chunk: int) -> int:
    """Largest c in [0, max_chunk] whose predicted time is within the budget."""
    best = 0
    for c in range(1, max_chunk + 1):
        if chunk_time(m, kv_size, c) <= t_budget:
            best = c
        else:
            break       # the time grows with c
    return best


def get_chunk_size(m: TimeModel, kv_size: int, remaining: int, is_long: bool,
                   batch_has_long: bool, rel_slack: float, rho_max: float, t_current: float,
                   t_target: float, max_chunk: int) -> int:
    """Algorithm 2: no second long prefill in a batch; a request with relative slack rho
    yields the fraction min(rho_max, max(0, rho)) of the target; the chunk is the largest
    that fits what is left of the effective budget (and of the request)."""
    if is_long and batch_has_long:
        return 0
    rho = min(rho_max, max(0.0, rel_slack))
    t_effective = t_target * (1.0 - rho)
    t_budget = t_effective - t_current
    if t_budget <= 0:
        return 0
    return max_chunk_within(m, kv_size, t_budget, min(max_chunk, remaining))


def simulate_prefill(m: TimeModel, length: int, t_target: float, max_chunk: int) -> float:
    """Algorithm 3, SimulatePrefill: chunk after chunk, each the largest whose iteration
    (t_fixed + chunk time) stays within t_target; stops early if none fits."""
    t_total, done = 0.0, 0
    while done < length:
        c = max_chunk_within(m, done, t_target - m.t_fixed, min(max_chunk, length - done))
        if c == 0:
            break
        t_total += m.t_fixed + chunk_time(m, done, c)
        done += c
    return t_total


def build_prefill_cache(m: TimeModel, l_max: int, delta: int, t_target: float, max_chunk: int):
    """Algorithm 3, BuildPrefillCache: entry i holds the prefill time of i * delta tokens."""
    return [simulate_prefill(m, i * delta, t_target, max_chunk) for i in range(l_max // delta + 1)]


def lookup(cache, delta: int, length: int) -> float:
    """Reading: lengths between two cache entries are interpolated linearly; lengths past the
    last entry take the last entry."""
    i, r = divmod(length, delta)
    if i >= len(cache) - 1:
        return cache[-1]
    return cache[i] + (cache[i + 1] - cache[i]) * (r / delta)


def remaining_time(cache, delta: int, l_total: int, l_processed: int) -> float:
    return lookup(cache, delta, l_total) - lookup(cache, delta, l_processed)


def relative_slack(arrival: float, deadline: float, now: float, remaining_work: float,
                   total_work: float) -> float:
    """rho = (a + d - t - w(t)) / w_total   (section 4, LARS)."""
    return (arrival + deadline - now - remaining_work) / total_work


def simulate_schedule(policy: str, arrival, work, deadline, quantum: float):
    """One server, decisions every `quantum` seconds (an iteration), requests given by arrival
    time, total work and relative deadline.  'fcfs' runs the earliest arrival to completion;
    'edf' runs the earliest absolute deadline, 'lars' the smallest relative slack, both
    re-decided every quantum (ties: lower index).  Returns (finish times, first-start times)."""
    n = len(arrival)
    left = list(work)
    finish = [None] * n
    start = [None] * n
    t, current = 0.0, None
    steps = 0
    while any(f is None for f in finish):
        ready = [i for i in range(n) if finish[i] is None and arrival[i] <= t + 1e-12]
        if not ready:
            t = min(arrival[i] for i in range(n) if finish[i] is None)
            continue
        if policy == "fcfs":
            if current is None or finish[current] is not None:
                current = min(ready, key=lambda i: (arrival[i], i))
        elif policy == "edf":
            current = min(ready, key=lambda i: (arrival[i] + deadline[i], i))
        elif policy == "lars":
            current = min(ready, key=lambda i: (relative_slack(arrival[i], deadline[i], t,
                                                               left[i], work[i]), i))
        else:
            raise ValueError(policy)
        if start[current] is None:
            start[current] = t
        run = min(quantum, left[current])
        left[current] -= run
        t += run
        if left[current] <= 1e-12:
            finish[current] = t
        steps += 1
        assert steps < 10_000_000
    return finish, start
