"""TEST INFRASTRUCTURE -- oracle of the task-fusion planner (section 3.3): the cost model of a hybrid
task (Eq. 3: latency of one stage, Eq. 4: end-to-end latency in a pipeline of S stages with C
micro-batches) and the choice of the hybrid tasks (Eq. 6).  Pure Python, double precision, written
from the definitions; nothing here is shared with the library's planner.

A model is a dict
    {"C": micro-batches, "stages": [ {"n_gpus": N_g,
                                      "baseops":  [curve, ...],                 # t_o
                                      "adapters": [(t_a curve, u_a curve), ...]} , ... ]}
and a curve a pair (tokens, values) of equally long lists, tokens strictly increasing: the profile of
one operator, measured at a few token counts (section 5, offline profiling).

Readings (the paper gives no rule for them):
  * between two profiled token counts a curve is linear; below the first it keeps the first value
    (a launch costs what it costs); above the last it continues the last segment (through the origin
    if there is only one sample);
  * u_a in Eq. 3 is the adapter's utilisation at the task's own token count, u_a(n_k);
  * the tasks are taken in ascending order of their token counts, ties in their given order;
  * Eq. 6 prints the last hybrid task as H_(i+1)->k; it is H_(i+1)->m, and i stops at m-1 (a hybrid
    task holds at least one task).
"""
from __future__ import annotations

import itertools
from typing import Dict, List, Sequence, Tuple


def curve_value(curve, x: float) -> float:
    xs, ys = curve
    if len(xs) != len(ys) or len(xs) == 0:
        raise ValueError("bad curve")
    if x <= xs[0]:
        return float(ys[0])
    if len(xs) == 1:
        return float(ys[0]) * (x / xs[0])
    for i in range(1, len(xs)):
        if x <= xs[i]:
            return float(ys[i - 1]) + (float(ys[i]) - float(ys[i - 1])) * ((x - xs[i - 1]) / (xs[i] - xs[i - 1]))
    return float(ys[-2]) + (float(ys[-1]) - float(ys[-2])) * ((x - xs[-2]) / (xs[-1] - xs[-2]))


def stage_latency(model: Dict, s: int, tokens: Sequence[int]) -> float:
    """Eq. 3: the BaseOps see the summed tokens of the hybrid task and are sharded over the stage's GPUs; each fused
    adapter group costs the utilisation-weighted sum of its members' latencies, but at least the slowest member."""
    st = model["stages"][s]
    total = sum(tokens)
    base = 0.0
    for t_o in st["baseops"]:
        base += curve_value(t_o, total) / st["n_gpus"]
    adapters = 0.0
    for t_a, u_a in st["adapters"]:
        weighted = 0.0
        slowest = 0.0
        for n in tokens:
            lat = curve_value(t_a, n)
            weighted += curve_value(u_a, n) * lat
            slowest = max(slowest, lat)
        adapters += max(weighted, slowest)
    return base + adapters


def htask_latency(model: Dict, tokens: Sequence[int]) -> float:
    """Eq. 4: warm-up and drain pass every stage but the last once each way; the steady phase runs C micro-batches,
    forward and backward, at the pace of the slowest stage."""
    per_stage = [stage_latency(model, s, tokens) for s in range(len(model["stages"]))]
    return 2.0 * sum(per_stage[:-1]) + 2.0 * model["C"] * max(per_stage)


def task_order(tokens: Sequence[int]) -> List[int]:
    return sorted(range(len(tokens)), key=lambda i: (tokens[i], i))


def plan_cost(model: Dict, sorted_tokens: Sequence[int], begins: Sequence[int]) -> float:
    """What Eq. 6 minimises, for one given cut of the sorted tasks into consecutive hybrid tasks
    (begins = first task of each hybrid task, then the number of tasks): the first hybrid task counts with its full
    end-to-end latency, every further one with its average per-stage latency."""
    S = len(model["stages"])
    cost = htask_latency(model, sorted_tokens[begins[0]:begins[1]])
    for h in range(1, len(begins) - 1):
        cost += htask_latency(model, sorted_tokens[begins[h]:begins[h + 1]]) / S
    return cost


def fusion_bruteforce(model: Dict, tokens: Sequence[int], max_htasks: int = 0) -> Tuple[float, List[int], List[int]]:
    """Every cut of the sorted tasks into consecutive groups, one by one (2^(M-1) of them)."""
    order = task_order(tokens)
    srt = [tokens[i] for i in order]
    M = len(srt)
    limit = M if max_htasks <= 0 else min(M, max_htasks)
    best = None
    for n_cuts in range(0, limit):
        for cuts in itertools.combinations(range(1, M), n_cuts):
            begins = [0, *cuts, M]
            c = plan_cost(model, srt, begins)
            if best is None or c < best[0]:
                best = (c, begins)
    return best[0], order, best[1]


def fusion_dp(model: Dict, tokens: Sequence[int], max_htasks: int = 0) -> Tuple[float, List[int], List[int]]:
    """Eq. 6: F(m, n) = min over i of F(i, n-1) + L(H_(i+1)->m) / S, F(m, 1) = L(H_1->m), answer min over n of F(M, n)."""
    order = task_order(tokens)
    srt = [tokens[i] for i in order]
    M = len(srt)
    S = len(model["stages"])
    limit = M if max_htasks <= 0 else min(M, max_htasks)
    F = {}
    arg = {}
    for m in range(1, M + 1):
        F[(m, 1)] = htask_latency(model, srt[0:m])
    for n in range(2, limit + 1):
        for m in range(n, M + 1):
            for i in range(n - 1, m):
                c = F[(i, n - 1)] + htask_latency(model, srt[i:m]) / S
                if (m, n) not in F or c < F[(m, n)]:
                    F[(m, n)] = c
                    arg[(m, n)] = i
    best_n = min(range(1, limit + 1), key=lambda n: (F[(M, n)], n))
    begins = [M]
    m, n = M, best_n
    while n > 1:
        m = arg[(m, n)]
        begins.append(m)
        n -= 1
    begins.append(0)
    begins.reverse()
    return F[(M, best_n)], order, begins
