"""Pins of the planner oracle (oracle/planner.py): a hand-worked example of Eq. 3, 4 and 6 of section 3.3,
closed forms, and the recurrence of Eq. 6 against the enumeration of every cut."""
import json
import os
import random

import pytest

from oracle import planner

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "planner_hand_example.json")


def load_model(m):
    return {"C": m["C"], "stages": [{"n_gpus": s["n_gpus"], "baseops": [tuple(c) for c in s["baseops"]],
                                     "adapters": [(tuple(a[0]), tuple(a[1])) for a in s["adapters"]]} for s in m["stages"]]}


def random_curve(rng, kind):
    n = rng.randint(1, 5)
    xs = sorted(rng.sample(range(16, 4096), n))
    if kind == "util":
        return xs, [rng.uniform(0.05, 1.0) for _ in xs]
    base = rng.uniform(0.01, 0.5)
    shape = rng.choice(["flat", "linear", "convex", "concave"])
    f = {"flat": lambda x: 0.0, "linear": lambda x: x / 1000.0, "convex": lambda x: (x / 1000.0) ** 2,
         "concave": lambda x: (x / 1000.0) ** 0.5}[shape]
    return xs, [base + f(x) for x in xs]


def random_model(rng):
    stages = []
    for _ in range(rng.randint(1, 3)):
        stages.append({"n_gpus": rng.choice([1, 1, 2, 4]),
                       "baseops": [random_curve(rng, "lat") for _ in range(rng.randint(1, 3))],
                       "adapters": [(random_curve(rng, "lat"), random_curve(rng, "util")) for _ in range(rng.randint(0, 2))]})
    return {"C": rng.randint(1, 8), "stages": stages}


def check_pins(pl):
    """Every pin, on the module object `pl` (the mutation test runs them on broken copies)."""
    g = json.load(open(GOLDEN))
    model = load_model(g["model"])
    for c in g["stage_latency"]:
        assert pl.stage_latency(model, c["stage"], c["tokens"]) == pytest.approx(c["value"], rel=1e-12), c
    for c in g["htask_latency"]:
        assert pl.htask_latency(model, c["tokens"]) == pytest.approx(c["value"], rel=1e-12), c
    f = g["fusion"]
    for solve in (pl.fusion_dp, pl.fusion_bruteforce):
        value, order, begins = solve(model, f["tokens"])
        assert value == pytest.approx(f["value"], rel=1e-12) and order == f["order"] and begins == f["begins"]
    # curves: the samples themselves, a midpoint, below the first, above the last, a single sample
    cv = ([100, 300, 400], [1.0, 2.0, 4.0])
    assert [pl.curve_value(cv, x) for x in (100, 300, 400)] == [1.0, 2.0, 4.0]
    assert pl.curve_value(cv, 200) == pytest.approx(1.5) and pl.curve_value(cv, 350) == pytest.approx(3.0)
    assert pl.curve_value(cv, 7) == 1.0 and pl.curve_value(cv, 500) == pytest.approx(6.0)
    assert pl.curve_value(([200], [0.5]), 800) == pytest.approx(2.0) and pl.curve_value(([200], [0.5]), 50) == 0.5
    # order: ascending token counts, equal counts in their given order
    assert pl.task_order([5, 3, 9, 3, 1]) == [4, 1, 3, 0, 2]
    # closed forms with one stage and no adapters, tokens inside the profiled range
    toks = [120, 340, 560, 780, 900]
    lin = {"C": 3, "stages": [{"n_gpus": 1, "baseops": [([1, 4000], [0.001, 4.0])], "adapters": []}]}
    v, _, b = pl.fusion_dp(lin, toks)          # latency proportional to tokens: every cut costs 2 C a sum(n)
    assert v == pytest.approx(2 * 3 * 0.001 * sum(toks), rel=1e-12)
    for cut in ([0, 5], [0, 2, 5], [0, 1, 2, 3, 4, 5]):
        assert pl.plan_cost(lin, sorted(toks), cut) == pytest.approx(v, rel=1e-12)
    flat = {"C": 2, "stages": [{"n_gpus": 1, "baseops": [([1, 4000], [0.7, 0.7])], "adapters": []}]}
    v, _, b = pl.fusion_dp(flat, toks)         # launch-bound operator: one hybrid task
    assert b == [0, 5] and v == pytest.approx(2 * 2 * 0.7)
    xs = list(range(0, 4001, 20))
    conv = {"C": 1, "stages": [{"n_gpus": 1, "baseops": [(xs[1:], [(x / 1000.0) ** 2 for x in xs[1:]])], "adapters": []}]}
    v, _, b = pl.fusion_dp(conv, toks)         # strictly convex latency through the origin: every task alone
    assert b == [0, 1, 2, 3, 4, 5] and v == pytest.approx(2 * sum((n / 1000.0) ** 2 for n in toks), rel=1e-9)
    v2, _, b2 = pl.fusion_dp(conv, toks, max_htasks=2)
    assert len(b2) == 3 and v2 > v
    # Eq. 6 against every cut, one by one
    rng = random.Random(1234)
    for case in range(60):
        m = random_model(rng)
        M = rng.randint(1, 9)
        tk = [rng.randint(16, 3000) for _ in range(M)]
        cap = rng.choice([0, 0, 1, 2, 3])
        vd, od, bd = pl.fusion_dp(m, tk, cap)
        vb, ob, bb = pl.fusion_bruteforce(m, tk, cap)
        assert od == ob and vd == pytest.approx(vb, rel=1e-12), (case, vd, vb)
        srt = [tk[i] for i in od]
        assert pl.plan_cost(m, srt, bd) == pytest.approx(vb, rel=1e-12)
        assert bd[0] == 0 and bd[-1] == M and all(x < y for x, y in zip(bd, bd[1:]))
        assert cap == 0 or len(bd) - 1 <= cap


def test_planner_oracle_pins():
    check_pins(planner)


MUTATIONS = [
    ('curve_value(t_o, total) / st["n_gpus"]', 'curve_value(t_o, total)'),                 # sharding forgotten
    ('total = sum(tokens)', 'total = max(tokens)'),                                          # BaseOp sees one task only
    ('adapters += max(weighted, slowest)', 'adapters += weighted'),                          # no bottleneck bound
    ('adapters += max(weighted, slowest)', 'adapters += slowest'),                           # no weighted sum
    ('weighted += curve_value(u_a, n) * lat', 'weighted += lat'),                            # utilisation dropped
    ('2.0 * model["C"] * max(per_stage)', 'model["C"] * max(per_stage)'),                    # one pass instead of two
    ('2.0 * model["C"] * max(per_stage)', '2.0 * model["C"] * sum(per_stage)'),              # sum instead of slowest stage
    ('2.0 * sum(per_stage[:-1])', '2.0 * sum(per_stage)'),                                   # warm-up over all stages
    ('c = F[(i, n - 1)] + htask_latency(model, srt[i:m]) / S', 'c = F[(i, n - 1)] + htask_latency(model, srt[i:m])'),
    ('for i in range(n - 1, m):', 'for i in range(n, m):'),                                  # first split point skipped
    ('c = F[(i, n - 1)] + htask_latency(model, srt[i:m]) / S', 'c = F[(i, n - 1)] + htask_latency(model, srt[i + 1:m]) / S'),
    ('return float(ys[-2]) + (float(ys[-1]) - float(ys[-2])) * ((x - xs[-2]) / (xs[-1] - xs[-2]))', 'return float(ys[-1])'),
    ('key=lambda i: (tokens[i], i))', 'key=lambda i: (-tokens[i], i))'),                     # descending order
]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_planner_pins_catch_planted_mistakes(idx):
    """One mistake at a time in a copy of the oracle's source: the pins must fail."""
    import types
    old, new = MUTATIONS[idx]
    src = open(planner.__file__).read()
    assert src.count(old) == 1, old
    mod = types.ModuleType("planner_mutant")
    exec(compile(src.replace(old, new), "planner_mutant", "exec"), mod.__dict__)
    with pytest.raises((AssertionError, KeyError, IndexError)):
        check_pins(mod)
