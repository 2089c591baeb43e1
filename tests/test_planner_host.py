"""The library's task-fusion planner (host code, include/mux_plan.h) against the planner oracle: latencies of Eq. 3
and Eq. 4 to rounding, the fusion of Eq. 6 by its minimum and by the validity and cost of the plan it returns (equal
minima may be reached by different cuts)."""
import json
import os
import random

import pytest

from oracle import planner as opl
from tests.test_oracle_planner import GOLDEN, load_model, random_model


@pytest.fixture(scope="module")
def mx():
    import paper_2603_02885_amd as m
    if not os.path.exists(m.library_path()):
        from paper_2603_02885_amd.build import build_library
        build_library()
    m.load_library()
    return m


def to_lib(mx, model):
    return mx.CostModel(model["stages"], model["C"])


def test_hand_example(mx):
    g = json.load(open(GOLDEN))
    model = load_model(g["model"])
    cm = to_lib(mx, model)
    for c in g["stage_latency"]:
        assert mx.mux_plan_stage_latency(cm, c["stage"], c["tokens"]) == pytest.approx(c["value"], rel=1e-12)
    for c in g["htask_latency"]:
        assert mx.mux_plan_htask_latency(cm, c["tokens"]) == pytest.approx(c["value"], rel=1e-12)
    f = g["fusion"]
    lat, order, begins = mx.mux_plan_fusion(cm, f["tokens"])
    assert lat == pytest.approx(f["value"], rel=1e-12) and order == f["order"] and begins == f["begins"]


@pytest.mark.parametrize("seed", range(6))
def test_random_models_against_oracle(mx, seed):
    rng = random.Random(9000 + seed)
    for case in range(40):
        model = random_model(rng)
        cm = to_lib(mx, model)
        M = rng.randint(1, 10) if case % 8 else rng.randint(30, 60)          # some cases beyond enumeration
        tk = [rng.randint(1, 6000) for _ in range(M)]
        if case % 5 == 0:
            tk[rng.randrange(M)] = tk[0]                                      # equal token counts
        cap = rng.choice([0, 0, 1, 2, 5])
        for s in range(len(model["stages"])):
            sub = tk[:rng.randint(1, M)]
            assert mx.mux_plan_stage_latency(cm, s, sub) == pytest.approx(opl.stage_latency(model, s, sub), rel=1e-12)
        assert mx.mux_plan_htask_latency(cm, tk) == pytest.approx(opl.htask_latency(model, tk), rel=1e-12)
        lat, order, begins = mx.mux_plan_fusion(cm, tk, cap)
        ref, oorder, _ = opl.fusion_dp(model, tk, cap) if M > 10 else opl.fusion_bruteforce(model, tk, cap)
        assert order == oorder                                                # unique: stable ascending order
        assert lat == pytest.approx(ref, rel=1e-12)
        assert begins[0] == 0 and begins[-1] == M and all(a < b for a, b in zip(begins, begins[1:]))
        assert cap == 0 or len(begins) - 1 <= cap
        assert opl.plan_cost(model, [tk[i] for i in order], begins) == pytest.approx(ref, rel=1e-12)


def test_argument_checks(mx):
    model = {"C": 2, "stages": [{"n_gpus": 1, "baseops": [([100, 200], [1.0, 2.0])], "adapters": []}]}
    cm = to_lib(mx, model)
    with pytest.raises(mx.MuxError):
        mx.mux_plan_fusion(cm, [])                                            # no tasks
    with pytest.raises(mx.MuxError):
        mx.mux_plan_fusion(cm, [10, 0])                                       # a task without tokens
    with pytest.raises(mx.MuxError):
        mx.mux_plan_stage_latency(cm, 1, [10])                                # no such stage
    with pytest.raises(mx.MuxError):
        mx.mux_plan_fusion(cm, [10, 20], -1)
    bad = {"C": 2, "stages": [{"n_gpus": 1, "baseops": [([200, 100], [1.0, 2.0])], "adapters": []}]}
    with pytest.raises(mx.MuxError):
        mx.mux_plan_htask_latency(to_lib(mx, bad), [10])                      # token counts not increasing
    with pytest.raises(mx.MuxError):
        mx.mux_plan_htask_latency(mx.CostModel(model["stages"], 0), [10])     # no micro-batch
