"""Pipeline time (Eq. 5 / Eq. 8) in the oracle: hand-worked fixture, a Python
rewrite, special cases.  CPU only."""
import json
import os

import numpy as np

import gbmw_inputs as gi
import oracle
import pins
from test_oracle_pins import solve


def py_pipeline(m, C, Cns):
    total = np.float32(C[0])
    for x in C[1:]:
        total = np.float32(total + np.float32(x))
    mx = max(np.float32(x) for x in Cns)
    if np.isinf(total) or np.isinf(mx):
        return pins.INF
    return np.float32(np.float32(np.float32(m - 1) * mx) + total)


def stage_times(sol, c, c_ns, M, R, e):
    """(C, Cns) of one stage at budget e: the table's best, and the plan
    re-evaluated with the costs without gradient synchronisation."""
    if e < 0 or np.isinf(sol.best[e]):
        return pins.INF, pins.INF
    plan, cost, _ = sol.backtrack(e)
    v, _ = pins.py_plan_cost(c_ns, M, R, [int(x) for x in plan])
    return cost, v


def test_worked_example():
    with open(os.path.join(pins.GOLDEN, "worked_example_pipeline.json")) as f:
        g = json.load(f)
    with open(os.path.join(pins.GOLDEN, g["base"])) as f:
        b = json.load(f)
    c = np.array(b["c"], np.float32); M = np.array(b["M"], np.int32); R = np.array(b["R"], np.float32)
    c_ns = np.array(g["c_nosync"], np.float32)
    sol = solve(c, M, R, b["E"])
    for case in g["cases"]:
        cn = c_ns if case["use_c_nosync"] else c
        C, Cns = zip(*[stage_times(sol, c, cn, M, R, e) for e in case["stage_e"]])
        assert [float(x) for x in C] == [float(pins._val(x)) for x in case["C"]]
        assert [float(x) for x in Cns] == [float(pins._val(x)) for x in case["Cns"]]
        got = oracle.pipeline_cost(case["m"], C, Cns)
        assert float(got) == float(pins._val(case["cost"])) == float(py_pipeline(case["m"], C, Cns))


def test_against_python_rewrite_and_special_cases():
    st = gi.Stream(900)
    for trial in range(200):
        P = int(st.integers(1, 1, 8)[0])
        m = int(st.integers(1, 1, 16)[0])
        C = st.uniform(P, 0.001, 500.0)
        Cns = (C * st.uniform(P, 0.3, 1.0)).astype(np.float32)
        got = oracle.pipeline_cost(m, C, Cns)
        assert pins.bits(got) == pins.bits(py_pipeline(m, C, Cns))
        if m == 1:                               # a single micro-batch: the plain sum of the stages
            assert pins.bits(got) == pins.bits(py_pipeline(1, C, C))
        if P == 1:                               # one stage: m - 1 times the short run plus one full run
            assert pins.bits(got) == pins.bits(np.float32(np.float32(np.float32(m - 1) * Cns[0]) + C[0]))
        assert got >= C.max() and not np.isnan(got)
    assert np.isinf(oracle.pipeline_cost(1, [1.0, np.inf], [1.0, np.inf]))
    assert np.isinf(oracle.pipeline_cost(3, [np.inf], [np.inf]))
