"""Pipeline time (Eq. 5 / Eq. 8) on the GPU against the oracle (needs an MI355X)."""
import json
import os

import numpy as np
import pytest

import gbmw_inputs as gi
import oracle
import pins
from gpu_util import solve_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2307_02031_amd as g
    return g


def _oracle_stage(p, refs, b, e, c_ns):
    if e < 0 or np.isinf(refs[b].best[e]):
        return pins.INF, pins.INF
    o, Lb = int(p.offsets[b]), int(p.L[b])
    plan, cost, _ = refs[b].backtrack(e)
    if c_ns is None:
        return cost, cost
    v, _ = oracle.plan_cost(c_ns[o:o + Lb], p.M[o:o + Lb], p.R[o:o + Lb], plan)
    return cost, v


def test_worked_example(g):
    with open(os.path.join(pins.GOLDEN, "worked_example_pipeline.json")) as f:
        gold = json.load(f)
    with open(os.path.join(pins.GOLDEN, gold["base"])) as f:
        b = json.load(f)
    one = gi.Problem(1, b["S"], b["E"], np.array([b["L"]]), np.array(b["c"], np.float32),
                     np.array(b["M"], np.int32), np.array(b["R"], np.float32))
    p = gi.stack([one, one], "pipeline-golden")
    ctx = solve_gpu(p)
    c_ns = np.tile(np.array(gold["c_nosync"], np.float32), (2, 1))
    for case in gold["cases"]:
        cost, sc, scn = g.gbmw_pipeline_cost(ctx, [0, 2], [0, 1], case["stage_e"], [case["m"]],
                                             c_ns if case["use_c_nosync"] else None)
        assert float(cost[0]) == float(pins._val(case["cost"]))
        assert [float(x) for x in sc] == [float(pins._val(x)) for x in case["C"]]
        assert [float(x) for x in scn] == [float(pins._val(x)) for x in case["Cns"]]
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("S,E,Ls", [(5, 200, [4, 6, 3, 5, 2, 7, 1, 4]), (22, 900, [6, 6, 5, 7]),
                                    (44, 1500, [3, 4, 5, 6, 2, 8]), (70, 300, [3, 4, 2])])
@pytest.mark.parametrize("lazy", [False, True], ids=["records", "lazy-argmin"])
def test_random_pipelines_against_the_oracle(g, S, E, Ls, lazy):
    parts = [gi.random_instance(4000 + 7 * S + i, L, S, E, M_rng=(1, max(2, E // 8))) for i, L in enumerate(Ls)]
    p = gi.stack(parts, f"pipe-S{S}")
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_LAZY_ARGMIN if lazy else 0, device_inputs=True)
    refs = [oracle.solve_problem(p, b, keep_C=False) for b in range(p.B)]
    st = gi.Stream(5000 + S)
    c_ns = (p.c * st.uniform(p.c.size, 0.3, 1.0).reshape(p.c.shape)).astype(np.float32)
    # pipelines: consecutive groups of stages, budgets from feasible, tight and infeasible ranges
    sizes, left = [], p.B
    while left:
        k = min(left, int(st.integers(1, 1, 4)[0]))
        sizes.append(k); left -= k
    begin = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    inst = np.arange(p.B, dtype=np.int32)
    for variant in range(3):
        es = st.integers(p.B, -1 if variant == 2 else E // 2, E).astype(np.int32)
        if variant == 1:
            es[:] = E
        mb = st.integers(len(sizes), 1, 9).astype(np.int32)
        for cn in (c_ns, None):
            cost, sc, scn = g.gbmw_pipeline_cost(ctx, begin, inst, es, mb, cn)
            for q in range(p.B):
                C, Cns = _oracle_stage(p, refs, q, int(es[q]), cn)
                assert pins.bits(sc[q]) == pins.bits(C) and pins.bits(scn[q]) == pins.bits(Cns), (q, es[q])
            for k in range(len(sizes)):
                lo, hi = begin[k], begin[k + 1]
                assert pins.bits(cost[k]) == pins.bits(oracle.pipeline_cost(int(mb[k]), sc[lo:hi], scn[lo:hi]))
    with pytest.raises(g.GbmwError):
        g.gbmw_pipeline_cost(ctx, [0, 0], [], [], [1])
    with pytest.raises(g.GbmwError):
        g.gbmw_pipeline_cost(ctx, [0, 1], [p.B], [0], [1])
    with pytest.raises(g.GbmwError):
        g.gbmw_pipeline_cost(ctx, [0, 1], [0], [0], [0])
    g.gbmw_destroy(ctx)
