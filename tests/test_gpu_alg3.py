"""Algorithm 3's outer loop on the GPU (gbmw_select_forward_budget) against the
oracle, instance by instance (needs an MI355X)."""
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


def _compare(g, ctx, p, Of, Ob, Oms, instances=None, nthreads=16):
    e_opt, cost, plan, e_all = g.gbmw_select_forward_budget(ctx, Of, Ob, Oms)
    for b in (range(p.B) if instances is None else instances):
        o, Lb = int(p.offsets[b]), int(p.L[b])
        ref = oracle.solve_problem(p, b, keep_C=False, keep_A=True, nthreads=nthreads)
        r_e, r_cost, r_plan, r_all = oracle.select_budget(ref, Of[o:o + Lb], Ob[o:o + Lb], Oms[o:o + Lb])
        assert e_opt[b] == r_e, (p.name, b, e_opt[b], r_e)
        assert pins.bits(cost[b]) == pins.bits(r_cost)
        assert np.array_equal(plan[b, :Lb], r_plan) and np.all(plan[b, Lb:] == 255)
        assert e_all[b] == r_all
        if r_all >= 0:
            assert r_all <= p.E
    return e_opt, cost, plan, e_all


def test_worked_example(g):
    with open(os.path.join(pins.GOLDEN, "worked_example_alg3.json")) as f:
        gold = json.load(f)
    with open(os.path.join(pins.GOLDEN, gold["base"])) as f:
        b = json.load(f)
    p = gi.Problem(1, b["S"], b["E"], np.array([b["L"]]), np.array(b["c"], np.float32),
                   np.array(b["M"], np.int32), np.array(b["R"], np.float32), "alg3-golden")
    ctx = solve_gpu(p)
    Of = np.array(gold["Of"], np.int32); Oms = np.array(gold["Oms"], np.int32)
    for case in gold["cases"]:
        e_opt, cost, plan, e_all = g.gbmw_select_forward_budget(ctx, Of, np.array(case["Ob"], np.int32), Oms)
        assert (int(e_opt[0]), float(cost[0]), plan[0].tolist(), int(e_all[0])) == \
               (case["e_opt"], case["cost"], case["plan"], case["e_all"])
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("S,E,Ls,Mhi", [(4, 120, [4, 2, 6, 1], 30), (7, 300, [5, 3], 60), (22, 1000, [6, 9, 3], 200),
                                        (44, 2500, [8, 5], 400), (64, 900, [4, 6], 150), (70, 400, [3, 4], 100),
                                        (3, 10, [4, 3], 12)])
@pytest.mark.parametrize("lazy", [False, True], ids=["records", "lazy-argmin"])
def test_batches_against_the_oracle(g, S, E, Ls, Mhi, lazy):
    parts = [gi.random_instance(2000 + 13 * S + i, L, S, E, M_rng=(1, Mhi)) for i, L in enumerate(Ls)]
    p = gi.stack(parts, f"alg3-S{S}")
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_LAZY_ARGMIN if lazy else 0, device_inputs=True)
    for variant in range(5):
        Of, Ob, Oms = gi.split_memory(p, 3000 + variant)
        if variant == 1:
            Ob[:] = 0                              # no backward peak: e_opt = E when feasible
        if variant == 2:
            Ob[:] = np.minimum(Ob, 5)              # tiny window
        if variant == 3:
            Ob[:] = Ob + E                         # b_up > E: nothing valid a priori
        if variant == 4:
            Ob[:] = np.where(Ob > Mhi // 2, E // 2, 0)
        e_opt, cost, plan, e_all = _compare(g, ctx, p, Of, Ob, Oms)
        if variant == 1:
            best, _ = g.gbmw_get_best(ctx)
            for b in range(p.B):
                if np.isfinite(best[b, E]):
                    assert e_opt[b] == E
    # O_f + O_ms must be the M of the solve
    Of, Ob, Oms = gi.split_memory(p, 1)
    Of[0, 0] += 1
    with pytest.raises(g.GbmwError) as ei:
        g.gbmw_select_forward_budget(ctx, Of, Ob, Oms)
    assert ei.value.status == g.GBMW_ERR_INVALID_ARG
    g.gbmw_destroy(ctx)


def test_config4_full_size(g):
    p = gi.make_config(4)
    ctx = solve_gpu(p, device_inputs=True)
    Of, Ob, Oms = gi.split_memory(p, 4)
    e_opt, cost, plan, e_all = _compare(g, ctx, p, Of, Ob, Oms, instances=range(0, 64, 5))
    # properties for every instance: the chosen plan fits overall, and every budget
    # up to E - b_up would have fitted
    for b in range(p.B):
        o, Lb = int(p.offsets[b]), int(p.L[b])
        b_up = int(Ob[o:o + Lb].max())
        assert e_opt[b] >= min(p.E, max(-1, p.E - b_up))
        if e_all[b] >= 0:
            assert e_all[b] <= p.E
            assert e_all[b] == pins.py_e_all(Of[o:o + Lb], Ob[o:o + Lb], Oms[o:o + Lb], plan[b, :Lb].tolist())
    g.gbmw_destroy(ctx)
