"""Algorithm 2's partition search on the GPU against the oracle (needs an MI355X)."""
import json
import os

import numpy as np
import pytest

import gbmw_inputs as gi
import pins
import pins_partition as pp
from gpu_util import check_partition_search, pack_models

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2307_02031_amd as g
    return g


def _search(g, models, max_iter=64, flags=0, ctx=None):
    a = pack_models(models)
    return g.gbmw_partition_search(a["P"], a["Lm"], a["m"], a["c"], a["c_nosync"], a["R"], a["M"], a["p0"],
                                   a["p_t"], a["S"], a["E"], max_iter=max_iter, flags=flags, ctx=ctx,
                                   O_b=a["O_b"], O_ms=a["O_ms"])


def test_worked_example(g):
    """The hand-worked cases, straight against the fixture's numbers."""
    with open(os.path.join(pins.GOLDEN, "worked_example_partition.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        model, m = pp.fixture_model(gold, case)
        P, Lm = model["M"].shape[0], model["c"].shape[0]
        res, ctx = g.gbmw_partition_search([P], [Lm], [m], model["c"], model["c_ns"], model["R"],
                                           model["M"].reshape(P * Lm, -1), case["p0"], case["p_t"],
                                           model["c"].shape[1], case["E"], max_iter=16,
                                           O_b=model["Ob"].reshape(P * Lm, -1) if "Ob" in model else None,
                                           O_ms=model["Oms"].reshape(P * Lm, -1) if "Ob" in model else None)
        n = int(res["n_iter"][0])
        got = dict(O_t=int(res["O_t"][0]), strat=res["strat"][0],
                   trace=[dict(p=list(res["p"][0, j]), cost=res["cost"][0, j], C=res["C"][0, j],
                               Cns=res["Cns"][0, j], O=res["O"][0, j], alpha_t=res["alpha_t"][0, j],
                               alpha_m=res["alpha_m"][0, j]) for j in range(n)])
        pp.check_trace_against(case, got)
        g.gbmw_destroy(ctx)


@pytest.mark.parametrize("flags", [0, 8, 16, 24], ids=["changed-stages", "resolve-all", "lazy-argmin", "lazy-resolve-all"])
def test_uniform_models(g, flags):
    """Closed-form models (S = 1): neighbour choice, ties, the searched-before
    rule, memory limits, an infeasible start, single-stage and one-layer-per-stage
    pairs -- all in one lockstep call."""
    models = [gi.uniform_pipeline_model(Lm, 2, 1000, [1, Lm - 1], m=3) for Lm in (6, 7, 10, 11)]
    models += [gi.uniform_pipeline_model(10, 3, 1000, p0) for p0 in ([2, 6, 2], [7, 2, 1], [4, 2, 4])]
    models += [gi.uniform_pipeline_model(5, 1, 1000, [5]), gi.uniform_pipeline_model(3, 3, 1000, [1, 1, 1])]
    res, ctx = _search(g, models, flags=flags)
    check_partition_search(res, models, 64)
    assert [list(x) for x in res["p"][4, :4]] == [[2, 6, 2], [3, 5, 2], [3, 4, 3], [4, 3, 3]]
    for p_t in (None, [2, 8], [5, 5]):
        lim = [gi.uniform_pipeline_model(10, 2, 9, p0, mem=[3, 1], p_t=p_t) for p0 in ([1, 9], [4, 6])]
        res, ctx = _search(g, lim, flags=flags, ctx=ctx)
        check_partition_search(res, lim, 64)
    res, ctx = _search(g, models, max_iter=2, flags=flags, ctx=ctx)
    check_partition_search(res, models, 2)
    assert res["n_iter"].max() == 2
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("flags", [0, 8, 16], ids=["changed-stages", "resolve-all", "lazy-argmin"])
@pytest.mark.parametrize("S,E,with_pt", [(3, 60, True), (5, 90, False), (22, 400, True), (44, 700, True),
                                         (70, 500, False)])
def test_random_models(g, S, E, with_pt, flags):
    """Pairs of different depth and PP degree searched in lockstep."""
    st = gi.Stream(8100 + S)
    models = []
    for k in range(9):
        P = int(st.integers(1, 1, 6)[0])
        Lm = int(st.integers(1, P, P + 14)[0])
        models.append(gi.random_pipeline_model(9000 + 31 * S + k, Lm, S, P, E, m=int(st.integers(1, 1, 9)[0]),
                                               M_rng=(1, max(2, E // 24)), R_rng=(0.0, 0.5), with_pt=with_pt,
                                               skew=(k % 2 == 0)))
    res, ctx = _search(g, models, max_iter=24, flags=flags)
    check_partition_search(res, models, 24)
    assert res["n_iter"].max() > 2, "the models must exercise the adjustment"
    assert res["stage_solves"] >= sum(m.P for m in models)
    g.gbmw_destroy(ctx)


def test_kept_tables_are_extended_not_recomputed(g):
    """Layer steps actually executed (cell_updates / ((E+1) S^2)) on closed-form traces:
    a stage that gains a layer at its end costs one step, a stage that loses its last
    layer costs none, a stage whose first layer changes is solved again."""
    two = gi.uniform_pipeline_model(10, 2, 1000, [1, 9])
    res, ctx = _search(g, [two])
    assert [list(x) for x in res["p"][0, :5]] == [[1, 9], [2, 8], [3, 7], [4, 6], [5, 5]]
    # [1,9]: 0+8; then each round: 1 step for stage 0 plus all of stage 1: 7, 6, 5, 4
    assert res["cell_updates"] == (8 + 8 + 7 + 6 + 5) * 1001 and res["stage_solves"] == 2 * 5
    res, ctx = _search(g, [two], flags=g.GBMW_FLAG_RESOLVE_ALL, ctx=ctx)
    assert res["cell_updates"] == 5 * 8 * 1001
    # without argmin records every layer's table is kept, so a stage may lose its last layer
    # any number of times in a row for free: [2,2,8] -> [2,3,7] -> ... costs 7 + (1 + 6) + (1 + 5) + ...
    res, ctx = _search(g, [two], flags=g.GBMW_FLAG_LAZY_ARGMIN, ctx=ctx)
    assert res["cell_updates"] == (8 + 8 + 7 + 6 + 5) * 1001
    three = gi.uniform_pipeline_model(10, 3, 1000, [2, 6, 2])
    res, ctx = _search(g, [three], ctx=ctx)
    assert [list(x) for x in res["p"][0, :4]] == [[2, 6, 2], [3, 5, 2], [3, 4, 3], [4, 3, 3]]
    # [2,6,2]: 1+5+1; -> [3,5,2]: stage 0 one step, stage 1 again (4); -> [3,4,3]: stage 1 lost its
    # last layer (0), stage 2 again (2); -> [4,3,3]: stage 0 one step, stage 1 again (2)
    assert res["cell_updates"] == (7 + 5 + 2 + 3) * 1001
    # with a time-balanced partition searched first: 10 - 3 more steps; its largest stage
    # memory (4) then rejects [3,5,2] by limit 3, so the trace ends after [2,6,2]
    three.p_t = np.array([4, 3, 3], np.int32)
    res, ctx = _search(g, [three], ctx=ctx)
    check_partition_search(res, [three], 64)
    assert res["cell_updates"] == (7 + 7) * 1001 and res["n_iter"][0] == 1
    g.gbmw_destroy(ctx)


def test_large_launch_extends_tables_that_small_launches_produced(g):
    """Eight pairs whose long first stage (10 layers) takes one more layer at its end after the
    first search.  In the first round the deep layers of those stages run in small launches
    (four stages per stream group: the shape in which the waves of a workgroup share a tile);
    the extension runs as ONE launch over all eight (the shape with the shortcut for runs of
    equal columns), which decides from the summaries the small launches left.  Traces against
    the oracle, with and without records, and the count of executed layer steps."""
    E = 32768
    models = []
    for k in (0, 2, 4, 5, 6, 7, 8, 9):
        mod = gi.random_pipeline_model(900 + k, 13, 5, 2, E=E, m=4, M_rng=(200, 2400), R_rng=(0.0, 0.5),
                                       with_pt=False)
        mod.c[11:] *= 8.0; mod.c_ns[11:] *= 8.0          # the last two layers make stage 1 the slowest
        mod.p0 = np.array([10, 3], np.int32)
        models.append(mod)
    ctx = None
    for flags in (0, g.GBMW_FLAG_LAZY_ARGMIN):
        res, ctx = _search(g, models, max_iter=6, flags=flags, ctx=ctx)
        check_partition_search(res, models, 6)
        assert all(list(res["p"][k, 1, :2]) == [11, 2] for k in range(8))
        # first round 8 x (9 + 2) steps; second 8 x (1 + 1); the last pair goes on to [12, 1]: 1 + 0
        assert res["cell_updates"] == (88 + 16 + 1) * (E + 1) * 25, res["cell_updates"]
    g.gbmw_destroy(ctx)


def test_changed_stage_reuse_solves_less_and_agrees(g):
    models = [gi.random_pipeline_model(9500 + k, 24, 22, 4, 600, M_rng=(1, 40)) for k in range(6)]
    a, ctx = _search(g, models, max_iter=32)
    b, ctx = _search(g, models, max_iter=32, flags=g.GBMW_FLAG_RESOLVE_ALL, ctx=ctx)
    for key in ("n_iter", "O_t", "p", "cost", "C", "Cns", "O", "alpha_t", "alpha_m", "strat"):
        assert np.array_equal(a[key].view(np.uint8), b[key].view(np.uint8)), key
    assert a["rounds"] == b["rounds"] and a["n_iter"].max() > 2
    assert a["stage_solves"] < b["stage_solves"] and a["cell_updates"] < b["cell_updates"]
    # the context goes on to serve an ordinary solve
    p = gi.make_config(1)
    ctx = g.gbmw_dp_solve_batched(p.L, p.c, p.M, p.R, p.S, p.E, ctx=ctx)
    best, _ = g.gbmw_get_best(ctx)
    assert np.isfinite(best[0, -1])
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("flags", [0, 16], ids=["records", "lazy-argmin"])
def test_structured_models(g, flags):
    """Paper-shaped pairs: 44 strategies, 24-32 layers, PP degrees 2, 4 and 8."""
    models = [gi.structured_pipeline_model(70 + k, Lm, P, 3072, m=8)
              for k, (Lm, P) in enumerate([(24, 2), (24, 4), (32, 4), (32, 8)])]
    res, ctx = _search(g, models, max_iter=12, flags=flags)
    check_partition_search(res, models, 12)
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("flags", [0, 8, 16], ids=["changed-stages", "resolve-all", "lazy-argmin"])
def test_alg3_stage_searches(g, flags):
    """Stage searches with the overall-memory check (Appendix A, Algorithm 3) inside the
    partition loop: random and structured models with O_b / O_ms tables, among them
    O_b = 0 (every budget valid), a window wider than a wave, b_up above E (the walk
    starts at budget 0) and budgets so tight that some searches are infeasible."""
    models = []
    special = [(8, 2, 6, 1), (12, 3, 20, 2), (16, 4, 150, 3), (9, 1, 40, 4), (10, 5, 3, 1), (14, 2, 700, 2),
               (12, 4, 0, 3), (20, 3, 90, 5)]
    for seed, (Lm, P, ob_max, f) in enumerate(special):
        base = gi.random_pipeline_model(300 + seed, Lm, 5, P, E=260, m=4, R_rng=(0.0, 0.5), skew=bool(seed % 2))
        models.append(gi.with_memory_split(base, 400 + seed, ob_max=ob_max))
        models[-1].M *= f; models[-1].Oms *= f          # one E per call: tighter budgets by larger memories
    for seed in (4, 12, 16, 18, 33, 53):                 # several accepted moves each
        st = gi.Stream(9000 + seed)
        P = int(st.integers(1, 2, 5)[0]); Lm = int(st.integers(1, 3 * P, 5 * P)[0])
        ob_max = int(st.integers(1, 2, 60)[0]); f = int(st.integers(1, 1, 3)[0])
        base = gi.random_pipeline_model(300 + seed, Lm, 5, P, E=260, m=4, R_rng=(0.0, 0.5), skew=True)
        models.append(gi.with_memory_split(base, 400 + seed, ob_max=ob_max))
        models[-1].M *= f; models[-1].Oms *= f
    res, ctx = _search(g, models, flags=flags)
    check_partition_search(res, models, 64)
    assert (res["n_iter"] > 2).sum() >= 6
    # the check changes results: the same models searched without it differ somewhere
    plain = [gi.PipelineModel(m.S, m.E, m.P, m.m, m.c, m.c_ns, m.R, m.M, m.p0, m.p_t, m.name) for m in models]
    res0, ctx = _search(g, plain, flags=flags, ctx=ctx)
    assert any(int(res0["n_iter"][k]) != int(res["n_iter"][k]) or
               not np.array_equal(res0["C"][k, 0], res["C"][k, 0]) for k in range(len(models)))
    # structured models at the benchmark's S
    big = [gi.with_memory_split(gi.structured_pipeline_model(70 + k, 24, P, 1200, S=44, act_scale=0.25), 500 + k,
                                ob_max=ob) for k, (P, ob) in enumerate([(2, 100), (4, 300), (8, 30)])]
    res, ctx = _search(g, big, max_iter=12, flags=flags, ctx=ctx)
    check_partition_search(res, big, 12)
    g.gbmw_destroy(ctx)


def test_outer_loops_throughput(g):
    """Algorithm 2 end to end for three batch sizes x PP degrees 2 and 4: the pairs' values,
    the best degree per batch size, the stop at the first batch size that fits nowhere, Tpt."""
    import oracle.bmw as bmw
    models, batch, group = [], [], []
    for gi_, (B, act) in enumerate([(16.0, 0.5), (32.0, 1.0), (64.0, 40.0), (128.0, 1.5)]):
        for P in (2, 4):
            models.append(gi.structured_pipeline_model(300 + gi_, 16, P, 3000, m=4, act_scale=act, S=22))
            batch.append(B); group.append(gi_)
    a = pack_models(models)
    res, ctx = g.gbmw_partition_search(a["P"], a["Lm"], a["m"], a["c"], a["c_nosync"], a["R"], a["M"], a["p0"],
                                       a["p_t"], a["S"], a["E"], max_iter=8, batch_size=batch, batch_group=group)
    check_partition_search(res, models, 8)
    last = [res["cost"][k, res["n_iter"][k] - 1] for k in range(len(models))]
    want, want_g = bmw.throughput([16.0, 32.0, 64.0, 128.0], [last[0:2], last[2:4], last[4:6], last[6:8]])
    assert pins.bits(res["tpt"]) == pins.bits(want) and res["tpt_group"] == want_g
    assert np.isinf(last[4]) and np.isinf(last[5]), "the third batch size must be out of memory"
    assert np.isfinite(last[6]) or np.isfinite(last[7]), "... although the fourth would fit"
    assert want_g in (0, 1) and res["tpt_pair"] == 2 * want_g + int(np.argmin(last[2 * want_g:2 * want_g + 2]))
    g.gbmw_destroy(ctx)


def test_benchmark_workload_all_modes_agree(g):
    """The workload bench.py times (16 pairs, 48 layers, S = 44, E = 32768): kept tables,
    every stage re-solved, no argmin records, and dense arithmetic (no shortcut for waves whose
    budgets share one input column) give the same traces bit for bit, with and without
    O_b / O_ms tables; the
    first pair is also checked against the oracle."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(pins.GOLDEN), "..", "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    models = bench.partition_workload(gi)
    ref, ctx = _search(g, models, max_iter=32)
    for flags in (g.GBMW_FLAG_RESOLVE_ALL, g.GBMW_FLAG_LAZY_ARGMIN, g.GBMW_FLAG_DENSE_ARITHMETIC,
                  g.GBMW_FLAG_DENSE_ARITHMETIC | g.GBMW_FLAG_LAZY_ARGMIN):
        res, ctx = _search(g, models, max_iter=32, flags=flags, ctx=ctx)
        for key in ("n_iter", "O_t", "p", "cost", "C", "Cns", "O", "alpha_t", "alpha_m", "strat"):
            assert np.array_equal(ref[key].view(np.uint8), res[key].view(np.uint8)), (flags, key)
    first = {k: (v[:1] if isinstance(v, np.ndarray) else v) for k, v in ref.items()}
    check_partition_search(first, models[:1], 32)
    # the same pairs with O_b / O_ms tables (every stage search with Appendix A's check)
    split = [gi.with_memory_split(m, 900 + k) for k, m in enumerate(models)]
    ref, ctx = _search(g, split, max_iter=32, ctx=ctx)
    for flags in (g.GBMW_FLAG_RESOLVE_ALL, g.GBMW_FLAG_LAZY_ARGMIN, g.GBMW_FLAG_DENSE_ARITHMETIC):
        res, ctx = _search(g, split, max_iter=32, flags=flags, ctx=ctx)
        for key in ("n_iter", "O_t", "p", "cost", "C", "Cns", "O", "alpha_t", "alpha_m", "strat"):
            assert np.array_equal(ref[key].view(np.uint8), res[key].view(np.uint8)), (flags, key)
    g.gbmw_destroy(ctx)
    last = {k: (v[-1:] if isinstance(v, np.ndarray) else v) for k, v in ref.items()}
    check_partition_search(last, split[-1:], 32)             # P = 16: sixteen short stages
