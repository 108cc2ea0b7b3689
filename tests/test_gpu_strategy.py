"""The analytic cost model on the GPU against the oracle, bit for bit, and its
device outputs feeding the table solve directly (needs an MI355X)."""
import json
import os

import numpy as np
import pytest

import gbmw_inputs as gi
import oracle
import oracle.strategy as ost
import pins

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2307_02031_amd as g
    return g


def _layers_as_dicts(layers):
    return [dict(params=float(r[0]), flops=float(r[1]), bnd=float(r[2]), int=float(r[3])) for r in layers]


def _compare(got, ref):
    for k in ("c", "c_nosync", "R"):
        pins.assert_same_f32(np.asarray(got[k]), ref["c_ns" if k == "c_nosync" else k], k)
    for k in ("O_f", "O_b", "O_ms", "M"):
        assert np.array_equal(np.asarray(got[k]), ref[k]), k


def test_worked_example(g):
    with open(os.path.join(pins.GOLDEN, "worked_example_cost_model.json")) as f:
        gold = json.load(f)
    strat = np.zeros(len(gold["cases"]), g.STRATEGY_DTYPE)
    for s, case in enumerate(gold["cases"]):
        strat[s]["n_levels"] = len(case["levels"])
        for i, (k, d) in enumerate(case["levels"]):
            strat[s]["kind"][i], strat[s]["degree"][i] = k, d
        strat[s]["ckpt"] = case["ckpt"]
    ly = gold["layer"]
    layers = np.array([[ly["params"], ly["flops"], ly["bnd"], ly["int"]]] * 2)
    out = g.gbmw_cost_model(layers, strat, gold["hw"], gold["Bm"], 3)
    for s, case in enumerate(gold["cases"]):
        assert float(out["c"][1, s]) == case["c"] and float(out["c_nosync"][0, s]) == case["c_ns"]
        assert [int(out[k][1, s]) for k in ("O_ms", "O_f", "O_b")] == case["units"]
        assert [int(out["M"][i, 0, s]) for i in range(3)] == [case["units"][0] + (3 - i) * case["units"][1] for i in range(3)]
    assert not out["R"][0].any()
    assert [float(out["R"][1, 0, 1]), float(out["R"][1, 0, 2]), float(out["R"][1, 0, 0])] == [0.01171875, 0.015625, 0.0]


@pytest.mark.parametrize("name,group,P,Bm,island", [("BERT-Huge-32", 8, 1, 16.0, 8), ("BERT-Huge-48", 4, 2, 8.0, 4),
                                                     ("ViT-Huge-32", 2, 4, 24.0, 2), ("GPT3-15B", 16, 4, 6.0, 8),
                                                     ("BERT-xHuge", 1, 8, 3.0, 8)])
def test_table1_models_against_the_oracle(g, name, group, P, Bm, island):
    layers = gi.table1_layers(name)
    layers[1::3, 1] *= 1.37                     # some variety between the layers
    layers[2::5, 2] *= 0.61
    hw = dict(gi.default_hardware(unit_mb=3.0), island=island)
    strat = g.gbmw_enumerate_strategies(group)
    ref = ost.cost_model(_layers_as_dicts(layers), ost.enumerate_strategies(group), hw, Bm, P, hw["unit_bytes"])
    _compare(g.gbmw_cost_model(layers, strat, hw, Bm, P), ref)
    dev = g.gbmw_cost_model(layers, strat, hw, Bm, P, device=True)
    _compare({k: v.cpu().numpy() for k, v in dev.items()}, ref)


def test_device_outputs_feed_the_search(g):
    """Shapes -> cost model on the device -> table solve, nothing passing through the
    host; against the oracle's cost model and table solve."""
    import torch
    layers = gi.table1_layers("BERT-Huge-32")[:12]
    hw = gi.default_hardware(unit_mb=16.0)
    strat = g.gbmw_enumerate_strategies(8)
    P, Bm, E = 2, 16.0, 1536                                   # 24 GiB in 16 MiB units
    dev = g.gbmw_cost_model(layers, strat, hw, Bm, P, device=True)
    S = len(strat)
    for i in range(P):
        M = dev["M"][i].contiguous()
        ctx = g.gbmw_dp_solve_batched([len(layers)], dev["c"], M, dev["R"], S, E)
        best, _ = g.gbmw_get_best(ctx)
        ref_in = ost.cost_model(_layers_as_dicts(layers), ost.enumerate_strategies(8), hw, Bm, P, hw["unit_bytes"])
        ref = oracle.solve(ref_in["c"], np.ascontiguousarray(ref_in["M"][i]), ref_in["R"], E, keep_C=False)
        pins.assert_same_f32(best[0], ref.best, f"best, stage position {i}")
        plan, cost, mem = g.gbmw_backtrack(ctx, [0], [E])
        rp, rc, rm = ref.backtrack(E)
        assert np.array_equal(plan[0], rp) and pins.bits(cost[0]) == pins.bits(rc) and mem[0] == rm
        assert np.isfinite(cost[0]), "the budget must admit a plan"
        g.gbmw_destroy(ctx)
    del torch


def test_argument_errors(g):
    layers = gi.table1_layers("ViT-Huge-32")
    strat = g.gbmw_enumerate_strategies(4)
    hw = gi.default_hardware()
    with pytest.raises(g.GbmwError):
        g.gbmw_cost_model(layers, strat, dict(hw, unit_bytes=1e-6), 8.0, 2)      # memories overflow int32
    with pytest.raises(g.GbmwError):
        g.gbmw_cost_model(layers, strat, dict(hw, rate=0.0), 8.0, 2)
    bad = strat.copy(); bad[3]["degree"][0] = 3
    with pytest.raises(g.GbmwError):
        g.gbmw_cost_model(layers, bad, hw, 8.0, 2)
    bad = strat.copy(); bad[-1]["kind"][1] = bad[-1]["kind"][0]
    with pytest.raises(g.GbmwError):
        g.gbmw_cost_model(layers, bad, hw, 8.0, 2)


@pytest.mark.parametrize("overall", [False, True], ids=["forward-memory", "overall-memory"])
@pytest.mark.parametrize("P", [1, 2, 4, 8])
def test_shapes_to_partition_search(g, P, overall):
    """The whole planner path for one (batch size, PP degree) pair of a Table-1 model
    on 8 devices: strategies of the 8/P-device group, cost model, Algorithm 2's
    partition loop -- library against oracle, each on its own cost model output.
    overall: the stage searches check the overall memory (Appendix A) with the cost
    model's O_b and O_ms, the same for every stage a layer may sit in."""
    import oracle.bmw as bmw
    layers = gi.table1_layers("BERT-Huge-32")
    layers[:, 1] *= np.linspace(0.7, 1.4, len(layers))           # deeper layers cost more time
    hw = gi.default_hardware(unit_mb=16.0)
    group, Bm, m, E = 8 // P, 4.0, 8, 384                         # 6 GiB in 16 MiB units: the budget binds
    strat = g.gbmw_enumerate_strategies(group)
    S, Lm = len(strat), len(layers)
    got = g.gbmw_cost_model(layers, strat, hw, Bm, P)
    ref = ost.cost_model(_layers_as_dicts(layers), ost.enumerate_strategies(group), hw, Bm, P, hw["unit_bytes"])
    _compare(got, ref)
    p0 = gi.proportional_partition(Lm, 1.0 / np.arange(P, 0, -1))
    p_t = gi.proportional_partition(Lm, np.ones(P))
    tile = lambda a: np.ascontiguousarray(np.broadcast_to(a, (P, Lm, S)))
    res, ctx = g.gbmw_partition_search([P], [Lm], [m], got["c"], got["c_nosync"], got["R"],
                                       got["M"].reshape(P * Lm, S), p0, p_t, S, E, max_iter=16,
                                       O_b=tile(got["O_b"]).reshape(P * Lm, S) if overall else None,
                                       O_ms=tile(got["O_ms"]).reshape(P * Lm, S) if overall else None)
    model = dict(c=ref["c"], c_ns=ref["c_ns"], R=ref["R"], M=ref["M"])
    if overall:
        model.update(Ob=tile(ref["O_b"]), Oms=tile(ref["O_ms"]))
    want = bmw.partition_search(model, p0, E, m, p_t=p_t, max_iter=16)
    n = len(want["trace"])
    assert int(res["n_iter"][0]) == n and int(res["O_t"][0]) == want["O_t"]
    for j, t in enumerate(want["trace"]):
        assert list(res["p"][0, j, :P]) == t["p"] and pins.bits(res["cost"][0, j]) == pins.bits(t["cost"])
        assert [int(x) for x in res["O"][0, j, :P]] == [int(x) for x in t["O"]]
    assert np.array_equal(res["strat"][0], want["strat"])
    assert np.isfinite(res["cost"][0, n - 1]), "the budget must admit a plan"
    g.gbmw_destroy(ctx)


def test_forbidden_padding_changes_nothing(g):
    """A strategy set padded with forbidden strategies (c = +inf) gives the same trace,
    costs and plan: how pairs with different strategy sets share one call."""
    import oracle.bmw as bmw
    layers = gi.table1_layers("BERT-Huge-32")[:16]
    hw = gi.default_hardware(unit_mb=16.0)
    P, Bm, m, E, Lm = 2, 4.0, 8, 384, 16
    strat = g.gbmw_enumerate_strategies(4)
    n_s, S = len(strat), 22
    cm = g.gbmw_cost_model(layers, strat, hw, Bm, P)
    c = np.full((Lm, S), np.inf, np.float32); c[:, :n_s] = cm["c"]
    cn = np.full((Lm, S), np.inf, np.float32); cn[:, :n_s] = cm["c_nosync"]
    R = np.zeros((Lm, S, S), np.float32); R[:, :n_s, :n_s] = cm["R"]
    M = np.zeros((P, Lm, S), np.int32); M[:, :, :n_s] = cm["M"]
    p0, p_t = np.array([5, 11], np.int32), np.array([8, 8], np.int32)
    a, ctx = g.gbmw_partition_search([P], [Lm], [m], cm["c"], cm["c_nosync"], cm["R"], cm["M"].reshape(P * Lm, n_s),
                                     p0, p_t, n_s, E, max_iter=16)
    b, ctx = g.gbmw_partition_search([P], [Lm], [m], c, cn, R, M.reshape(P * Lm, S), p0, p_t, S, E, max_iter=16,
                                     ctx=ctx)
    for key in ("n_iter", "O_t", "p", "cost", "C", "Cns", "O", "alpha_t", "alpha_m", "strat"):
        assert np.array_equal(a[key].view(np.uint8), b[key].view(np.uint8)), key
    assert a["n_iter"][0] > 1 and np.isfinite(a["cost"][0, a["n_iter"][0] - 1])
    want = bmw.partition_search(dict(c=c, c_ns=cn, R=R, M=M), p0, E, m, p_t=p_t, max_iter=16)
    assert int(b["n_iter"][0]) == len(want["trace"])
    assert pins.bits(b["cost"][0, len(want["trace"]) - 1]) == pins.bits(want["trace"][-1]["cost"])
    assert np.array_equal(b["strat"][0], want["strat"])
    g.gbmw_destroy(ctx)
