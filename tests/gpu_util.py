"""Helpers shared by the GPU parity tests: run the library through its C ABI
(via the thin binding) and compare with the CPU oracle, bit for bit."""
from __future__ import annotations

import numpy as np

import gbmw_inputs as gi
import oracle
import pins


def solve_gpu(p: gi.Problem, flags: int = 0, device_inputs: bool = False, ctx=None):
    import torch
    import paper_2307_02031_amd as g
    if not device_inputs:
        flags |= g.GBMW_FLAG_ONE_STREAM      # host-input cases also cover the one-stream path
    if device_inputs:
        c = torch.from_numpy(p.c).cuda()
        M = torch.from_numpy(p.M).cuda()
        R = torch.from_numpy(p.R).cuda()
    else:
        c, M, R = p.c, p.M, p.R
    ctx = g.gbmw_dp_solve_batched(p.L, c, M, R, p.S, p.E, flags=flags, ctx=ctx)
    g.gbmw_synchronize(ctx)
    return ctx


def check_instance(g, ctx, p: gi.Problem, b: int, full_C: bool, q_es=None, nthreads: int = 16,
                   best=None, best_s=None, with_C: bool = True):
    """Everything the library can return for instance b against the oracle (with_C=False:
    everything but the fp32 tables, so that the oracle need not hold them)."""
    ref = oracle.solve_problem(p, b, keep_C=with_C, keep_A=True, nthreads=nthreads)
    Lb = int(p.L[b])
    if best is None:
        best, best_s = g.gbmw_get_best(ctx)
    pins.assert_same_f32(best[b], ref.best, f"{p.name}[{b}] best")
    assert np.array_equal(best_s[b], ref.best_s), f"{p.name}[{b}] best_s"
    if with_C:
        l0 = 0 if full_C else max(0, Lb - 2)
        C, _ = g.gbmw_export_tables(ctx, b, l0, Lb, want_C=True, want_A=False)
        for l in range(l0, Lb):
            pins.assert_same_f32(C[l - l0], ref.C[l], f"{p.name}[{b}] C layer {l}")
        del C
    _, A = g.gbmw_export_tables(ctx, b, 0, Lb, want_C=False, want_A=True)
    for l in range(Lb):
        if not np.array_equal(A[l], ref.A[l]):
            bad = np.argwhere(A[l] != ref.A[l])
            raise AssertionError(f"{p.name}[{b}] A layer {l}: {len(bad)} cells differ, first (e,s)={bad[0]}: "
                                 f"{A[l][tuple(bad[0])]} vs {ref.A[l][tuple(bad[0])]}")
    del A
    if q_es is None:
        E = p.E
        q_es = sorted(set([0, E, E // 2, E // 3, (2 * E) // 3] + list(range(0, E + 1, max(1, E // 61)))))
    q_es = np.asarray(q_es, np.int32)
    plan, cost, mem = g.gbmw_backtrack(ctx, np.full(len(q_es), b, np.int32), q_es)
    for i, e in enumerate(q_es):
        rp, rc, rm = ref.backtrack(int(e))
        assert np.array_equal(plan[i, :Lb], rp), (p.name, b, e, plan[i, :Lb], rp)
        assert np.all(plan[i, Lb:] == 255)
        assert pins.bits(cost[i]) == pins.bits(rc) and int(mem[i]) == rm
    return ref


def check_plans_by_definition(g, ctx, p: gi.Problem, b: int, q_es, best):
    """Size-independent property: the returned plan, re-evaluated by the plain
    definition of a plan's cost (Eq. 3 unrolled), costs exactly best[e] and
    fits the budget; best is non-increasing in e."""
    o, Lb = int(p.offsets[b]), int(p.L[b])
    q_es = np.asarray(q_es, np.int32)
    plan, cost, mem = g.gbmw_backtrack(ctx, np.full(len(q_es), b, np.int32), q_es)
    assert np.all(best[b][1:] <= best[b][:-1])
    for i, e in enumerate(q_es):
        assert pins.bits(cost[i]) == pins.bits(best[b][e])
        if np.isinf(best[b][e]):
            assert mem[i] == -1 and np.all(plan[i] == 255)
            continue
        v, m = oracle.plan_cost(p.c[o:o + Lb], p.M[o:o + Lb], p.R[o:o + Lb], plan[i, :Lb])
        assert pins.bits(v) == pins.bits(cost[i]), (p.name, b, e, v, cost[i])
        assert m == mem[i] and m <= e


def pack_models(models):
    """Concatenate PipelineModels (same S and E) into the arrays of one
    gbmw_partition_search call."""
    S, E = models[0].S, models[0].E
    assert all(m.S == S and m.E == E for m in models)
    have_pt = [m.p_t is not None for m in models]
    assert all(have_pt) or not any(have_pt)
    have_split = [m.Ob is not None for m in models]
    assert all(have_split) or not any(have_split)
    cat = lambda name: np.concatenate([getattr(m, name).reshape(m.P * m.Lm, S) for m in models])
    return dict(
        O_b=cat("Ob") if all(have_split) else None, O_ms=cat("Oms") if all(have_split) else None,
        P=np.array([m.P for m in models], np.int32), Lm=np.array([m.Lm for m in models], np.int32),
        m=np.array([m.m for m in models], np.int32),
        c=np.concatenate([m.c for m in models]), c_nosync=np.concatenate([m.c_ns for m in models]),
        R=np.concatenate([m.R for m in models]),
        M=np.concatenate([m.M.reshape(m.P * m.Lm, S) for m in models]),
        p0=np.concatenate([m.p0 for m in models]),
        p_t=np.concatenate([m.p_t for m in models]) if all(have_pt) else None, S=S, E=E)


def check_partition_search(res, models, max_iter):
    """The library's traces against the oracle's, pair by pair, bit for bit."""
    import oracle.bmw as bmw
    for k, mod in enumerate(models):
        ref = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, p_t=mod.p_t, max_iter=max_iter)
        what = f"{mod.name} (pair {k})"
        n = len(ref["trace"])
        assert int(res["n_iter"][k]) == n, (what, int(res["n_iter"][k]), [t["p"] for t in ref["trace"]])
        assert int(res["O_t"][k]) == ref["O_t"], what
        P = mod.P
        for j, t in enumerate(ref["trace"]):
            assert list(res["p"][k, j, :P]) == t["p"], (what, j)
            assert pins.bits(res["cost"][k, j]) == pins.bits(t["cost"]), (what, j, res["cost"][k, j], t["cost"])
            pins.assert_same_f32(res["C"][k, j, :P], t["C"], f"{what} C[{j}]")
            pins.assert_same_f32(res["Cns"][k, j, :P], t["Cns"], f"{what} Cns[{j}]")
            assert [int(x) for x in res["O"][k, j, :P]] == [int(x) for x in t["O"]], (what, j)
            assert pins.bits(res["alpha_t"][k, j]) == pins.bits(t["alpha_t"]), (what, j)
            assert pins.bits(res["alpha_m"][k, j]) == pins.bits(t["alpha_m"]), (what, j)
        assert np.array_equal(res["strat"][k, :mod.Lm], ref["strat"]), what
        assert np.all(res["strat"][k, mod.Lm:] == 255)
        assert not res["p"][k, n:].any() and not res["cost"][k, n:].any()
    return True
