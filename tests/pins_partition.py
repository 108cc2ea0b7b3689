"""Pins of the oracle's pipeline-partition search (Algorithm 2's inner loop):
a hand-worked fixture, closed forms on uniform models, brute force of every
stage on tiny models, and the properties Section 4.2.2 / Appendix B state.
Each pin takes the module under test, so that the mutation tests can hand in a
deliberately broken copy."""
import itertools
import json
import os

import numpy as np

import gbmw_inputs as gi
import pins

INT_MAX = 2**31 - 1


def _frac(x):
    return float(x[0]) / float(x[1])


def fixture_model(g, case):
    mo = g["model"]
    Lm, S, P = mo["Lm"], mo["S"], mo["P"]
    R = np.full((Lm, S, S), mo["R_offdiag"], np.float32)
    R[:, np.arange(S), np.arange(S)] = 0.0
    Ms = case.get("M_stage", mo["M_stage"])
    M = np.array([[Ms[i]] * Lm for i in range(P)], np.int32)
    model = dict(c=np.array(mo["c"], np.float32), c_ns=np.array(mo["c_ns"], np.float32), R=R, M=M)
    if "Ob_stage" in case:                       # Algorithm 3 stage searches (Eq. 2's memory split)
        model["Ob"] = np.array([[case["Ob_stage"][i]] * Lm for i in range(P)], np.int32)
        model["Oms"] = np.array([[case["Oms_stage"][i]] * Lm for i in range(P)], np.int32)
    return model, mo["m"]


def check_trace_against(case, res):
    assert res["O_t"] == case["O_t"], (case["name"], res["O_t"])
    assert len(res["trace"]) == len(case["trace"]), (case["name"], [t["p"] for t in res["trace"]])
    for got, want in zip(res["trace"], case["trace"]):
        assert list(got["p"]) == want["p"]
        assert float(got["cost"]) == float(pins._val(want["cost"])), (case["name"], got["cost"])
        assert [float(x) for x in got["C"]] == [float(pins._val(x)) for x in want["C"]]
        assert [float(x) for x in got["Cns"]] == [float(pins._val(x)) for x in want["Cns"]]
        assert [int(x) for x in got["O"]] == want["O"]
        assert abs(float(got["alpha_t"]) - _frac(want["alpha_t"])) < 1e-6
        assert abs(float(got["alpha_m"]) - _frac(want["alpha_m"])) < 1e-6
    assert [int(x) for x in res["strat"]] == case["strat"]


def pin_fixture(bmw):
    with open(os.path.join(pins.GOLDEN, "worked_example_partition.json")) as f:
        g = json.load(f)
    for case in g["cases"]:
        model, m = fixture_model(g, case)
        res = bmw.partition_search(model, case["p0"], case["E"], m, p_t=case["p_t"], max_iter=16)
        check_trace_against(case, res)


def _stage_time(n, cost, r):
    return n * cost + (n - 1) * r


def pin_uniform_two_stages(bmw):
    """S = 1, all layers alike, P = 2, p0 = [1, Lm-1]: the slowest stage is the
    second until the halves meet, so the trace is [1,Lm-1], [2,Lm-2], ...  For
    even Lm it ends at [h,h] (the move on to [h-1,h+1] would exceed the maximum);
    for odd Lm it passes [h,h+1] -> [h+1,h] (equal maximum, allowed) and ends
    there because [h,h+1] has been searched."""
    for Lm in (6, 7, 10, 11):
        mod = gi.uniform_pipeline_model(Lm, 2, 1000, [1, Lm - 1], cost=2.0, r=0.5, m=3)
        res = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, max_iter=64)
        h = Lm // 2
        want = [[a, Lm - a] for a in range(1, h + 1)] + ([[h + 1, h]] if Lm % 2 else [])
        assert [t["p"] for t in res["trace"]] == want, (Lm, [t["p"] for t in res["trace"]])
        for t in res["trace"]:
            C = [_stage_time(n, 2.0, 0.5) for n in t["p"]]
            Cns = [_stage_time(n, 1.0, 0.5) for n in t["p"]]
            assert [float(x) for x in t["C"]] == C and [float(x) for x in t["Cns"]] == Cns
            assert float(t["cost"]) == (mod.m - 1) * max(Cns) + sum(C)
            assert [int(x) for x in t["O"]] == t["p"]
            assert abs(float(t["alpha_t"]) - (1 - max(C) / sum(C))) < 1e-6
            assert abs(float(t["alpha_m"]) - (1 - max(t["p"]) / Lm)) < 1e-6
        # max_iter cuts the trace short
        cut = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, max_iter=2)
        assert [t["p"] for t in cut["trace"]] == want[:2]


def pin_uniform_memory_limits(bmw):
    """Same model, but stage 0 pays 3 units per layer and the budget is 9: the
    stage can hold 3 layers, so [4, 6] fails limit 2 and the trace ends at
    [3, 7].  With p_t = [2, 8] (largest stage memory max(6, 8) = 8) limit 3
    stops one step earlier still: [3, 7] would put 9 > 8 on stage 0."""
    mod = gi.uniform_pipeline_model(10, 2, 9, [1, 9], mem=[3, 1])
    res = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m)
    assert [t["p"] for t in res["trace"]] == [[1, 9], [2, 8], [3, 7]] and res["O_t"] == INT_MAX
    res = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, p_t=[2, 8])
    assert [t["p"] for t in res["trace"]] == [[1, 9], [2, 8]] and res["O_t"] == 8
    # an infeasible p_t sets no limit 3
    res = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, p_t=[5, 5])
    assert [t["p"] for t in res["trace"]] == [[1, 9], [2, 8], [3, 7]] and res["O_t"] == INT_MAX
    # an infeasible first partition: one entry, infinite cost
    res = bmw.partition_search(mod.as_dict(), [4, 6], mod.E, mod.m)
    assert len(res["trace"]) == 1 and np.isinf(res["trace"][0]["cost"])
    assert [int(x) for x in res["trace"][0]["O"]] == [-1, 6]


def pin_uniform_three_stages(bmw):
    """P = 3, S = 1: which neighbour takes the layer.  [2,6,2]: the middle is
    slowest, its neighbours tie, the earlier one takes the FIRST layer of the
    middle stage -> [3,5,2]; then stage 2 is the cheaper neighbour and takes the
    LAST layer -> [3,4,3]; then stage 0 again -> [4,3,3]: its time equals the old
    maximum (allowed); now stage 0 is slowest, its only neighbour is stage 1 ->
    [3,4,3], already searched: the end.  [7,2,1]: stage 0 can only give to
    stage 1 although stage 2 is cheaper."""
    mod = gi.uniform_pipeline_model(10, 3, 1000, [2, 6, 2])
    res = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m)
    assert [t["p"] for t in res["trace"]] == [[2, 6, 2], [3, 5, 2], [3, 4, 3], [4, 3, 3]]
    res = bmw.partition_search(mod.as_dict(), [7, 2, 1], mod.E, mod.m)
    assert [t["p"] for t in res["trace"]][:3] == [[7, 2, 1], [6, 3, 1], [5, 4, 1]]
    # two slowest stages: the earlier one gives ([4,2,4] -> [3,3,4], not [4,3,3] yet)
    res = bmw.partition_search(mod.as_dict(), [4, 2, 4], mod.E, mod.m)
    assert [t["p"] for t in res["trace"]] == [[4, 2, 4], [3, 3, 4], [3, 4, 3], [4, 3, 3]]
    # a single stage has no neighbour: one search, no adjustment
    one = gi.uniform_pipeline_model(5, 1, 1000, [5])
    res = bmw.partition_search(one.as_dict(), one.p0, one.E, one.m)
    assert [t["p"] for t in res["trace"]] == [[5]] and float(res["trace"][0]["alpha_t"]) == 0.0
    # a slowest stage of one layer keeps it, even where limit 1 would let it go
    # (the neighbour costs nothing, so taking the layer would only reach the old maximum)
    free = gi.uniform_pipeline_model(3, 2, 1000, [1, 2], r=0.0)
    free.c[1:] = 0.0
    res = bmw.partition_search(free.as_dict(), free.p0, free.E, free.m)
    assert [t["p"] for t in res["trace"]] == [[1, 2]]
    # stages of one layer each: nothing to give away
    flat = gi.uniform_pipeline_model(3, 3, 1000, [1, 1, 1])
    res = bmw.partition_search(flat.as_dict(), flat.p0, flat.E, flat.m)
    assert len(res["trace"]) == 1


def _stage_bruteforce(mod, i, a, n, E):
    """Best (cost, mem, plan) of layers [a, a+n) in stage i over all S^n plans
    that fit E (first in lexicographic order among equals is not needed: the
    callers use instances without ties at e = E)."""
    best = (pins.INF, -1, None)
    cnt = 0
    for plan in itertools.product(range(mod.S), repeat=n):
        v, mem = pins.py_plan_cost(mod.c[a:a + n], mod.M[i][a:a + n], mod.R[a:a + n], plan)
        if mem <= E:
            if v < best[0]:
                best, cnt = (v, mem, plan), 1
            elif v == best[0]:
                cnt += 1
    return best, cnt


def pin_properties(bmw, seeds=range(12)):
    """Random tiny models: every stage time is the brute-force optimum of its
    layer slice under ITS stage's memory; the cost is Eq. 8 of the stage times;
    and along the trace: partitions are compositions of Lm, all different, each
    made from the last by moving one boundary layer out of the slowest stage
    into a neighbour; the maximum stage time never rises (limit 1 plus the
    optimality of the re-search); every stage fits E."""
    n_multi = 0
    for seed in seeds:
        st = gi.Stream(7000 + seed)
        P = int(st.integers(1, 2, 4)[0])
        Lm = int(st.integers(1, P + 2, 9)[0])
        S = int(st.integers(1, 2, 3)[0])
        mod = gi.random_pipeline_model(seed, Lm, S, P, E=int(st.integers(1, 30, 70)[0]), m=int(st.integers(1, 1, 6)[0]))
        res = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, p_t=mod.p_t, max_iter=32)
        tr = res["trace"]
        assert 1 <= len(tr) <= 32
        n_multi += len(tr) > 1
        seen = set()
        for k, t in enumerate(tr):
            p = t["p"]
            assert len(p) == P and min(p) >= 1 and sum(p) == Lm and tuple(p) not in seen
            seen.add(tuple(p))
            a = 0
            for i, n in enumerate(p):
                (v, mem, plan), cnt = _stage_bruteforce(mod, i, a, n, mod.E)
                assert pins.bits(t["C"][i]) == pins.bits(v), (seed, k, i)
                if not np.isinf(v) and cnt == 1:
                    assert int(t["O"][i]) == mem and int(t["O"][i]) <= mod.E
                    if k == len(tr) - 1:
                        assert [int(x) for x in res["strat"][a:a + n]] == list(plan)
                    vns, _ = pins.py_plan_cost(mod.c_ns[a:a + n], mod.M[i][a:a + n], mod.R[a:a + n], plan)
                    assert pins.bits(t["Cns"][i]) == pins.bits(vns)
                a += n
            feasible = not any(np.isinf(x) for x in t["C"])
            assert np.isinf(t["cost"]) == (not feasible)
            if feasible:
                tot = np.float32(0)
                for x in t["C"]:
                    tot = np.float32(tot + x)
                want = np.float32(np.float32(np.float32(mod.m - 1) * max(t["Cns"])) + tot)
                assert pins.bits(t["cost"]) == pins.bits(want)
                assert -1e-6 <= float(t["alpha_t"]) <= 1 - 1 / P + 1e-6
                assert -1e-6 <= float(t["alpha_m"]) <= 1 - 1 / P + 1e-6
            else:
                assert k == len(tr) - 1
            if k > 0:
                q, C = tr[k - 1]["p"], tr[k - 1]["C"]
                i = int(np.argmax(C))
                d = [x - y for x, y in zip(p, q)]
                assert d[i] == -1 and sorted(d) == [-1] + [0] * (P - 2) + [1]
                j = d.index(1)
                assert abs(j - i) == 1
                other = 2 * i - j
                if 0 <= other < P:
                    assert (C[j], j) < (C[other], other)
                assert max(t["C"]) <= max(C)
    assert n_multi >= 4, "the random models must exercise the adjustment"


def _stage_alg3_bruteforce(mod, i, a, n):
    """Appendix A, Algorithm 3 for layers [a, a+n) in stage i from the list of
    optimal plans per budget (brute force): (cost, E_all, plan), or None where
    some budget in the walk has several optimal plans (the result then depends
    on the tie rule, which other pins cover)."""
    E = mod.E
    sl = slice(a, a + n)
    Oms, Ob = mod.Oms[i][sl], mod.Ob[i][sl]
    Of = mod.M[i][sl] - Oms
    opt, argopt = pins.py_bruteforce(mod.c[sl], mod.M[i][sl], mod.R[sl], E)
    b_up = int(Ob.max())
    e_opt = E - b_up if E >= b_up else -1
    for e in range(e_opt + 1, E + 1):
        if np.isinf(opt[e]):
            continue
        if len(argopt[e]) != 1:
            return None
        if pins.py_e_all(Of, Ob, Oms, argopt[e][0]) <= E:
            e_opt = e
        else:
            break
    if e_opt < 0 or np.isinf(opt[e_opt]):
        return pins.INF, -1, None
    if len(argopt[e_opt]) != 1:
        return None
    plan = argopt[e_opt][0]
    return opt[e_opt], pins.py_e_all(Of, Ob, Oms, plan), plan


def pin_alg3_in_loop(bmw, seeds=range(14)):
    """Stage searches with the overall-memory check (Appendix A, Algorithm 3;
    Eq. 2).  (1) With O_b = 0 the overall memory of a plan is its forward
    memory, every budget is valid and the trace is that of the plain search.
    (2) With random O_b every stage's (time, memory, plan) is what the
    algorithm gives on the brute-force list of optimal plans, the memory is
    E_all <= E, and an accepted move keeps E_all of every stage under the kept
    strategies within E and O_t."""
    n_checked = n_bound = n_multi = 0
    for seed in seeds:
        st = gi.Stream(7100 + seed)
        P = int(st.integers(1, 2, 4)[0])
        Lm = int(st.integers(1, P + 2, 8)[0])
        S = int(st.integers(1, 2, 3)[0])
        E = int(st.integers(1, 25, 60)[0])
        base = gi.random_pipeline_model(100 + seed, Lm, S, P, E=E, m=int(st.integers(1, 1, 6)[0]),
                                        R_rng=(0.0, 0.5), skew=bool(seed % 2))
        plain = bmw.partition_search(base.as_dict(), base.p0, E, base.m, p_t=base.p_t, max_iter=32)
        zero = gi.with_memory_split(base, 40 + seed)
        zero.Ob[:] = 0
        res = bmw.partition_search(zero.as_dict(), zero.p0, E, zero.m, p_t=zero.p_t, max_iter=32)
        assert res["O_t"] == plain["O_t"] and len(res["trace"]) == len(plain["trace"])
        for t, u in zip(res["trace"], plain["trace"]):
            assert list(t["p"]) == list(u["p"]) and pins.bits(t["cost"]) == pins.bits(u["cost"])
            pins.assert_same_f32(t["C"], u["C"]); pins.assert_same_f32(t["Cns"], u["Cns"])
            assert [int(x) for x in t["O"]] == [int(x) for x in u["O"]]
        assert np.array_equal(res["strat"], plain["strat"])

        mod = gi.with_memory_split(base, 60 + seed, ob_max=int(st.integers(1, 2, 12)[0]))
        res = bmw.partition_search(mod.as_dict(), mod.p0, E, mod.m, p_t=mod.p_t, max_iter=32)
        tr = res["trace"]
        n_multi += len(tr) > 1
        for k, t in enumerate(tr):
            a = 0
            for i, n in enumerate(t["p"]):
                want = _stage_alg3_bruteforce(mod, i, a, n)
                if want is not None:
                    v, mem, plan = want
                    n_checked += 1
                    assert pins.bits(t["C"][i]) == pins.bits(v), (seed, k, i)
                    assert int(t["O"][i]) == mem and mem <= E
                    if plan is not None:
                        plain_best, _ = _stage_bruteforce(mod, i, a, n, E)
                        n_bound += plain_best[0] < v          # the check made the stage slower
                        if k == len(tr) - 1:
                            assert [int(x) for x in res["strat"][a:a + n]] == list(plan)
                a += n
        # accepted moves: E_all under the kept strategies within the limits (needs the
        # strategies of every round: recompute them stage by stage from the brute force)
        for k in range(1, len(tr)):
            q, p = tr[k]["p"], tr[k - 1]["p"]
            kept, a, ok = [], 0, True
            for i, n in enumerate(p):
                want = _stage_alg3_bruteforce(mod, i, a, n)
                ok = ok and want is not None and want[2] is not None
                kept += list(want[2]) if ok else []
                a += n
            if not ok:
                continue
            a = 0
            for i, n in enumerate(q):
                sl = slice(a, a + n)
                ea = pins.py_e_all(mod.M[i][sl] - mod.Oms[i][sl], mod.Ob[i][sl], mod.Oms[i][sl], kept[sl])
                assert ea <= E and ea <= res["O_t"], (seed, k, i)
                a += n
    assert n_checked >= 30 and n_bound >= 3 and n_multi >= 3, (n_checked, n_bound, n_multi)


def pin_throughput(bmw):
    """Outer loops: best pipeline time over the PP degrees per batch size, the
    best batch/time, stopping at the first batch size with no feasible degree."""
    inf = np.float32(np.inf)
    t, k = bmw.throughput([8, 16, 24], [[4.0, 2.0], [inf, 5.0], [12.0, 6.0]])
    assert (float(t), k) == (4.0, 0)                   # 8/2 = 4 > 16/5 ; 24/6 = 4 is not greater
    t, k = bmw.throughput([8, 16, 24], [[4.0, 8.0], [inf, 3.0], [1.0, 6.0]])
    assert (float(t), k) == (24.0, 2)
    t, k = bmw.throughput([8, 16, 24], [[4.0, 8.0], [inf, inf], [1.0, 6.0]])
    assert (float(t), k) == (2.0, 0)                   # out of memory at 16: 24 is never tried
    t, k = bmw.throughput([8], [[inf]])
    assert (float(t), k) == (0.0, -1)


def run_all(bmw):
    pin_fixture(bmw)
    pin_uniform_two_stages(bmw)
    pin_uniform_memory_limits(bmw)
    pin_uniform_three_stages(bmw)
    pin_properties(bmw)
    pin_alg3_in_loop(bmw)
    pin_throughput(bmw)
