"""Pins for the CPU oracle: facts fixed by the paper and by mathematics, each
computed here WITHOUT the oracle's recurrence (hand-worked fixtures, brute-force
enumeration written separately in Python, closed forms, textbook routines).

Every pin takes the solver under test as an argument, so that the same pins can
be run against deliberately broken copies of the oracle (see
test_oracle_mutants.py) to show that a plausible mistake fails at least one.

A "solver" is a callable  solve(c, M, R, E) -> object with fields
C [L][E+1][S], A [L][E+1][S], T [L][E+1][S], best [E+1], best_s [E+1] and a
method backtrack(e) -> (plan, cost, mem).
"""
from __future__ import annotations

import itertools
import json
import os

import numpy as np

import gbmw_inputs as gi

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
INF = np.float32(np.inf)


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def assert_same_f32(a, b, what=""):
    a = np.asarray(a, np.float32)
    b = np.asarray(b, np.float32)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    bad = np.nonzero(bits(a).ravel() != bits(b).ravel())[0]
    assert bad.size == 0, f"{what}: {bad.size} differing cells, first at {bad[0]}: " \
                          f"{a.ravel()[bad[0]]!r} vs {b.ravel()[bad[0]]!r}"


# ---------------------------------------------------------------- helpers
def py_plan_cost(c, M, R, plan):
    """Eq. 3 unrolled along one plan, in numpy float32 scalars:
    v = c[0][s0]; v = (v + R[l][s_{l-1}][s_l]) + c[l][s_l]."""
    v = np.float32(c[0, plan[0]])
    mem = int(M[0, plan[0]])
    for l in range(1, len(plan)):
        v = np.float32(v + R[l, plan[l - 1], plan[l]])
        v = np.float32(v + c[l, plan[l]])
        mem += int(M[l, plan[l]])
    return v, mem


def py_bruteforce(c, M, R, E):
    """OPT(e) = min cost over all S^L plans with memory <= e, plus the set of
    optimal plans per e (written with itertools; shares nothing with the C
    oracle)."""
    L, S = c.shape
    by_mem = {}
    for plan in itertools.product(range(S), repeat=L):
        v, mem = py_plan_cost(c, M, R, plan)
        if mem <= E:
            by_mem.setdefault(mem, []).append((v, plan))
    opt = np.full(E + 1, INF, np.float32)
    argopt = [[] for _ in range(E + 1)]
    cur, cur_plans = INF, []
    for e in range(E + 1):
        for v, plan in by_mem.get(e, ()):
            if v < cur:
                cur, cur_plans = v, [plan]
            elif v == cur:
                cur_plans = cur_plans + [plan]
        opt[e] = cur
        argopt[e] = cur_plans
    return opt, argopt


def py_viterbi_f32(c, R):
    """Unconstrained layered shortest path (textbook Viterbi), float32 with the
    same two roundings per edge: v_l[s] = min_s' ((v_{l-1}[s'] + R_l[s'][s]) + c_l[s])."""
    v = c[0].astype(np.float32).copy()
    for l in range(1, c.shape[0]):
        x = (v[:, None] + R[l]).astype(np.float32)          # [s'][s]
        x = (x + c[l][None, :]).astype(np.float32)
        v = x.min(axis=0)
    return v


def py_mckp_f32(c, M, E):
    """Multiple-choice knapsack (one item per class, weight limit e), float32:
    K_l[e] = min_s K_{l-1}[e - M[l][s]] + c[l][s];  K over all e = 0..E."""
    L, S = c.shape
    e = np.arange(E + 1)
    K = np.full(E + 1, INF, np.float32)
    for s in range(S):
        K = np.minimum(K, np.where(e >= M[0, s], c[0, s], INF).astype(np.float32))
    for l in range(1, L):
        Kn = np.full(E + 1, INF, np.float32)
        for s in range(S):
            m = int(M[l, s])
            sh = np.full(E + 1, INF, np.float32)
            if m <= E:
                sh[m:] = K[:E + 1 - m]
            Kn = np.minimum(Kn, (sh + c[l, s]).astype(np.float32))
        K = Kn
    return K


def _val(x):
    return INF if x == "inf" else np.float32(x)


def _tab(rows):
    return np.array([[_val(x) for x in r] for r in rows], np.float32)


# ---------------------------------------------------------------- the pins
def pin_golden(solve):
    """Hand-worked examples (tests/golden/*.json)."""
    for name in ("worked_example_eq3.json", "worked_example_ties.json"):
        with open(os.path.join(GOLDEN, name)) as f:
            g = json.load(f)
        c = np.array(g["c"], np.float32)
        M = np.array(g["M"], np.int32)
        R = np.array(g["R"], np.float32)
        sol = solve(c, M, R, g["E"])
        for key in ("C0", "C1", "C2"):
            if key in g:
                assert_same_f32(sol.C[int(key[1])], _tab(g[key]), f"{name}:{key}")
        for key in ("T1", "T2"):
            if key in g:
                assert_same_f32(sol.T[int(key[1])], _tab(g[key]), f"{name}:{key}")
        for key in ("A1", "A2"):
            if key in g:
                assert np.array_equal(sol.A[int(key[1])], np.array(g[key], np.uint8)), f"{name}:{key}"
        assert_same_f32(sol.best, np.array([_val(x) for x in g["best"]]), f"{name}:best")
        assert np.array_equal(sol.best_s, np.array(g["best_s"], np.uint8)), f"{name}:best_s"
        for e, plan in g["plans"].items():
            p, cost, mem = sol.backtrack(int(e))
            assert list(p) == plan, (name, e, list(p), plan)
            assert mem == g["plan_mem"][e]
            assert cost == _val(g["best"][int(e)])
        for e in range(g["E"] + 1):
            if g["best"][e] == "inf":
                p, cost, mem = sol.backtrack(e)
                assert list(p) == [255] * g["L"] and mem == -1 and cost == INF


def tiny_instances():
    """cfg1 plus random tiny instances, some with budgets too small for any or
    for most plans."""
    out = [gi.make_config(1)]
    for seed, (L, S, E, Mhi) in enumerate([(1, 3, 20, 8), (2, 4, 40, 16), (3, 3, 30, 12),
                                           (4, 4, 64, 32), (5, 3, 48, 16), (6, 2, 40, 10),
                                           (3, 4, 5, 6), (4, 3, 9, 4), (5, 2, 64, 20),
                                           (4, 4, 200, 32)]):
        out.append(gi.random_instance(100 + seed, L, S, E, M_rng=(1, Mhi)))
    # asymmetric, non-zero-diagonal R and a wide value range (rounding matters)
    p = gi.random_instance(200, 5, 3, 60, c_rng=(0.001, 1000.0), R_rng=(0.0, 300.0), M_rng=(1, 20))
    p.R[:] = gi.Stream(201).uniform(p.R.size, 0.0, 300.0).reshape(p.R.shape)
    out.append(p)
    return out


def pin_bruteforce(solve, instances=None):
    """Optimal substructure (Appendix A2): the recurrence's best[e] equals the
    minimum over ALL plans with memory <= e, for every e, bit for bit; the
    backtracked plan is one of the optimal plans."""
    for p in (instances or tiny_instances()):
        c, M, R = p.c, p.M, p.R
        opt, argopt = py_bruteforce(c, M, R, p.E)
        sol = solve(c, M, R, p.E)
        assert_same_f32(sol.best, opt, f"{p.name}: best vs brute force")
        for e in range(p.E + 1):
            plan, cost, mem = sol.backtrack(e)
            if opt[e] == INF:
                assert mem == -1 and all(x == 255 for x in plan)
                continue
            assert tuple(int(x) for x in plan) in argopt[e], (p.name, e, plan, argopt[e])
            v, m = py_plan_cost(c, M, R, [int(x) for x in plan])
            assert bits(v) == bits(cost) == bits(opt[e]) and m == mem and m <= e


def pin_invariants(solve, p):
    """Facts that hold at any size (single instance p)."""
    c, M, R, E = p.c, p.M, p.R, p.E
    L, S = c.shape
    sol = solve(c, M, R, E)
    C, A, T = sol.C, sol.A, sol.T
    # 1. a larger budget never costs more (Eq. 3 constraint is "at most")
    assert np.all(C[:, 1:, :] <= C[:, :-1, :]), "C not non-increasing in e"
    assert np.all(sol.best[1:] <= sol.best[:-1])
    assert not np.isnan(C).any()
    # 2. the infeasible region in closed form: C[l][e][s] is +inf exactly when
    #    e < M[l][s] + sum_{k<l} min_s M[k][s]   (all inputs finite)
    if np.isfinite(c).all() and np.isfinite(R).all():
        minmem = np.concatenate([[0], np.cumsum(M.min(axis=1))[:-1]])      # [L]
        thr = M + minmem[:, None]                                         # [L][S]
        e = np.arange(E + 1)[None, :, None]
        assert np.array_equal(np.isinf(C), e < thr[:, None, :]), "inf pattern"
    # 3. with enough budget for anything, the table equals the unconstrained
    #    layered shortest path (Viterbi)
    emax = int(M.max(axis=1).sum())
    if emax <= E:
        assert_same_f32(C[L - 1, emax], py_viterbi_f32(c, R), "saturated row vs Viterbi")
        assert_same_f32(C[L - 1, E], C[L - 1, emax], "constant beyond sum of max M")
    # 4. argmin records: T is reproduced by the recorded predecessor, no earlier
    #    predecessor reaches it, and all-infinite cells record 0
    for l in range(1, L):
        for s in range(S):
            x = (C[l - 1] + R[l][:, s][None, :]).astype(np.float32)       # [e][s']
            a = A[l][:, s].astype(np.int64)
            got = np.take_along_axis(x, a[:, None], axis=1)[:, 0]
            assert_same_f32(got, T[l][:, s], f"A reproduces T, l={l}, s={s}")
            assert_same_f32(x.min(axis=1), T[l][:, s], f"T is the row min, l={l}, s={s}")
            first = np.argmax(x == T[l][:, s][:, None], axis=1)
            assert np.array_equal(first, a), f"lowest-index argmin, l={l}, s={s}"
            assert np.all(a[np.isinf(T[l][:, s])] == 0)
    # 5. the shift: C_l[e][s] = T_l[e - M][s] + c, +inf below M
    for l in range(1, L):
        for s in range(S):
            m = int(M[l, s])
            exp = np.full(E + 1, INF, np.float32)
            if m <= E:
                exp[m:] = (T[l][:E + 1 - m, s] + c[l, s]).astype(np.float32)
            assert_same_f32(C[l][:, s], exp, f"shift-add, l={l}, s={s}")
    # 6. final reduce
    assert_same_f32(sol.best, C[L - 1].min(axis=1), "best")
    assert np.array_equal(sol.best_s, np.argmax(C[L - 1] == sol.best[:, None], axis=1))
    # 7. plans: re-evaluating the plan by the plain definition gives best[e]
    #    exactly, within the budget
    for e in sorted(set([0, E, E // 2, E // 3, int(M.min(axis=1).sum()),
                         max(0, int(M.min(axis=1).sum()) - 1)]
                        + list(range(0, E + 1, max(1, E // 37))))):
        if e > E:
            continue
        plan, cost, mem = sol.backtrack(e)
        if np.isinf(sol.best[e]):
            assert mem == -1 and all(x == 255 for x in plan) and cost == INF
        else:
            v, m = py_plan_cost(c, M, R, [int(x) for x in plan])
            assert bits(v) == bits(cost) == bits(sol.best[e]), (e, v, cost, sol.best[e])
            assert m == mem and m <= e
    return sol


def pin_special_cases(solve):
    # R == 0: the problem separates into a multiple-choice knapsack
    p = gi.random_instance(300, 6, 5, 120, M_rng=(1, 30))
    p.R[:] = 0
    sol = solve(p.c, p.M, p.R, p.E)
    assert_same_f32(sol.best, py_mckp_f32(p.c, p.M, p.E), "R=0 vs knapsack")
    for l in range(1, 6):        # predecessor does not depend on s
        assert np.all(sol.A[l] == sol.A[l][:, :1])
        assert np.array_equal(sol.A[l][:, 0], np.argmax(sol.C[l - 1] == sol.C[l - 1].min(axis=1)[:, None], axis=1))
    # S == 1: a left-to-right float32 sum once the budget covers sum M
    p = gi.random_instance(301, 7, 1, 100, M_rng=(1, 20), R_rng=(0.0, 3.0))
    p.R[:] = gi.Stream(302).uniform(p.R.size, 0.0, 3.0).reshape(p.R.shape)   # diagonal non-zero
    sol = solve(p.c, p.M, p.R, p.E)
    v = np.float32(p.c[0, 0])
    for l in range(1, 7):
        v = np.float32(np.float32(v + p.R[l, 0, 0]) + p.c[l, 0])
    need = int(p.M.sum())
    assert need <= p.E
    assert np.all(np.isinf(sol.best[:need])) and np.all(bits(sol.best[need:]) == bits(v))
    # L == 1: base case only
    p = gi.random_instance(303, 1, 4, 40, M_rng=(1, 30))
    sol = solve(p.c, p.M, p.R, p.E)
    e = np.arange(41)[:, None]
    assert_same_f32(sol.C[0], np.where(e >= p.M[0][None, :], p.c[0][None, :], INF))
    # E below every first-layer memory: nothing is feasible
    p = gi.random_instance(304, 3, 3, 4, M_rng=(5, 9))
    sol = solve(p.c, p.M, p.R, p.E)
    assert np.all(np.isinf(sol.C)) and np.all(np.isinf(sol.best)) and np.all(sol.A == 0) and np.all(sol.best_s == 0)
    # E == 0 with zero-memory strategies is feasible (nothing special about e = 0)
    p = gi.random_instance(305, 3, 2, 0, M_rng=(0, 0))
    sol = solve(p.c, p.M, p.R, p.E)
    opt, _ = py_bruteforce(p.c, p.M, p.R, 0)
    assert np.isfinite(opt[0]) and bits(sol.best[0]) == bits(opt[0])
    # duplicated strategy columns: the lower index must win everywhere
    p = gi.random_instance(306, 5, 3, 80, M_rng=(1, 20))
    c2 = np.concatenate([p.c, p.c], axis=1)
    M2 = np.concatenate([p.M, p.M], axis=1)
    R2 = np.ascontiguousarray(np.tile(p.R, (1, 2, 2)))
    sol = solve(np.ascontiguousarray(c2), np.ascontiguousarray(M2), R2, p.E)
    assert np.all(sol.A < 3) and np.all(sol.best_s < 3)
    ref = solve(p.c, p.M, p.R, p.E)
    assert_same_f32(sol.best, ref.best)
    assert_same_f32(sol.C[:, :, :3], ref.C, "duplicated columns leave C unchanged")
    assert np.array_equal(sol.A[:, :, :3], ref.A) and np.array_equal(sol.A[:, :, 3:], ref.A)
    # +inf costs forbid a strategy or a transition without producing NaN
    p = gi.random_instance(307, 4, 3, 60, M_rng=(1, 12))
    p.c[1, 2] = INF
    p.R[2, 0, 1] = INF
    p.R[3, :, 0] = INF
    sol = solve(p.c, p.M, p.R, p.E)
    assert not np.isnan(sol.C).any()
    opt, argopt = py_bruteforce(p.c, p.M, p.R, p.E)
    assert_same_f32(sol.best, opt, "inf costs vs brute force")
    for e in range(p.E + 1):
        if np.isfinite(opt[e]):
            plan, _, _ = sol.backtrack(e)
            assert plan[1] != 2 and plan[3] != 0 and not (plan[1] == 0 and plan[2] == 1)


# ---------------------------------------------------------------- Algorithm 3 outer loop
def py_e_all(Of, Ob, Oms, plan):
    """Eq. 2 written out: max over i of (forward activations of layers <= i plus
    backward activations of layer i), plus the model states of all layers."""
    L = len(plan)
    ms = sum(int(Oms[k, plan[k]]) for k in range(L))
    return max(sum(int(Of[k, plan[k]]) for k in range(i + 1)) + int(Ob[i, plan[i]]) for i in range(L)) + ms


def py_select(sol, Of, Ob, Oms, E):
    """Algorithm 3's loop in Python on top of a solver's best[] and plans."""
    b_up = int(Ob.max())
    opt = E - b_up if E - b_up >= 0 else -1
    for e in range(opt + 1, E + 1):
        if np.isinf(sol.best[e]):
            continue
        plan, _, _ = sol.backtrack(e)
        if py_e_all(Of, Ob, Oms, [int(x) for x in plan]) <= E:
            opt = e
        else:
            break
    if opt < 0 or np.isinf(sol.best[opt]):
        return opt, INF, None, -1
    plan, cost, _ = sol.backtrack(opt)
    return opt, cost, plan, py_e_all(Of, Ob, Oms, [int(x) for x in plan])


def pin_select_golden(solve, select, e_all):
    with open(os.path.join(GOLDEN, "worked_example_alg3.json")) as f:
        g = json.load(f)
    with open(os.path.join(GOLDEN, g["base"])) as f:
        b = json.load(f)
    c = np.array(b["c"], np.float32); M = np.array(b["M"], np.int32); R = np.array(b["R"], np.float32)
    Of = np.array(g["Of"], np.int32); Oms = np.array(g["Oms"], np.int32)
    assert np.array_equal(Of + Oms, M)
    sol = solve(c, M, R, b["E"])
    for case in g["cases"]:
        Ob = np.array(case["Ob"], np.int32)
        for k, v in case["e_all_of"].items():
            plan = [int(x) for x in k.split(",")]
            assert e_all(Of, Ob, Oms, plan) == v == py_e_all(Of, Ob, Oms, plan), (k, v)
        e_opt, cost, plan, ea = select(sol, Of, Ob, Oms)
        assert (e_opt, float(cost), list(plan), ea) == (case["e_opt"], case["cost"], case["plan"], case["e_all"])


def pin_select_properties(solve, select, e_all):
    for seed, (L, S, E, Mhi) in enumerate([(4, 4, 120, 30), (6, 3, 90, 20), (5, 5, 60, 25), (3, 4, 40, 30),
                                           (7, 2, 200, 40), (4, 3, 10, 12)]):
        p = gi.random_instance(700 + seed, L, S, E, M_rng=(1, Mhi))
        sol = solve(p.c, p.M, p.R, E)
        for variant in range(3):
            Of, Ob, Oms = gi.split_memory(p, 800 + 10 * seed + variant)
            if variant == 1:
                Ob[:] = 0                       # no backward peak: every budget is valid
            if variant == 2:
                Ob[:] = np.minimum(Ob, 3)       # tiny window
            b_up = int(Ob.max())
            # E_all against the definition, for the plans of all budgets
            for e in range(E + 1):
                if np.isfinite(sol.best[e]):
                    plan, _, mem = sol.backtrack(e)
                    ea = e_all(Of, Ob, Oms, plan)
                    assert ea == py_e_all(Of, Ob, Oms, [int(x) for x in plan])
                    assert mem <= ea <= mem + b_up          # E_f <= E_all <= E_f + b_up
                    if e <= E - b_up:
                        assert ea <= E                      # no check needed below E - b_up
            got = select(sol, Of, Ob, Oms)
            exp = py_select(sol, Of, Ob, Oms, E)
            assert got[0] == exp[0] and bits(got[1]) == bits(exp[1]) and got[3] == exp[3], (got, exp)
            if exp[2] is None:
                assert all(x == 255 for x in got[2])
            else:
                assert np.array_equal(got[2], exp[2]) and got[3] <= E
            if variant == 1 and np.isfinite(sol.best[E]):
                assert got[0] == E


def run_all_pins(solve):
    pin_golden(solve)
    pin_bruteforce(solve)
    pin_special_cases(solve)
    pin_invariants(solve, gi.make_config(1))
    pin_invariants(solve, gi.random_instance(400, 6, 5, 150, M_rng=(1, 25)))
