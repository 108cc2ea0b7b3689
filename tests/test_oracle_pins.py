"""The CPU oracle against its pins (hand-worked fixtures, brute force written
separately in Python, closed forms, textbook routines).  CPU only."""
import numpy as np
import pytest

import gbmw_inputs as gi
import oracle
import pins


def solve(c, M, R, E):
    return oracle.solve(np.ascontiguousarray(c, np.float32), np.ascontiguousarray(M, np.int32),
                        np.ascontiguousarray(R, np.float32), E, keep_T=True)


def test_golden_worked_examples():
    pins.pin_golden(solve)


def test_recurrence_equals_brute_force_over_all_plans():
    pins.pin_bruteforce(solve)


def test_special_cases():
    pins.pin_special_cases(solve)


def _cfg3_small():
    """First 6 layers of the structured config with memory scaled down 8x."""
    p = gi.make_config(3)
    return gi.Problem(1, 44, 2048, np.array([6]), p.c[:6], p.M[:6] // 8 + 1, p.R[:6], "cfg3-small")


@pytest.mark.parametrize("make", [
    lambda: gi.make_config(1),
    lambda: gi.random_instance(400, 6, 5, 150, M_rng=(1, 25)),
    lambda: gi.random_instance(401, 9, 7, 300, M_rng=(3, 60), R_rng=(0.0, 20.0)),
    lambda: _cfg3_small(),
])
def test_invariants(make):
    pins.pin_invariants(solve, make())


def test_invariants_config2_full_size():
    pins.pin_invariants(solve, gi.make_config(2))


def test_c_bruteforce_agrees_with_python_bruteforce():
    """The oracle's own enumerator (used at sizes Python cannot reach) against
    the itertools one."""
    for p in pins.tiny_instances():
        opt_py, argopt = pins.py_bruteforce(p.c, p.M, p.R, p.E)
        e_q = p.E
        opt_c, nopt, plan = oracle.bruteforce(p.c, p.M, p.R, p.E, e_q=e_q)
        pins.assert_same_f32(opt_c, opt_py)
        assert [len(a) for a in argopt] == nopt.tolist()
        if np.isfinite(opt_py[e_q]):
            assert tuple(int(x) for x in plan) == min(argopt[e_q])
        else:
            assert all(x == 255 for x in plan)


def test_larger_brute_force_in_c():
    """5^8 = 390625 plans: recurrence == enumeration for every budget."""
    p = gi.random_instance(500, 8, 5, 200, M_rng=(1, 40))
    opt, nopt, plan = oracle.bruteforce(p.c, p.M, p.R, p.E, e_q=p.E)
    sol = solve(p.c, p.M, p.R, p.E)
    pins.assert_same_f32(sol.best, opt)
    got, cost, mem = sol.backtrack(p.E)
    if nopt[p.E] == 1:
        assert np.array_equal(got, plan)
    v, m = oracle.plan_cost(p.c, p.M, p.R, got)
    assert pins.bits(v) == pins.bits(opt[p.E]) and m == mem <= p.E


def test_threads_do_not_change_the_result():
    p = gi.random_instance(600, 7, 6, 500, M_rng=(1, 60))
    a = oracle.solve(p.c, p.M, p.R, p.E, nthreads=1)
    b = oracle.solve(p.c, p.M, p.R, p.E, nthreads=4)
    assert np.array_equal(pins.bits(a.C), pins.bits(b.C)) and np.array_equal(a.A, b.A)
    r = oracle.solve(p.c, p.M, p.R, p.E, keep_C=False, keep_A=False)
    pins.assert_same_f32(r.best, a.best)
    assert np.array_equal(r.best_s, a.best_s)
