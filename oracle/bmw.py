"""Bi-objective pipeline-partition search of one (batch size, PP degree) pair --
TEST INFRASTRUCTURE ONLY (see the package docstring for who may import this).

Follows Algorithm 2's inner loop (queue of partitions, Galvatron_Search,
PP_Partition_Adjust, Validate), Section 4.2.2's description of the adjustment
and its three limits, Eq. 6 (balance degrees), Eq. 8 (pipeline time) and
Appendix B.  Plain Python over the C oracle's table solve; nothing here is
blocked, cached or reused between iterations: every searched partition solves
all of its stages from scratch.

Notation: a partition p is the list of layer counts per stage; stage i of p
holds the model's layers [a_i, a_i + p_i) with a_i = p_0 + ... + p_{i-1}.
Model: c, c_ns [Lm][S] (layer time with / without gradient synchronisation),
R [Lm][S][S] (R[l][s'][s]: layer l-1 under s' to layer l under s; not charged
for the first layer of a stage), M [P][Lm][S] (memory of layer l under s when
it sits in stage i: under 1F1B a shallower stage stashes more activations).

With the optional tables O_b and O_ms [P][Lm][S] in the model (O_f = M - O_ms;
Eq. 2) a stage is searched as Appendix A, Algorithm 3 does it: the plan is read
at the largest forward budget whose overall memory E_all fits E, and the memory
of a stage, in the balance degrees and in limits 2 and 3, is E_all of its plan.

Where the paper leaves a choice open, the reading taken is marked READING.
"""
from __future__ import annotations

import numpy as np

from . import e_all, pipeline_cost, plan_cost, select_budget, solve

INT_MAX = 2**31 - 1


def starts(p):
    a = [0]
    for n in p[:-1]:
        a.append(a[-1] + int(n))
    return a


def stage_under_plan(model, i, a, n, strat):
    """Time (fp32, in the recurrence's order), time without gradient
    synchronisation and memory of layers [a, a+n) placed in stage i, every
    layer keeping its strategy strat[l]."""
    sl = slice(a, a + n)
    M = np.ascontiguousarray(model["M"][i][sl])
    C, O = plan_cost(np.ascontiguousarray(model["c"][sl]), M, np.ascontiguousarray(model["R"][sl]), strat[sl])
    Cns, _ = plan_cost(np.ascontiguousarray(model["c_ns"][sl]), M, np.ascontiguousarray(model["R"][sl]), strat[sl])
    if "Ob" in model:                                      # overall memory of the plan (Eq. 2)
        Of, Ob, Oms = stage_memory_tables(model, i, sl)
        O = e_all(Of, Ob, Oms, strat[sl])
    return C, Cns, O


def stage_memory_tables(model, i, sl):
    """O_f, O_b, O_ms of layers sl placed in stage i, with O_f = M - O_ms."""
    Oms = np.ascontiguousarray(model["Oms"][i][sl])
    Ob = np.ascontiguousarray(model["Ob"][i][sl])
    Of = np.ascontiguousarray(model["M"][i][sl] - Oms)
    return Of, Ob, Oms


def galvatron_search(model, p, E, m):
    """Galvatron_Search of Algorithm 1/2 for one pipeline: every stage's table
    solve under budget E, the plan at e = E, and the pipeline time of Eq. 8.
    Returns (cost, C[P], Cns[P], O[P], strat[Lm]); an infeasible stage has
    C = Cns = inf and O = -1, and makes the cost inf."""
    P, Lm = len(p), model["c"].shape[0]
    C = np.full(P, np.inf, np.float32)
    Cns = np.full(P, np.inf, np.float32)
    O = np.full(P, -1, np.int64)
    strat = np.full(Lm, 0xFF, np.uint8)
    for i, (a, n) in enumerate(zip(starts(p), p)):
        sl = slice(a, a + n)
        sol = solve(np.ascontiguousarray(model["c"][sl]), np.ascontiguousarray(model["M"][i][sl]),
                    np.ascontiguousarray(model["R"][sl]), E, keep_C=False)
        if "Ob" in model:                                  # Algorithm 3: largest valid forward budget
            Of, Ob, Oms = stage_memory_tables(model, i, sl)
            _, cost, plan, mem = select_budget(sol, Of, Ob, Oms)
        else:
            plan, cost, mem = sol.backtrack(E)
        if np.isinf(cost):
            continue
        strat[sl] = plan
        C[i], O[i] = cost, mem
        Cns[i] = stage_under_plan(model, i, a, n, strat)[1]
    cost = pipeline_cost(m, C, Cns)
    return cost, C, Cns, O, strat


def balance_degrees(C, O):
    """Eq. 6.  alpha_t in fp32 (stage times are fp32, summed in stage order),
    alpha_m in fp64 from the integer memories, rounded to fp32.
    READING: a zero sum gives 0."""
    tot = np.float32(0)
    for x in C:
        tot = np.float32(tot + np.float32(x))
    a_t = np.float32(0) if tot == 0 else np.float32(np.float32(1) - np.float32(np.float32(max(C)) / tot))
    so = int(sum(int(x) for x in O))
    a_m = np.float32(0) if so == 0 else np.float32(1.0 - float(max(int(x) for x in O)) / float(so))
    return a_t, a_m


def partition_adjust(p, C):
    """PP_Partition_Adjust: take the boundary layer of the slowest stage to an
    adjacent stage.  READING: the slowest stage is the lowest-index maximum of
    C; of its (one or two) neighbours the one with the smaller time takes the
    layer, the earlier one on a tie; a stage of one layer gives nothing away.
    Returns (p', i_max, j) or (None, i_max, -1)."""
    P = len(p)
    i = int(np.argmax(C))                 # first maximum
    cand = [j for j in (i - 1, i + 1) if 0 <= j < P]
    if not cand or p[i] < 2:
        return None, i, -1
    j = min(cand, key=lambda k: (C[k], k))
    q = list(p)
    q[i] -= 1
    q[j] += 1
    return q, i, j


def validate(model, q, strat, Cmax, E, O_t):
    """Validate: with every layer keeping the strategy the search of p gave it,
    each stage of p' must (1) take no longer than the previous maximum stage
    time, (2) fit the budget and (3) not exceed the largest stage memory of the
    time-balanced partition."""
    for k, (a, n) in enumerate(zip(starts(q), q)):
        Ck, _, Ok = stage_under_plan(model, k, a, n, strat)
        if not (Ck <= Cmax and Ok <= E and Ok <= O_t):
            return False
    return True


def partition_search(model, p0, E, m, p_t=None, max_iter=64):
    """Algorithm 2's while-loop for one (batch size, PP degree).

    READINGS: p_t, when given, is searched once first and the largest stage
    memory of its plan is limit 3 (no limit 3 if p_t is infeasible or absent);
    a partition whose search is infeasible ends the loop; a partition already
    searched is not searched again; at most max_iter partitions are searched.
    The listing's value for this pair is the cost of the last trace entry.

    Returns dict(O_t, trace=[dict(p, cost, C, Cns, O, alpha_t, alpha_m)], strat)
    with strat the per-layer strategies of the last searched partition."""
    O_t = INT_MAX
    if p_t is not None:
        cost, _, _, O, _ = galvatron_search(model, list(p_t), E, m)
        if not np.isinf(cost):
            O_t = int(max(O))
    Q = [list(int(x) for x in p0)]
    seen = [list(Q[0])]
    trace = []
    strat = None
    while Q and len(trace) < max_iter:
        p = Q.pop()
        cost, C, Cns, O, strat = galvatron_search(model, p, E, m)
        feasible = not np.isinf(cost)
        a_t, a_m = balance_degrees(C, O) if feasible else (np.float32(0), np.float32(0))
        trace.append(dict(p=list(p), cost=cost, C=C, Cns=Cns, O=O, alpha_t=a_t, alpha_m=a_m))
        if not feasible:
            break
        q, i, j = partition_adjust(p, C)
        if q is None or q in seen:
            break
        if validate(model, q, strat, C[i], E, O_t):
            Q.append(q)
            seen.append(q)
    return dict(O_t=O_t, trace=trace, strat=strat)


def throughput(batch_sizes, costs_per_batch):
    """Outer loops of Algorithm 1/2: for batch sizes in the given order, the
    best pipeline time over the PP degrees; stop at the first batch size where
    none is feasible.  Returns (Tpt fp32, index of the batch size that gave it
    or -1).  batch / cost is an fp32 division."""
    tpt, arg = np.float32(0), -1
    for k, (B, costs) in enumerate(zip(batch_sizes, costs_per_batch)):
        c_opt = np.float32(min(np.float32(x) for x in costs))
        if np.isinf(c_opt):
            break
        t = np.float32(np.float32(B) / c_opt)
        if t > tpt:
            tpt, arg = t, k
    return tpt, arg
