"""GPU library vs CPU oracle, bit for bit, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

import gbmw_inputs as gi
import oracle
import pins
from gpu_util import check_instance, check_plans_by_definition, solve_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2307_02031_amd as g
    return g


def _log(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("launches", ["single-launch", "single-launch-cooperative", "layer-launches"])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_single_configs_full_tables(g, k, launches):
    """cfg1-3 through both ways of filling a small problem: the single launch in which the tiles
    hand their layers to each other (default), and one launch per layer."""
    p = gi.make_config(k)
    _log(f"config {k}: {p.name} {launches}")
    extra = {"single-launch": 0, "single-launch-cooperative": g.GBMW_FLAG_COOPERATIVE_LAUNCH,
             "layer-launches": g.GBMW_FLAG_LAYER_LAUNCHES}[launches]
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_KEEP_ALL_C | extra)
    q = None if k > 1 else list(range(p.E + 1))
    check_instance(g, ctx, p, 0, full_C=True, q_es=q)
    g.gbmw_destroy(ctx)


def test_config1_against_brute_force(g):
    """The GPU's best[e] against the enumeration of all 4^4 plans directly."""
    p = gi.make_config(1)
    ctx = solve_gpu(p)
    best, _ = g.gbmw_get_best(ctx)
    opt, argopt = pins.py_bruteforce(p.c, p.M, p.R, p.E)
    pins.assert_same_f32(best[0], opt)
    plan, cost, mem = g.gbmw_backtrack(ctx, np.zeros(p.E + 1, np.int32), np.arange(p.E + 1, dtype=np.int32))
    for e in range(p.E + 1):
        if np.isfinite(opt[e]):
            assert tuple(int(x) for x in plan[e]) in argopt[e]


SHAPES = [  # (S, E, list of L): ragged tails, tile boundaries, every kernel variant
    (1, 300, [1, 5, 3]),
    (2, 0, [3, 1]),
    (3, 1, [2, 4]),
    (4, 63, [4, 2, 6]),
    (5, 64, [3]),
    (7, 255, [5, 2]),
    (8, 256, [2, 7]),
    (13, 257, [4]),
    (10, 520, [3, 5]),       # S = 10 .. 58: the remaining register-blocked instantiations
    (18, 777, [4, 2]),
    (22, 1000, [6, 3, 9]),
    (24, 1023, [3]),
    (31, 2049, [4, 2]),
    (27, 640, [3, 4]),
    (35, 900, [2, 5]),
    (38, 511, [4, 3]),
    (44, 3000, [5, 8, 2]),
    (45, 700, [3, 3]),
    (50, 650, [3, 4]),
    (55, 1025, [2, 4]),
    (58, 800, [4, 2]),
    (64, 1500, [4, 6]),
    (65, 500, [3, 2]),       # 65..128: register-blocked in larger workgroups (8 or 12 waves)
    (100, 300, [3]),
    (97, 1700, [3, 2]),
    (128, 2000, [2, 4]),
    (129, 300, [3]),         # above 128: LDS-staged generic kernel
    (256, 130, [2, 3]),
]


@pytest.mark.parametrize("S,E,Ls", SHAPES, ids=[f"S{s}-E{e}" for s, e, _ in SHAPES])
@pytest.mark.parametrize("device_inputs,lazy,extra", [(False, False, 0), (True, False, 0), (True, True, 0),
                                                      (True, False, 128), (True, True, 128), (True, False, "roll")],
                         ids=["host", "device", "device-lazy-argmin", "device-layer-launches",
                              "device-lazy-argmin-layer-launches", "device-rolling-tables"])
def test_ragged_batches_all_shapes(g, S, E, Ls, device_inputs, lazy, extra):
    """Small batches: by default one launch for the whole fill (S <= 64), with
    GBMW_FLAG_LAYER_LAUNCHES (128) one launch per layer; with all tables kept and (rolling) with
    the rolling pair, where a tile also has to wait for the readers of the table it overwrites."""
    _log(f"S={S} E={E} L={Ls} device_inputs={device_inputs} lazy={lazy} extra={extra}")
    if extra == "roll":
        Mhi = max(2, E // 3 + 1)
        parts = [gi.random_instance(1000 + 17 * S + i, L + 3, S, E, M_rng=(0 if E == 0 else 1, Mhi),
                                    R_rng=(0.0, 4.0)) for i, L in enumerate(Ls)]
        p = gi.stack(parts, f"S{S}E{E}roll")
        ctx = solve_gpu(p, flags=0, device_inputs=True)
        for b in range(p.B):
            check_instance(g, ctx, p, b, full_C=False, q_es=list(range(0, E + 1, max(1, E // 40))) + [E])
        g.gbmw_destroy(ctx)
        return
    Mhi = max(2, E // 3 + 1)
    parts = [gi.random_instance(1000 + 17 * S + i, L, S, E, M_rng=(0 if E == 0 else 1, Mhi),
                                R_rng=(0.0, 4.0)) for i, L in enumerate(Ls)]
    p = gi.stack(parts, f"S{S}E{E}")
    ctx = solve_gpu(p, flags=(g.GBMW_FLAG_LAZY_ARGMIN if lazy else g.GBMW_FLAG_KEEP_ALL_C) | int(extra),
                    device_inputs=device_inputs)
    for b in range(p.B):
        check_instance(g, ctx, p, b, full_C=True, q_es=list(range(0, E + 1, max(1, E // 40))) + [E])
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("lazy", [False, True], ids=["records", "lazy-argmin"])
@pytest.mark.parametrize("S", [3, 7, 11, 15, 19, 23, 26, 30, 34, 39, 43, 47, 51, 54, 59, 62])
def test_wide_launches_every_instantiation(g, S, lazy):
    """Launches of 640 workgroups and more take the kernel's other path (each wave owns
    its own 64 budgets instead of sharing a tile with the other waves of its workgroup):
    ten instances of E = 32805 for every register-blocked instantiation, with
    integer-valued costs so that ties are everywhere."""
    E = 32805
    _log(f"wide S={S}")
    st = gi.Stream(6000 + S)
    parts = []
    for i, L in enumerate([3, 3, 3, 3, 3, 3, 3, 3, 3, 2]):
        c = st.integers(L * S, 1, 4).astype(np.float32).reshape(L, S)
        M = st.integers(L * S, 0, E // 2).reshape(L, S)
        R = st.integers(L * S * S, 0, 2).astype(np.float32).reshape(L, S, S)
        parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
    p = gi.stack(parts, f"wide-S{S}")
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_LAZY_ARGMIN if lazy else 0, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in (0, 4, 9):
        check_instance(g, ctx, p, b, full_C=False, q_es=[0, 1, E // 2, E - 1, E], best=best, best_s=best_s)
    for b in range(p.B):
        ref = oracle.solve_problem(p, b, keep_C=False, keep_A=False, nthreads=16)
        pins.assert_same_f32(best[b], ref.best, f"wide-S{S}[{b}] best")
        assert np.array_equal(best_s[b], ref.best_s)
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("lazy", [False, True], ids=["records", "lazy-argmin"])
@pytest.mark.parametrize("S", [65, 68, 83, 96, 97, 113, 128])
def test_wide_launches_above_64_strategies(g, S, lazy):
    """65 to 128 strategies in launches of at least 1024 waves take the register-blocked kernel in
    workgroups of eight or twelve waves (smaller launches and larger S the generic one): seven
    instances of 2 or 3 layers, a ragged last workgroup, integer costs (ties everywhere), every
    table cell of three instances and the best rows of all against the oracle."""
    E = 12000 + S
    _log(f"wide S={S} lazy={lazy}")
    st = gi.Stream(6500 + S)
    parts = []
    for i, L in enumerate([3, 3, 3, 3, 3, 3, 2]):
        c = st.integers(L * S, 1, 4).astype(np.float32).reshape(L, S)
        M = st.integers(L * S, 0, E // 2).reshape(L, S)
        R = st.integers(L * S * S, 0, 2).astype(np.float32).reshape(L, S, S)
        parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
    p = gi.stack(parts, f"wide-S{S}")
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_LAZY_ARGMIN if lazy else g.GBMW_FLAG_KEEP_ALL_C, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in (0, 3, 6):
        check_instance(g, ctx, p, b, full_C=True, q_es=[0, 1, E // 2, E - 1, E], best=best, best_s=best_s)
    for b in range(p.B):
        ref = oracle.solve_problem(p, b, keep_C=False, keep_A=False, nthreads=16)
        pins.assert_same_f32(best[b], ref.best, f"wide-S{S}[{b}] best")
        assert np.array_equal(best_s[b], ref.best_s)
    g.gbmw_destroy(ctx)


def test_rolling_tables_keep_the_last_two_layers(g):
    p = gi.stack([gi.random_instance(50 + i, L, 6, 400, M_rng=(1, 90)) for i, L in enumerate([5, 2, 8, 1])], "roll")
    ctx = solve_gpu(p, flags=0)
    for b in range(p.B):
        check_instance(g, ctx, p, b, full_C=False)
    with pytest.raises(g.GbmwError) as ei:
        g.gbmw_export_tables(ctx, 2, 0, 8)
    assert ei.value.status == g.GBMW_ERR_UNSUPPORTED
    g.gbmw_destroy(ctx)


def test_degenerate_inputs(g):
    cases = []
    # budget below every first-layer memory: everything infeasible
    cases.append(gi.random_instance(304, 3, 3, 4, M_rng=(5, 9)))
    # zero memory everywhere: e = 0 is feasible
    cases.append(gi.random_instance(305, 3, 2, 7, M_rng=(0, 0)))
    # memories larger than E and mixed
    p = gi.random_instance(306, 4, 5, 100, M_rng=(1, 40))
    p.M[1, 2] = 1000; p.M[2, :] = [0, 101, 100, 50, 2**31 - 1]
    cases.append(p)
    # +inf costs (forbidden strategy / transition)
    p = gi.random_instance(307, 4, 3, 60, M_rng=(1, 12))
    p.c[1, 2] = np.inf; p.R[2, 0, 1] = np.inf; p.R[3, :, 0] = np.inf
    cases.append(p)
    # duplicated columns: every minimum ties, lowest index must win
    q = gi.random_instance(308, 5, 4, 200, M_rng=(1, 30))
    cases.append(gi.Problem(1, 12, 200, q.L, np.tile(q.c, (1, 3)), np.tile(q.M, (1, 3)),
                            np.tile(q.R, (1, 3, 3)), "dup"))
    # all-equal costs and zero R: massive ties
    q = gi.random_instance(309, 6, 9, 150, M_rng=(1, 20))
    q.c[:] = 1.0; q.R[:] = 0.0
    cases.append(q)
    # subnormal and huge magnitudes
    q = gi.random_instance(310, 5, 6, 120, M_rng=(1, 20))
    q.c[:] = (q.c * np.float32(1e-42)).astype(np.float32)
    q.R[:] = (q.R * np.float32(3e-43)).astype(np.float32)
    assert (q.c > 0).all() and q.c.max() < 1.2e-38
    cases.append(q)
    q = gi.random_instance(311, 5, 6, 120, M_rng=(1, 20), c_rng=(1e37, 3e38), R_rng=(0.0, 3e38))
    cases.append(q)
    for p in cases:
        _log(f"degenerate case {p.name}")
        ctx = solve_gpu(p, flags=g.GBMW_FLAG_KEEP_ALL_C)
        ref = check_instance(g, ctx, p, 0, full_C=True, q_es=list(range(p.E + 1)))
        assert not np.isnan(ref.C).any()
        g.gbmw_destroy(ctx)


def test_context_reuse_and_errors(g):
    import torch
    a = gi.stack([gi.random_instance(70 + i, L, 10, 900, M_rng=(1, 200)) for i, L in enumerate([4, 6])], "a")
    b = gi.stack([gi.random_instance(80 + i, L, 7, 300, M_rng=(1, 50)) for i, L in enumerate([3, 2, 5])], "b")
    ctx = solve_gpu(a, flags=g.GBMW_FLAG_KEEP_ALL_C)
    check_instance(g, ctx, a, 1, full_C=True)
    ctx = solve_gpu(b, flags=g.GBMW_FLAG_KEEP_ALL_C | g.GBMW_FLAG_TIME_KERNELS, ctx=ctx)   # smaller: same buffers
    for i in range(3):
        check_instance(g, ctx, b, i, full_C=True)
    total, mp, n = g.gbmw_last_solve_ms(ctx)
    assert total > 0 and mp > 0 and n == 4 and mp <= total * 1.05
    ctx = solve_gpu(a, flags=0, ctx=ctx)                                 # larger again
    check_instance(g, ctx, a, 0, full_C=False)
    # bad queries
    with pytest.raises(g.GbmwError):
        g.gbmw_backtrack(ctx, [2], [10])
    with pytest.raises(g.GbmwError):
        g.gbmw_backtrack(ctx, [0], [901])
    plan, cost, mem = g.gbmw_backtrack(ctx, np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert plan.shape == (0, 6)
    # device-resident inputs with a bad value: reported at synchronize
    c = torch.from_numpy(b.c).cuda(); M = torch.from_numpy(b.M).cuda(); R = torch.from_numpy(b.R).cuda()
    M[1, 1] = -5
    ctx2 = g.gbmw_dp_solve_batched(b.L, c, M, R, b.S, b.E)
    with pytest.raises(g.GbmwError) as ei:
        g.gbmw_synchronize(ctx2)
    assert ei.value.status == g.GBMW_ERR_INVALID_ARG and "M" in str(ei.value)
    M[1, 1] = 5; R[3, 1, 2] = float("nan")        # row 3 = instance 1, layer 0: ignored slab
    ctx2 = g.gbmw_dp_solve_batched(b.L, c, M, R, b.S, b.E, ctx=ctx2)
    g.gbmw_synchronize(ctx2)
    R[4, 1, 2] = float("nan")
    ctx2 = g.gbmw_dp_solve_batched(b.L, c, M, R, b.S, b.E, ctx=ctx2)
    with pytest.raises(g.GbmwError):
        g.gbmw_get_best(ctx2)
    g.gbmw_destroy(ctx2)
    g.gbmw_destroy(ctx)


def test_non_default_stream(g):
    import torch
    p = gi.random_instance(90, 6, 22, 2000, M_rng=(1, 300))
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ctx = solve_gpu(p, flags=g.GBMW_FLAG_KEEP_ALL_C, device_inputs=True)
    check_instance(g, ctx, p, 0, full_C=True)
    g.gbmw_destroy(ctx)


def test_device_inputs_may_be_overwritten_after_the_solve(g):
    """The caller's device arrays are read by the solve's own enqueued work only: once a
    waiting call has returned they are overwritten with garbage here, and the walkers, the
    export (which rebuilds cells from M under the run shortcut), Algorithm 3's loop and the
    pipeline cost still give the oracle's results, with and without records."""
    import torch
    for flags in (0, g.GBMW_FLAG_LAZY_ARGMIN):
        # 700 row tiles x 2 instances: unsplit launches with the run shortcut; integer costs and
        # coarse memories, so that most cells are left to their summary words
        E, S = 700 * 256 - 13, 6
        st = gi.Stream(9100)
        parts = []
        for L in (4, 3):
            c = st.integers(L * S, 1, 6).astype(np.float32).reshape(L, S)
            M = (st.integers(L * S, 1, 50) * 640).reshape(L, S)
            R = st.integers(L * S * S, 0, 3).astype(np.float32).reshape(L, S, S)
            parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
        p = gi.stack(parts, "overwrite")
        c = torch.from_numpy(p.c).cuda(); M = torch.from_numpy(p.M).cuda(); R = torch.from_numpy(p.R).cuda()
        ctx = g.gbmw_dp_solve_batched(p.L, c, M, R, p.S, p.E, flags=flags)
        g.gbmw_synchronize(ctx)
        c.fill_(float("nan")); M.fill_(-7); R.fill_(float("nan"))
        torch.cuda.synchronize()
        for b in range(p.B):
            check_instance(g, ctx, p, b, full_C=False, q_es=[0, 640, E // 2, E - 1, E])
        Of, Ob, Oms = gi.split_memory(p, 4)
        e_opt, cost, plan, e_all = g.gbmw_select_forward_budget(ctx, Of, Ob, Oms)
        for b in range(p.B):
            o, Lb = int(p.offsets[b]), int(p.L[b])
            ref = oracle.solve_problem(p, b, keep_C=False, keep_A=True, nthreads=8)
            r = oracle.select_budget(ref, Of[o:o + Lb], Ob[o:o + Lb], Oms[o:o + Lb])
            assert int(e_opt[b]) == r[0] and pins.bits(cost[b]) == pins.bits(r[1]) and int(e_all[b]) == r[3]
            if r[0] >= 0 and np.isfinite(r[1]):
                assert np.array_equal(plan[b, :Lb], r[2])
        g.gbmw_destroy(ctx)


def test_work_counters_match_the_tables(g):
    """GBMW_FLAG_COUNT_WORK: the number of (wave, strategy) rows that the launches report as
    computed cell by cell is what the oracle's tables imply: a wave of 64 budgets escapes the
    dense arithmetic exactly when the 64 columns of the previous layer's table that it reads are
    the same bits (the kernel finds such waves from its summaries or, failing that, from the
    loaded values), and the counted solve returns the same tables as the plain one."""
    S, E = 9, 700 * 256 - 141
    st = gi.Stream(9300)
    parts = []
    for i, L in enumerate([4, 3, 2]):
        c = st.integers(L * S, 1, 6).astype(np.float32).reshape(L, S)
        M = (st.integers(L * S, 0, 60) * (97 if i else 64)).reshape(L, S)
        R = st.integers(L * S * S, 0, 3).astype(np.float32).reshape(L, S, S)
        parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
    p = gi.stack(parts, "counters")
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_COUNT_WORK | g.GBMW_FLAG_KEEP_ALL_C, device_inputs=True)
    wide, u1, u2, dense_rows = g.gbmw_last_solve_work(ctx)
    waves = uniform = 0
    nw = (E + 64) // 64
    for b in range(p.B):
        ref = check_instance(g, ctx, p, b, full_C=True, q_es=[0, E // 2, E])
        for l in range(1, int(p.L[b])):
            prev = ref.C[l - 1].view(np.uint32)                       # [E+1][S]
            pad = np.concatenate([prev, np.repeat(prev[-1:], nw * 64 - (E + 1), axis=0)])
            tiles = pad.reshape(nw, 64, S)
            uniform += int(np.all(tiles == tiles[:, :1, :], axis=(1, 2)).sum())
            waves += nw
    assert dense_rows == (waves - uniform) * S, (wide, u1, u2, dense_rows, waves, uniform)
    assert wide > 0 and u1 > 0 and dense_rows > 0
    # a solve with dense arithmetic computes every row
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_COUNT_WORK | g.GBMW_FLAG_DENSE_ARITHMETIC, device_inputs=True, ctx=ctx)
    assert g.gbmw_last_solve_work(ctx) == (0, 0, 0, waves * S)
    # and without the flag nothing is counted
    ctx = solve_gpu(p, flags=0, device_inputs=True, ctx=ctx)
    assert g.gbmw_last_solve_work(ctx) == (0, 0, 0, 0)
    g.gbmw_destroy(ctx)


def test_single_launch_wait_gives_up_cleanly(g):
    """The single-launch fill's waits are bounded.  With GBMW_FLAG_TEST_WAIT_GIVES_UP they ask for a
    layer that no tile ever publishes and give up after a millisecond: every workgroup ends, the
    solve's waiting calls report GBMW_ERR_DEVICE, and the same context solves correctly afterwards."""
    import torch
    p = gi.stack([gi.random_instance(5100 + i, L, 12, 3000, M_rng=(1, 500)) for i, L in enumerate([5, 3])], "give-up")
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_KEEP_ALL_C, device_inputs=True)
    check_instance(g, ctx, p, 0, full_C=True)
    c = torch.from_numpy(p.c).cuda(); M = torch.from_numpy(p.M).cuda(); R = torch.from_numpy(p.R).cuda()
    ctx = g.gbmw_dp_solve_batched(p.L, c, M, R, p.S, p.E, flags=g.GBMW_FLAG_KEEP_ALL_C | g.GBMW_FLAG_TEST_WAIT_GIVES_UP, ctx=ctx)
    for call in (lambda: g.gbmw_synchronize(ctx), lambda: g.gbmw_get_best(ctx), lambda: g.gbmw_backtrack(ctx, [0], [p.E])):
        with pytest.raises(g.GbmwError) as ei:
            call()
        assert ei.value.status == g.GBMW_ERR_DEVICE and "gave up" in str(ei.value)
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_KEEP_ALL_C, device_inputs=True, ctx=ctx)
    for b in range(p.B):
        check_instance(g, ctx, p, b, full_C=True)
    # a problem too large for the single launch refuses the test flag instead of ignoring it
    big = gi.random_instance(5200, 2, 4, 400000, M_rng=(1, 9))
    with pytest.raises(g.GbmwError) as ei:
        g.gbmw_dp_solve_batched(big.L, big.c, big.M, big.R, big.S, big.E, flags=g.GBMW_FLAG_TEST_WAIT_GIVES_UP)
    assert ei.value.status == g.GBMW_ERR_INVALID_ARG
    g.gbmw_destroy(ctx)


def test_single_launch_with_a_rolling_pair_of_tables(g):
    """The single launch keeps every layer's table only up to 1 GiB of them; beyond, it works on a
    rolling pair and a tile also waits for the tiles above it, whose input it is about to
    overwrite.  136 layers of 64 strategies over 512 tiles (1.06 GiB of tables): records, last
    tables, best and plans against the oracle."""
    E = 512 * 64 - 1
    p = gi.random_instance(5300, 136, 64, E, M_rng=(1, 480), R_rng=(0.0, 4.0))
    ctx = solve_gpu(p, flags=0, device_inputs=True)
    check_instance(g, ctx, p, 0, full_C=False, q_es=[0, 1000, E // 4, E // 2, E - 1, E])
    with pytest.raises(g.GbmwError):
        g.gbmw_export_tables(ctx, 0, 0, 5)
    g.gbmw_destroy(ctx)


MODES = {"records": 0, "lazy-argmin": 16, "records-dense": 32, "lazy-argmin-dense": 48}


@pytest.mark.parametrize("mode", list(MODES), ids=list(MODES))
@pytest.mark.parametrize("S", [5, 44, 61])
def test_runs_of_equal_columns_edge_cases(g, S, mode):
    """By default a wave whose 64 budgets read the same column of the previous table computes
    it once.  Layer-0 memories are placed so that the columns change exactly at, just before
    and just after the wave boundaries (budgets 63, 64, 65, 127, 128, ...), at budget 0, at E
    and beyond E, in unsplit launches (>= 640 workgroups) whose last wave is cut by E; later
    layers shift by multiples of 64 and by odd amounts.  Full tables against the oracle, with
    and without the shortcut, with and without records."""
    E = 26453                                       # E + 1 = 103 * 256 + 86: a ragged last wave
    flags = MODES[mode]
    edges = [0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 4095, 4096, 4097, E - 64, E - 63, E - 1, E, E + 1]
    st = gi.Stream(7700 + S)
    parts = []
    for i in range(12):
        L = 3 if i < 10 else 2
        c = st.integers(L * S, 1, 6).astype(np.float32).reshape(L, S)
        R = st.integers(L * S * S, 0, 3).astype(np.float32).reshape(L, S, S)
        M = np.zeros((L, S), np.int64)
        M[0] = [edges[(i + 3 * s) % len(edges)] for s in range(S)]
        if i % 2:                                   # shifts that keep the alignment / that break it
            M[1:] = 64 * st.integers((L - 1) * S, 0, 40).reshape(L - 1, S)
        else:
            M[1:] = st.integers((L - 1) * S, 0, 3000).reshape(L - 1, S)
        if i == 3:
            c[0, ::2] = np.inf                      # forbidden strategies: columns of +inf
        if i == 4:
            M[0] = E + 1                            # nothing fits: every column is +inf everywhere
        parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
    p = gi.stack(parts, f"runs-S{S}")
    keep = 0 if flags & 16 else g.GBMW_FLAG_KEEP_ALL_C
    # one stream: every layer's launch then covers all instances (1248 and 1040 workgroups)
    ctx = solve_gpu(p, flags=flags | keep | g.GBMW_FLAG_ONE_STREAM, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in range(p.B):
        _log(f"runs S={S} {mode} instance {b}")
        check_instance(g, ctx, p, b, full_C=True, q_es=[0, 63, 64, 4096, E - 1, E], best=best, best_s=best_s)
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("mode", list(MODES), ids=list(MODES))
@pytest.mark.parametrize("E", [0, 5, 100, 300, 767])
def test_many_small_instances_in_one_launch(g, E, mode):
    """Hundreds of instances with one to three workgroups each: a launch large enough for the
    unsplit shape whose workgroups are mostly cut by the end of the table (waves entirely
    beyond E, a ragged last wave, E + 1 a multiple of 256 for E = 767).  Integer costs, so runs
    of equal columns and ties are everywhere.  Every 37th instance cell by cell, best rows of all."""
    flags = MODES[mode]
    B, S = 700, 7
    st = gi.Stream(8800 + E)
    parts = []
    for i in range(B):
        L = 2 + i % 3
        c = st.integers(L * S, 1, 5).astype(np.float32).reshape(L, S)
        M = st.integers(L * S, 0, max(1, E // 3)).reshape(L, S)
        R = st.integers(L * S * S, 0, 2).astype(np.float32).reshape(L, S, S)
        parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
    p = gi.stack(parts, f"small-E{E}")
    keep = 0 if flags & 16 else g.GBMW_FLAG_KEEP_ALL_C
    ctx = solve_gpu(p, flags=flags | keep | g.GBMW_FLAG_ONE_STREAM, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in range(0, B, 37):
        check_instance(g, ctx, p, b, full_C=True, q_es=[0, E // 2, E], best=best, best_s=best_s, nthreads=2)
    for b in range(B):
        ref = oracle.solve_problem(p, b, keep_C=False, keep_A=False, nthreads=1)
        pins.assert_same_f32(best[b], ref.best, f"small-E{E}[{b}] best")
        assert np.array_equal(best_s[b], ref.best_s)
    g.gbmw_destroy(ctx)


@pytest.mark.parametrize("mode", list(MODES), ids=list(MODES))
@pytest.mark.parametrize("streams", ["one-stream", "two-groups"])
def test_launch_shapes_follow_one_another(g, mode, streams):
    """Six instances of 2..7 layers over 120 row tiles: the layer launches shrink from the unsplit
    shape (6 x 120 workgroups) to the split one, so that a split launch reads tables that an
    unsplit launch with the run shortcut left (cells of uniform groups unwritten, the summary
    words standing for them), later split launches read tables that split launches wrote, and
    the final reduce, the export and the walkers read both kinds.  Two kinds of inputs: integer
    costs with coarse memory (long runs, ties) and random ones (few runs).  Every cell of every
    layer against the oracle."""
    flags = MODES[mode] | (g.GBMW_FLAG_ONE_STREAM if streams == "one-stream" else 0)
    S, E = 9, 120 * 256 - 77
    for kind in (0, 1):
        st = gi.Stream(4100 + kind)
        parts = []
        for i, L in enumerate([7, 2, 5, 3, 6, 4]):
            if kind == 0:
                c = st.integers(L * S, 1, 6).astype(np.float32).reshape(L, S)
                M = (st.integers(L * S, 0, 40) * 97).reshape(L, S)
                R = st.integers(L * S * S, 0, 3).astype(np.float32).reshape(L, S, S)
                parts.append(gi.Problem(1, S, E, np.array([L]), c, M, R))
            else:
                parts.append(gi.random_instance(4200 + i, L, S, E, M_rng=(0, 5000)))
        p = gi.stack(parts, f"shapes-{kind}")
        keep = 0 if flags & 16 else g.GBMW_FLAG_KEEP_ALL_C
        ctx = solve_gpu(p, flags=flags | keep, device_inputs=bool(kind))
        best, best_s = g.gbmw_get_best(ctx)
        for b in range(p.B):
            check_instance(g, ctx, p, b, full_C=True, q_es=[0, 1, E // 3, E - 1, E], best=best, best_s=best_s,
                           nthreads=4)
        g.gbmw_destroy(ctx)


@pytest.mark.parametrize("lazy", [False, True], ids=["records", "lazy-argmin"])
def test_config4_dense_arithmetic(g, lazy):
    """The benchmark's batch with GBMW_FLAG_DENSE_ARITHMETIC (every lane computes its own
    cell): every ninth instance against the oracle."""
    p = gi.make_config(4)
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_DENSE_ARITHMETIC | (g.GBMW_FLAG_LAZY_ARGMIN if lazy else 0),
                    device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in range(0, p.B, 9):
        _log(f"cfg4 dense instance {b} L={p.L[b]}")
        check_instance(g, ctx, p, b, full_C=False, best=best, best_s=best_s)
    g.gbmw_destroy(ctx)


def test_config4_batched_full_size(g):
    """All 64 instances in the launch configuration the benchmark times; full A,
    last two layers of C, best, plans against the oracle for every instance."""
    p = gi.make_config(4)
    ctx = solve_gpu(p, flags=0, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in range(p.B):
        _log(f"cfg4 instance {b} L={p.L[b]}")
        check_instance(g, ctx, p, b, full_C=False, best=best, best_s=best_s)
    g.gbmw_destroy(ctx)


def test_config4_lazy_argmin_full_size(g):
    """The same batch without argmin records: tables, recomputed records, best and plans
    of every seventh instance against the oracle, plan properties for all."""
    p = gi.make_config(4)
    ctx = solve_gpu(p, flags=g.GBMW_FLAG_LAZY_ARGMIN, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    for b in range(0, p.B, 7):
        _log(f"cfg4 lazy instance {b} L={p.L[b]}")
        check_instance(g, ctx, p, b, full_C=False, best=best, best_s=best_s)
    q = sorted(set(list(range(0, p.E + 1, 1013)) + [p.E, p.E - 1]))
    for b in range(p.B):
        check_plans_by_definition(g, ctx, p, b, q, best)
    g.gbmw_destroy(ctx)


def test_config5_large_batched_full_size(g):
    """B=16, L=96, S=64, E=65536 in one solve, in the launch configuration the benchmark
    times.  Every one of the sixteen instances against the oracle: best, best_s, every
    argmin record of every layer and the plans of a list of budgets; two of them also cell by
    cell on the last layers of C (the oracle then holds all its fp32 tables, 1.6 GB); and
    the plans of all sixteen re-evaluated by the plain definition of a plan's cost."""
    p = gi.make_config(5)
    ctx = solve_gpu(p, flags=0, device_inputs=True)
    best, best_s = g.gbmw_get_best(ctx)
    q = sorted(set(list(range(0, p.E + 1, 997)) + [p.E, p.E - 1, 12288, 12287]))
    for b in range(p.B):
        _log(f"cfg5 instance {b}: oracle comparison")
        check_instance(g, ctx, p, b, full_C=False, q_es=q, best=best, best_s=best_s, with_C=b in (0, 11))
        check_plans_by_definition(g, ctx, p, b, q, best)
    g.gbmw_destroy(ctx)


def test_config5_all_modes_agree(g):
    """cfg5 under the four combinations of records / values only and run shortcut / dense
    arithmetic: best rows, their argmins, the last layer's table and the records of two
    layers of one instance are the same bytes (the default mode is checked against the
    oracle above)."""
    p = gi.make_config(5)
    ref = None
    for mode, flags in MODES.items():
        _log(f"cfg5 {mode}")
        ctx = solve_gpu(p, flags=flags, device_inputs=True)
        best, best_s = g.gbmw_get_best(ctx)
        Lb = int(p.L[3])
        C, _ = g.gbmw_export_tables(ctx, 3, Lb - 1, Lb, want_C=True, want_A=False)
        _, A = g.gbmw_export_tables(ctx, 3, Lb - 2, Lb, want_C=False, want_A=True)
        got = (best.copy(), best_s.copy(), C.copy(), A.copy())
        g.gbmw_destroy(ctx)
        if ref is None:
            ref = got
        else:
            for x, y, what in zip(ref, got, ("best", "best_s", "C", "A")):
                assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), (mode, what)

